"""Sweeps of the two MDPS hyper-parameters on a synthetic workload stage: the ratio p of exact
FPS iterations run first and the number of curve segments nseg (the ablations of Appendix B.6
and of the segment count, Section 5.3, run here on the seeded generators instead of the paper's
data sets).  For every setting the power-function estimator is fitted on the calibration clouds
as calibration.py does, then mdps_sample is timed on the workload's own clouds and its coverage
radius is compared with exact FPS.  Everything runs through the HIP library.

  python -m paper_2507_23480_amd.ablation [C3]      (on a GPU machine; prints a markdown table)
"""
from __future__ import annotations

import sys
from typing import List

import numpy as np

from . import calibration

P_VALUES = [0.05, 0.1, 0.2, 0.3]
NSEG_VALUES = [2, 4, 6, 8, 12]


def _time(torch, fn, reps=5):
    fn()
    torch.cuda.synchronize()
    best = None
    for _ in range(reps):
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        t = a.elapsed_time(b)
        best = t if best is None else min(best, t)
    return best


def run(name: str, log=print) -> List[dict]:
    import torch
    from . import binding as fp, inputs
    wl = inputs.WORKLOADS[name]
    st = wl.stages[0]
    cal = torch.from_numpy(inputs.make_batch(name, B=calibration.CALIBRATION_CLOUDS[name], calibration=True)).cuda()
    x = torch.from_numpy(inputs.make_batch(name)).cuda()
    fidx = fp.fps_exact(x, st.n)
    cov_f = fp.coverage2(x, fidx).sqrt()
    t_fps = _time(torch, lambda: fp.fps_exact(x, st.n))
    rows = []
    keep = (calibration.P_RATIO, calibration.NSEG)
    try:
        for p, nseg in [(p, keep[1]) for p in P_VALUES] + [(keep[0], k) for k in NSEG_VALUES if k != keep[1]]:
            calibration.P_RATIO, calibration.NSEG = p, nseg
            ent = calibration.fit_stage(cal, st.n, log=lambda *a: None)
            prm = fp.MdpsParams(p=p, nseg=nseg, exponent=ent["exponent"], bias=ent["bias"],
                                fit_window=calibration.FIT_WINDOW, m_min=calibration.M_MIN,
                                level_scale=ent["level_scale"])
            idx, info = fp.mdps_sample(x, st.n, prm, want_info=True)
            cov = fp.coverage2(x, idx).sqrt() / cov_f
            torch.cuda.synchronize()
            infos = fp.parse_info(info)
            t = _time(torch, lambda: fp.mdps_sample(x, st.n, prm))
            rows.append({"p": p, "nseg": nseg, "exponent": ent["exponent"], "bias": ent["bias"],
                         "mdps_ms": t, "fps_ms": t_fps, "coverage_ratio_max": float(cov.max()),
                         "coverage_ratio_mean": float(cov.mean()),
                         "fps_tail_mean": float(np.mean([(st.n - i.et_index) / st.n for i in infos])),
                         "rounds_mean": float(np.mean([i.rounds for i in infos]))})
            log("p %.2f nseg %2d: mdps %.3f ms (exact FPS %.3f), coverage max %.4f, tail %.1f %%"
                % (p, nseg, t, t_fps, rows[-1]["coverage_ratio_max"], 100 * rows[-1]["fps_tail_mean"]))
    finally:
        calibration.P_RATIO, calibration.NSEG = keep
    # the two other estimators at the default p and nseg: the pure power function of Appendix A.3
    # (no per-segment factors) and the MLP of the same appendix
    from . import mlp_estimator
    # ... and, with the default estimator, the other scan order of the threshold phase and the
    # cell-ordered sampler with pruned updates (both scan orders)
    import dataclasses
    base = calibration.params_for(name, 0)
    scattered = dataclasses.replace(base, scan_order=1)
    paper = calibration.params_for(name, 0, "paper")
    for label, prm, entry in (("pure power function", paper, fp.mdps_sample),
                              ("pure power function, no bias", dataclasses.replace(paper, bias=1.0), fp.mdps_sample),
                              ("MLP", mlp_estimator.params_for(name, 0), fp.mdps_sample),
                              ("segment factors, scattered scan order", scattered, fp.mdps_sample),
                              ("segment factors, pruned updates", base, fp.mdps_sample_pruned),
                              ("segment factors, scattered scan order, pruned updates", scattered,
                               fp.mdps_sample_pruned)):
        idx, info = entry(x, st.n, prm, want_info=True)
        cov = fp.coverage2(x, idx).sqrt() / cov_f
        torch.cuda.synchronize()
        infos = fp.parse_info(info)
        t = _time(torch, lambda: entry(x, st.n, prm))
        rows.append({"p": prm.p, "nseg": prm.nseg, "exponent": prm.exponent, "bias": prm.bias, "estimator": label,
                     "mdps_ms": t, "fps_ms": t_fps, "coverage_ratio_max": float(cov.max()),
                     "coverage_ratio_mean": float(cov.mean()),
                     "fps_tail_mean": float(np.mean([(st.n - i.et_index) / st.n for i in infos])),
                     "rounds_mean": float(np.mean([i.rounds for i in infos]))})
        log("%s: mdps %.3f ms, coverage max %.4f, tail %.1f %%"
            % (label, t, rows[-1]["coverage_ratio_max"], 100 * rows[-1]["fps_tail_mean"]))
    return rows


def markdown(name: str, rows: List[dict]) -> str:
    out = ["| workload | estimator | p | nseg | exponent | bias | mdps_sample ms | fps_exact ms | coverage / FPS (max) | "
           "coverage / FPS (mean) | exact-FPS tail | rounds |", "|---|---|---|---|---|---|---|---|---|---|---|---|"]
    for r in rows:
        out.append("| %s | %s | %.2f | %d | %.3f | %.2f | %.3f | %.3f | %.4f | %.4f | %.1f %% | %.0f |"
                   % (name, r.get("estimator", "power function x segment factors"), r["p"], r["nseg"],
                      r["exponent"], r["bias"], r["mdps_ms"], r["fps_ms"],
                      r["coverage_ratio_max"], r["coverage_ratio_mean"], 100 * r["fps_tail_mean"], r["rounds_mean"]))
    return "\n".join(out)


def main(argv: List[str]) -> int:
    for name in argv or ["C3"]:
        rows = run(name)
        print(markdown(name, rows), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
