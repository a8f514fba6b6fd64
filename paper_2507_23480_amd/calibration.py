"""Offline fit of the MDPS curve-estimator constants, per workload and stage.

Appendix A.3 of the paper fits the exponent of the power-function estimator on the
minimum-distance curves of a data set's training split and finds the factor `a`
per cloud at run time.  Here the "training split" is a set of calibration clouds
drawn from the same seeded generators as the workloads, with disjoint seeds.
Everything runs through the HIP library (exact FPS yields the curves).

Per (workload, stage) the fit produces
  exponent     least squares of log(curve) against log(position) over [m, n)
  level_scale  per segment end, the geometric mean over the calibration clouds of
               (true curve value) / (power-law prediction): the part of the curve's
               shape a single exponent misses (1 where the boundary lies inside the
               measured prefix)
  bias         the smallest factor >= 1.01 (steps of 0.01) for which, on every
               calibration cloud, the last level is exhausted and the coverage
               radius stays within 1.03x of exact FPS: an under-estimated last
               threshold would leave the final level unexhausted and the coverage
               unbounded, an over-estimate only costs extra exact FPS iterations.
               BIAS_MARGIN is added on top for clouds the fit has not seen.

Two tables are kept.  mdps_calibration.json holds the fit above: the power function of the
appendix extended by the per-segment factors.  mdps_calibration_paper.json holds the estimator
exactly as the appendix defines it -- a / x^e with a from the measured prefix, level_scale = 1
everywhere -- with only the exponent and the safety factor `bias` fitted the same way.

Run  python -m paper_2507_23480_amd.calibration [--paper] [workloads]  on a GPU machine to rewrite
mdps_calibration.json (or, with --paper, mdps_calibration_paper.json) next to this file.
"""
from __future__ import annotations

import json
import math
import os
import sys
from typing import Dict, List

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
TABLE_PATH = os.path.join(HERE, "mdps_calibration.json")
PAPER_TABLE_PATH = os.path.join(HERE, "mdps_calibration_paper.json")

CALIBRATION_CLOUDS = {"C1": 8, "C2": 32, "C3": 8, "C4": 8, "C5": 3}
P_RATIO, NSEG, FIT_WINDOW, M_MIN = 0.1, 6, 32, 8
BIAS_MARGIN = 0.02

_tables = {}


def table(variant: str = "calibrated") -> Dict[str, List[dict]]:
    """The fitted constants: "calibrated" (power function with per-segment factors) or "paper"
    (the pure power function of Appendix A.3)."""
    if variant not in _tables:
        with open(TABLE_PATH if variant == "calibrated" else PAPER_TABLE_PATH) as f:
            _tables[variant] = json.load(f)
    return _tables[variant]


def params_for(workload: str, stage: int, variant: str = "calibrated"):
    """MdpsParams with the fitted constants of one workload stage."""
    from . import binding
    ent = table(variant)[workload][stage]
    return binding.MdpsParams(p=P_RATIO, nseg=NSEG, exponent=ent["exponent"], bias=ent["bias"],
                              fit_window=FIT_WINDOW, m_min=M_MIN, level_scale=ent["level_scale"])


def _boundaries(n: int) -> List[int]:
    return [min(max(n * l // NSEG, 1), n - 1) for l in range(1, NSEG + 1)]


def fit_stage(xyz, n: int, log=print, pure: bool = False) -> dict:
    """xyz: CUDA float32 [Bc][N][3] calibration clouds of one stage.  pure: no per-segment factors
    (the estimator as Appendix A.3 defines it)."""
    import torch
    from . import binding as fp
    idx, mdc = fp.fps_exact(xyz, n, want_mdc=True)
    torch.cuda.synchronize()
    curves = mdc.cpu().numpy().astype(np.float64)
    Bc, N = xyz.shape[0], xyz.shape[1]
    m = max(int(math.floor(P_RATIO * n)), M_MIN)
    if m >= n - 1:
        return {"N": N, "n": n, "exponent": 1.0, "bias": 1.0, "level_scale": [1.0] * NSEG}
    pos = np.arange(m, n, dtype=np.float64)
    es = []
    for c in curves:
        y = np.log(np.maximum(c[m:n], 1e-300))
        A = np.stack([np.log(pos), np.ones_like(pos)], axis=1)
        es.append(-np.linalg.lstsq(A, y, rcond=None)[0][0])
    e = float(np.mean(es))
    W = min(FIT_WINDOW, m)
    bl = _boundaries(n)
    ratios = np.ones((Bc, NSEG))
    for b, c in enumerate(curves):
        i = np.arange(m - W + 1, m + 1, dtype=np.float64)
        a = float(np.mean(c[m - W + 1:m + 1] * i ** e))
        for l, x in enumerate(bl):
            if x > m:
                ratios[b, l] = c[x] / (a / float(x) ** e)
    scale = np.exp(np.mean(np.log(ratios), axis=0))
    scale = [1.0] * NSEG if pure else [float(round(s, 4)) for s in scale]
    # spread of the last level decides where the bias search starts
    spread = float(np.max(np.sqrt(scale[-1] / ratios[:, -1])))
    bias = max(1.01, round(spread, 2))
    cov_fps = fp.coverage2(xyz, idx).sqrt()
    while True:
        prm = fp.MdpsParams(p=P_RATIO, nseg=NSEG, exponent=e, bias=bias, fit_window=FIT_WINDOW,
                            m_min=M_MIN, level_scale=scale)
        midx, info = fp.mdps_sample(xyz, n, prm, want_info=True)
        cov = fp.coverage2(xyz, midx).sqrt()
        torch.cuda.synchronize()
        infos = fp.parse_info(info)
        exhausted = all(i.level_exhausted[NSEG - 1] == 1 or i.et_index < n for i in infos)
        worst = float((cov / cov_fps).max())
        tail = float(np.mean([(n - i.et_index) / n for i in infos]))
        log("    bias %.2f: last level exhausted on all: %s, worst coverage ratio %.4f, mean FPS tail %.1f%%"
            % (bias, exhausted, worst, 100 * tail))
        if (exhausted and worst <= 1.03) or bias >= 1.5:
            break
        bias = round(bias + 0.01, 2)
    return {"N": int(N), "n": int(n), "exponent": round(e, 5), "bias": round(float(bias) + BIAS_MARGIN, 2),
            "bias_found": float(bias), "level_scale": scale,
            "exponent_per_cloud_min": round(float(min(es)), 4),
            "exponent_per_cloud_max": round(float(max(es)), 4),
            "calibration_tail_mean": round(tail, 4), "calibration_worst_coverage_ratio": round(worst, 4)}


def calibrate_workload(name: str, log=print, pure: bool = False) -> List[dict]:
    import torch
    from . import binding as fp, inputs
    wl = inputs.WORKLOADS[name]
    Bc = CALIBRATION_CLOUDS[name]
    xyz = torch.from_numpy(inputs.make_batch(name, B=Bc, calibration=True)).cuda()
    out = []
    for s, st in enumerate(wl.stages):
        log("%s stage %d: %d calibration clouds of %d points -> %d samples" % (name, s, Bc, xyz.shape[1], st.n))
        ent = fit_stage(xyz, st.n, log, pure)
        log("    exponent %.4f bias %.2f scale %s" % (ent["exponent"], ent["bias"], ent["level_scale"]))
        out.append(ent)
        if s + 1 < len(wl.stages):          # the next stage's input: the exact-FPS samples
            xyz = fp.gather_xyz(xyz, fp.fps_exact(xyz, st.n)).contiguous()
    return out


def main(argv: List[str]) -> int:
    pure = "--paper" in argv
    names = [a for a in argv if not a.startswith("--")] or list(CALIBRATION_CLOUDS)
    path = PAPER_TABLE_PATH if pure else TABLE_PATH
    result = {}
    if os.path.exists(path):
        with open(path) as f:
            result = json.load(f)
    out_path = os.environ.get("FASTPOINT_CALIBRATION_OUT", path)
    for name in names:
        result[name] = calibrate_workload(name, pure=pure)
        with open(out_path, "w") as f:
            json.dump(result, f, indent=1, sort_keys=True)
            f.write("\n")
    print("wrote", out_path)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
