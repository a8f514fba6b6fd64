#!/usr/bin/env python3
"""Benchmark of the FPS / MDPS / ball-query hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of the workload, for
every stage of its hierarchy:
    exact path   fps_exact -> ball_query (brute force)          (Alg. 1 + Section 3.1)
    FastPoint    mdps_sample (records the radius tests) -> ball_query (cache reader)
                                                                (Alg. 2 + Section 4.2)
    gather of the exact-FPS samples = input of the next stage (which waits for it)
Inputs are resident in HBM before the timed region.  The last line of stdout is ONE compact JSON
line (headline workload C5, the largest one; a short entry per workload C1-C5 with the time of
each of the two paths); everything else measured goes to a side file (--detail-file, default
gpurun_out/bench_detail.json).

Workloads whose clouds take one workgroup each leave most of the device idle, so their step
runs the calls that do not wait for each other on four streams and is replayed as one captured
HIP graph (no host time between the launches); the replay's outputs are compared with the eager
ones.  The per-kernel times and rooflines always come from calls that run alone on one stream.

Outside the timed step the k nearest samples of every point (the k-NN of the up-sampling
step, redundancy-free form of Section 4.2) are timed per stage and reported under "detail".

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C5] [--no-extra]
"""
import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# fp32 vector rate of MI355X without FMA: 256 CUs x 128 lanes x 2.4 GHz = 78.6 T operations/s.
# The published 157.3 TFLOP/s counts an FMA as two flops; this path may not contract (every
# operation is rounded on its own), hence half of it.  (Measured on the device: plain
# add/sub/mul on register operands reach 73 T lane-operations/s when two or more waves share a
# SIMD; min, compares, selects, cross-lane moves and operations with a scalar-register operand
# run at half that rate, so the instruction mix of this path cannot reach the figure.)
ALU_PEAK_TOPS = 256 * 128 * 2.4e9 / 1e12
HBM_PEAK_GBS = 8000.0
OPS_PER_POINT_ITERATION = 10      # 3 sub, 3 mul, 2 add, 1 min, 1 compare (FPS min-update + arg-max)
OPS_PER_PAIR_TEST = 9             # 3 sub, 3 mul, 2 add, 1 compare (ball query, k-NN)
KNN_K = 3                         # neighbours of the up-sampling step (Section 3.1)
# entries per cloud of the ball-query cache (blocks of 64 radius tests that found a point); 0 = the
# library's default of 2 N + 16 n.  The LiDAR-like clouds have balls of several thousand points.
BQ_CACHE_ENTRIES = {"C4": 10 * 120000}
EXCL_MEMBER_BUDGET = 64 << 30      # bytes of exclusion-list members the benchmark is willing to build
CPU_SAMPLE_N = 4096               # cpu_baseline on C4 / C5: samples of each sampler that are timed ...
CPU_SAMPLE_M = 4096               # ... and ball-query centres
EAGER = "one stream, eager launches"
GRAPH = "four streams, step replayed as one HIP graph"

# HBM traffic per launch (bytes fetched + written) of the kernels that can dominate the step, from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (profiles/bench_C5_hbm_traffic.md, bench_C4_hbm_traffic.md,
# bench_C2_hbm_traffic.md), keyed by workload and kernel.  None where no counter run is recorded.  The
# samplers keep the cloud in registers: what they move beyond reading it once is the polling of the
# words exchanged between the workgroups of a cloud.
TRAFFIC_BYTES = {"C2": {"fps_exact": 427967, "mdps_sample+record": 2364746, "ball_query_cached": 1948914,
                        "ball_query_brute": 2004582},
                 # (C4, C5: the step's recorder is the cell-ordered one, its reader the one for cell-ordered records)
                 "C4": {"fps_exact": 91435788, "mdps_sample+record": 235871565, "ball_query_cached": 59670967,
                        "ball_query_brute": 90643229},
                 "C5": {"fps_exact": 167284349, "mdps_sample+record": 230724683, "ball_query_cached": 29243835,
                        "ball_query_brute": 204117378}}


PRUNED_RECORD_FROM = 1 << 14


def record_sampler(fp, sg):
    return fp.mdps_sample_pruned if sg["pruned_record"] else fp.mdps_sample


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C5", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--detail-file", default=os.path.join(ROOT, "gpurun_out", "bench_detail.json"),
                    help="where everything that does not fit the one result line is written")
    ap.add_argument("--no-extra", action="store_true", help="skip the other workloads' summary")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--plain-launch", action="store_true",
                    help="plain instead of cooperative kernel launches (for rocprofv3 traces)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for rocprofv3 byte counters)")
    return ap.parse_args()


class Timer:
    """Average duration of named calls, measured with events on the stream they run on."""

    def __init__(self, torch):
        self.torch = torch
        self.pending = []
        self.acc = {}

    def call(self, name, fn):
        a = self.torch.cuda.Event(enable_timing=True)
        b = self.torch.cuda.Event(enable_timing=True)
        a.record()
        out = fn()
        b.record()
        self.pending.append((name, a, b))
        return out

    def collect(self):
        for name, a, b in self.pending:
            self.acc.setdefault(name, []).append(a.elapsed_time(b))
        self.pending = []

    def reset(self):
        self.pending, self.acc = [], {}

    def mean_ms(self):
        return {k: sum(v) / len(v) for k, v in self.acc.items()}

    def min_median_ms(self):
        return {k: (min(v), sorted(v)[len(v) // 2]) for k, v in self.acc.items()}


def make_context(torch, fp, inputs, calibration, name):
    wl = inputs.WORKLOADS[name]
    xyz = torch.from_numpy(inputs.make_batch(name)).cuda()
    stages = []
    B, N = xyz.shape[0], xyz.shape[1]
    for s, st in enumerate(wl.stages):
        prm = calibration.params_for(name, s)
        pruned = N >= PRUNED_RECORD_FROM
        stages.append({"B": B, "N": N, "n": st.n, "radius": st.radius, "k": st.k,
                       "prm": prm,
                       # the step's MDPS: from 16384 points per cloud on the cell-ordered sampler with
                       # the scattered scan order of the threshold phase (the paper's step takes any
                       # available point), below that the index-ordered one with the lowest index
                       "step_prm": dataclasses.replace(prm, scan_order=1) if pruned else prm,
                       "cache": torch.empty(fp.load().fp_bq_cache_bytes(
                           B, N, st.n, BQ_CACHE_ENTRIES.get(name, 0) if s == 0 else 0), dtype=torch.uint8, device="cuda"),
                       "G": fp.plan(B, N)[0],
                       "pruned_record": pruned,
                       "ws": [fp.new_workspace(xyz.device, B, N), fp.new_workspace(xyz.device, B, N)]})
        N = st.n
    torch.cuda.synchronize()
    return {"wl": wl, "name": name, "stages": stages, "xyz": xyz, "side": torch.cuda.Stream(),
            "aux": torch.cuda.Stream(), "bqs": torch.cuda.Stream()}


def run_step(fp, ctx, timer, keep=None):
    """One step, every call on the current stream, each timed with events."""
    x = ctx["xyz"]
    for s, sg in enumerate(ctx["stages"]):
        n, r, k = sg["n"], sg["radius"], sg["k"]
        xs = x
        idx = timer.call("fps_exact/s%d" % s, lambda: fp.fps_exact(xs, n))
        bq = timer.call("ball_query_brute/s%d" % s, lambda: fp.ball_query(xs, idx, r, k))
        midx = timer.call("mdps_sample+record/s%d" % s,
                          lambda: record_sampler(fp, sg)(xs, n, sg["step_prm"], bq_cache=sg["cache"], bq_radius=r))
        mbq = timer.call("ball_query_cached/s%d" % s,
                         lambda: fp.ball_query(xs, midx, r, k, bq_cache=sg["cache"]))
        if s + 1 < len(ctx["stages"]):
            x = timer.call("gather/s%d" % s, lambda: fp.gather_xyz(xs, idx))
        if keep is not None:
            keep.append((xs, idx, bq, midx, mbq))


def run_step_streams(torch, fp, ctx, keep=None):
    """One step on four streams, for clouds that take one workgroup each (the work of all stages
    fits on the device side by side).  What has to happen in order is exact FPS of stage s ->
    gather -> the samplers of stage s+1: that chain runs on the current stream.  mdps_sample
    (with recording) and the cache reader that follows it run on a stream per stage, two in
    turn, as soon as the stage's input is there; the brute-force ball queries, which nothing
    waits for, on a stream of their own."""
    main = torch.cuda.current_stream()
    lanes = [ctx["side"], ctx["aux"]]
    bqs = ctx["bqs"]
    x = ctx["xyz"]
    for s, sg in enumerate(ctx["stages"]):
        n, r, k = sg["n"], sg["radius"], sg["k"]
        lane = lanes[s % 2]
        lane.wait_stream(main)                      # the stage's input is ready
        with torch.cuda.stream(lane):
            midx = fp.mdps_sample(x, n, sg["prm"], bq_cache=sg["cache"], bq_radius=r, ws=sg["ws"][1])   # (small clouds)
            mbq = fp.ball_query(x, midx, r, k, bq_cache=sg["cache"])
        idx = fp.fps_exact(x, n, ws=sg["ws"][0])
        x_next = None if s + 1 == len(ctx["stages"]) else fp.gather_xyz(x, idx)
        bqs.wait_stream(main)
        with torch.cuda.stream(bqs):
            bq = fp.ball_query(x, idx, r, k)
        if keep is not None:
            keep.append((x, idx, bq, midx, mbq))
        x = x_next
    for other in (lanes[0], lanes[1], bqs):
        main.wait_stream(other)


def measure_eager(torch, fp, ctx, steps, warmup):
    """(ms per step, mean ms per kernel): every call alone, one stream, eager launches."""
    timer = Timer(torch)
    for _ in range(warmup):
        run_step(fp, ctx, timer)
    torch.cuda.synchronize()
    timer.reset()
    t0 = time.perf_counter()
    for _ in range(steps):
        run_step(fp, ctx, timer)
    torch.cuda.synchronize()
    seq_ms = (time.perf_counter() - t0) * 1e3 / steps
    timer.collect()
    return seq_ms, timer.mean_ms(), timer.min_median_ms()


def one_workgroup_per_cloud(ctx):
    """A cloud spread over several workgroups fills the device: nothing to run beside it."""
    return all(sg["G"] == 1 for sg in ctx["stages"])


def measure_graph(torch, fp, ctx, steps, warmup):
    """ms per step for small clouds: four streams, the step captured once in a graph and
    replayed; the replay's outputs are checked against the eager ones.  Called after all eager
    measurements of the process: once a graph with a second stream has run, eager launches on
    the streams that existed by then take tens of microseconds longer each."""
    eager = []
    run_step_streams(torch, fp, ctx, eager)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    held = []
    with torch.cuda.graph(graph):
        run_step_streams(torch, fp, ctx, held)
    for _ in range(max(warmup, 1)):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    for got, want in zip(held, eager):
        for g, w in zip(got[1:], want[1:]):
            same = all(torch.equal(a, b) for a, b in zip(g, w)) if isinstance(g, tuple) else torch.equal(g, w)
            if not same:
                raise RuntimeError("graph replay of the step differs from the eager result")
    return ms


def quality_and_rooflines(torch, fp, ctx, kernel_ms):
    """Sampling quality of MDPS against exact FPS and achieved fraction of the binding
    roofline of every kernel of the step (stage 0 is where the time goes)."""
    timer = Timer(torch)
    keep = []
    run_step(fp, ctx, timer, keep)
    torch.cuda.synchronize()
    wl = ctx["wl"]
    out = {"stages": []}
    for s, sg in enumerate(ctx["stages"]):
        n, k = sg["n"], sg["k"]
        x, idx, bq, midx, mbq = keep[s]
        B, N = x.shape[0], x.shape[1]
        _, info = fp.mdps_sample(x, n, sg["prm"], want_info=True)
        cov_f = fp.coverage2(x, idx).sqrt()
        cov_m = fp.coverage2(x, midx).sqrt()
        torch.cuda.synchronize()
        infos = fp.parse_info(info)
        ratio = (cov_m / cov_f)
        brute_m = fp.ball_query(x, midx, sg["radius"], k)
        torch.cuda.synchronize()
        cached_equal = bool(torch.equal(brute_m[0], mbq[0]) and torch.equal(brute_m[1], mbq[1]))
        ms = {key.split("/")[0]: v for key, v in kernel_ms.items() if key.endswith("/s%d" % s)}
        point_iters = float(B) * (n - 1) * N
        pairs = float(B) * n * N
        roof = {}
        if "fps_exact" in ms:
            a = point_iters * OPS_PER_POINT_ITERATION / (ms["fps_exact"] * 1e-3) / 1e12
            roof["fps_exact"] = {"bound": "alu", "achieved": a, "peak": ALU_PEAK_TOPS, "unit": "TFLOP/s",
                                 "frac": a / ALU_PEAK_TOPS, "us_per_iteration": ms["fps_exact"] * 1e3 / max(n - 1, 1)}
        if "mdps_sample+record" in ms:
            a = point_iters * OPS_PER_POINT_ITERATION / (ms["mdps_sample+record"] * 1e-3) / 1e12
            roof["mdps_sample+record"] = {"bound": "alu", "achieved": a, "peak": ALU_PEAK_TOPS,
                                          "unit": "TFLOP/s", "frac": a / ALU_PEAK_TOPS}
            if sg["pruned_record"]:
                roof["mdps_sample+record"]["note"] = ("algorithmic operations of the unpruned update / time: "
                                                      "the cell-ordered sampler skips most of them")
        if "ball_query_brute" in ms:
            a = pairs * OPS_PER_PAIR_TEST / (ms["ball_query_brute"] * 1e-3) / 1e12
            roof["ball_query_brute"] = {"bound": "alu", "achieved": a, "peak": ALU_PEAK_TOPS,
                                        "unit": "TFLOP/s", "frac": a / ALU_PEAK_TOPS,
                                        "note": "pair tests priced at the 9 operations of the full test / time: "
                                                "most pairs are decided after 6"}
        if "ball_query_cached" in ms:
            # algorithmic bytes: the recorded entries of the centres' rows (12 bytes each) and their
            # offsets read, the result written
            cstats = fp.bq_cache_stats(sg["cache"])
            byts = 12.0 * sum(cstats["entries"]) + 8.0 * B * n + 4.0 * B * n * (k + 1)
            a = byts / (ms["ball_query_cached"] * 1e-3) / 1e9
            roof["ball_query_cached"] = {"bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                         "frac": a / HBM_PEAK_GBS, "bytes": byts,
                                         "cache_bytes": cstats["bytes"], "cache_entries": cstats["entries"],
                                         "cache_incomplete": cstats["incomplete"]}
        knn = time_knn(torch, fp, x, sg, midx)
        for kname in ("knn_brute", "knn_cached"):
            ms[kname] = knn[kname + "_ms"]
        # the same k-NN through a grid over the samples, search radius 3 x their coverage radius
        kg_radius = 3.0 * float(cov_m.max())
        kg = time_call(torch, lambda: fp.knn_grid(x, knn["samples"], KNN_K, kg_radius, want_deferred=True))
        if not (torch.equal(kg[1][0], knn["knn_brute"][0]) and torch.equal(kg[1][1], knn["knn_brute"][1])):
            raise RuntimeError("grid k-NN differs from the brute-force result")
        ms["knn_grid"] = kg[0]
        a = float(B) * N * n * OPS_PER_PAIR_TEST / (knn["knn_brute_ms"] * 1e-3) / 1e12
        roof["knn_brute"] = {"bound": "alu", "achieved": a, "peak": ALU_PEAK_TOPS, "unit": "TFLOP/s",
                             "frac": a / ALU_PEAK_TOPS}
        # the redundancy-free search reads the recorded entries (regrouped by point block) and the
        # points, and writes the result
        byts = (16.0 + 2 * 12.0) * sum(fp.bq_cache_stats(knn["cache"])["entries"]) + 12.0 * B * N + 2.0 * B * N * KNN_K * 4
        a = byts / (knn["knn_cached_ms"] * 1e-3) / 1e9
        roof["knn_cached"] = {"bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": a / HBM_PEAK_GBS, "bytes": byts,
                              "points_searched_by_brute_force": knn["deferred_fraction"]}
        # ball query through the uniform grid (outside the timed step): the brute-force result
        gq = time_call(torch, lambda: fp.ball_query_grid(x, idx, sg["radius"], k))
        if not (torch.equal(gq[1][0], bq[0]) and torch.equal(gq[1][1], bq[1])):
            raise RuntimeError("ball_query_grid differs from the brute-force ball query")
        ms["ball_query_grid"] = gq[0]
        byts = 12.0 * B * N + 4.0 * B * n + 4.0 * B * n * (k + 1)
        a = byts / (gq[0] * 1e-3) / 1e9
        roof["ball_query_grid"] = {"bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                   "frac": a / HBM_PEAK_GBS, "bytes": byts, "equals_brute_force": True}
        # exact FPS with pruned distance updates (outside the timed step): same samples, fewer
        # distance evaluations; priced against the same algorithmic count as fps_exact
        pr = time_call(torch, lambda: fp.fps_exact_pruned(x, n))
        if not torch.equal(pr[1], idx):
            raise RuntimeError("fps_exact_pruned differs from fps_exact")
        ms["fps_exact_pruned"] = pr[0]
        a = point_iters * OPS_PER_POINT_ITERATION / (pr[0] * 1e-3) / 1e12
        roof["fps_exact_pruned"] = {"bound": "alu", "achieved": a, "peak": ALU_PEAK_TOPS, "unit": "TFLOP/s",
                                    "frac": a / ALU_PEAK_TOPS, "equals_fps_exact": True,
                                    "note": "algorithmic operations of the unpruned update / time"}
        # MDPS with pruned distance updates (outside the timed step): the samples of mdps_sample,
        # timed without and with pruning (neither records the radius tests)
        mp_plain = time_call(torch, lambda: fp.mdps_sample(x, n, sg["prm"]))
        mp = time_call(torch, lambda: fp.mdps_sample_pruned(x, n, sg["prm"]))
        if not torch.equal(mp[1], mp_plain[1]):
            raise RuntimeError("mdps_sample_pruned differs from mdps_sample")
        ms["mdps_sample"] = mp_plain[0]
        ms["mdps_sample_pruned"] = mp[0]
        # both recording samplers with their readers (the step runs the one named in record_sampler)
        other = torch.empty_like(sg["cache"])
        for label, entry, prm_r in (("mdps_sample+record_index_order", fp.mdps_sample, sg["prm"]),
                                    ("mdps_sample_pruned+record", fp.mdps_sample_pruned, sg["prm"]),
                                    ("mdps_sample_pruned+record_scattered", fp.mdps_sample_pruned,
                                     dataclasses.replace(sg["prm"], scan_order=1))):
            rec = time_call(torch, lambda: entry(x, n, prm_r, bq_cache=other, bq_radius=sg["radius"]))
            rd = time_call(torch, lambda: fp.ball_query(x, rec[1], sg["radius"], k, bq_cache=other))
            chk = fp.ball_query_grid(x, rec[1], sg["radius"], k)
            if not (torch.equal(rd[1][0], chk[0]) and torch.equal(rd[1][1], chk[1])):
                raise RuntimeError(label + ": neighbours read from the record differ from the grid query's")
            if prm_r.scan_order == sg["step_prm"].scan_order and not torch.equal(rec[1], midx):
                raise RuntimeError(label + ": samples differ from the step's")
            ms[label] = rec[0]
            ms[label.replace("mdps_sample", "ball_query_cached_after")] = rd[0]
        del other
        # The scattered scan order of the threshold phase (Section 4.1 step 3 takes any available
        # point; here the first one of a walk with a golden-ratio stride instead of the lowest
        # index): on the cloud in walk order, and in cell order with pruned updates.  The fastest
        # sampler of the library on large clouds; it does not record, so its ball query is the
        # grid's (timed on its samples).
        sprm = dataclasses.replace(sg["prm"], scan_order=1)
        sc = time_call(torch, lambda: fp.mdps_sample(x, n, sprm, want_info=True))
        scp = time_call(torch, lambda: fp.mdps_sample_pruned(x, n, sprm))
        if not torch.equal(scp[1], sc[1][0]):
            raise RuntimeError("mdps_sample_pruned differs from mdps_sample (scattered scan order)")
        scov = fp.coverage2(x, scp[1]).sqrt() / cov_f
        gqs = time_call(torch, lambda: fp.ball_query_grid(x, scp[1], sg["radius"], k))
        torch.cuda.synchronize()
        sinfos = fp.parse_info(sc[1][1])
        ms["mdps_sample_scattered"] = sc[0]
        ms["mdps_sample_pruned_scattered"] = scp[0]
        ms["ball_query_grid_scattered"] = gqs[0]
        scattered_detail = {"coverage_ratio_max": float(scov.max()), "coverage_ratio_mean": float(scov.mean()),
                            "fps_tail_fraction_mean": float(sum((n - i.et_index) / n for i in sinfos) / len(sinfos)),
                            "rounds_mean": float(sum(i.rounds for i in sinfos) / len(sinfos)),
                            "sample_spacing_ratio": sample_spacing(torch, fp, x, scp[1]) / sample_spacing(torch, fp, x, idx)}
        # MDPS with the MLP curve estimator of Appendix A.3 in place of the power function
        # (outside the timed step): latency and sampling quality
        from paper_2507_23480_amd import mlp_estimator
        mprm = mlp_estimator.params_for(ctx["name"], s)
        ml = time_call(torch, lambda: fp.mdps_sample(x, n, mprm, want_info=True))
        mcov = fp.coverage2(x, ml[1][0]).sqrt() / cov_f
        torch.cuda.synchronize()
        minfos = fp.parse_info(ml[1][1])
        ms["mdps_sample_mlp"] = ml[0]
        mlp_detail = {"coverage_ratio_max": float(mcov.max()), "coverage_ratio_mean": float(mcov.mean()),
                      "fps_tail_fraction_mean": float(sum((n - i.et_index) / n for i in minfos) / len(minfos)),
                      "last_level_exhausted": int(sum(1 for i in minfos if i.et_index < n)),
                      "curve_mape_percent": mlp_estimator.table()[ctx["name"]][s].get("mape_percent_workload"),
                      "bias": mprm.bias}
        # MDPS with the estimator exactly as Appendix A.3 defines it (a / x^e, no per-segment
        # factors; exponent and bias fitted the same way): latency and sampling quality
        pprm = calibration_module().params_for(ctx["name"], s, "paper")
        pp = time_call(torch, lambda: fp.mdps_sample(x, n, pprm, want_info=True))
        pcov = fp.coverage2(x, pp[1][0]).sqrt() / cov_f
        torch.cuda.synchronize()
        pinfos = fp.parse_info(pp[1][1])
        ms["mdps_sample_paper_estimator"] = pp[0]
        paper_detail = {"coverage_ratio_max": float(pcov.max()), "coverage_ratio_mean": float(pcov.mean()),
                        "fps_tail_fraction_mean": float(sum((n - i.et_index) / n for i in pinfos) / len(pinfos)),
                        "last_level_exhausted": int(sum(1 for i in pinfos if i.et_index < n)),
                        "sample_spacing_ratio": sample_spacing(torch, fp, x, pp[1][0]) / sample_spacing(torch, fp, x, idx),
                        "bias": pprm.bias, "exponent": pprm.exponent}
        ex = time_excl_lists(torch, fp, x, sg, infos, midx, mbq)
        if not ex["built"]:
            roof["excl_lists_build"] = {"built": False, "members": ex["members"], "levels": ex["levels"],
                                        "reason": ex["reason"]}
        else:
            ms["excl_lists_count"], ms["excl_lists_fill"] = ex["count_ms"], ex["fill_ms"]
            # the lists have to be written once and the points read once
            byts = 4.0 * ex["members"] + 8.0 * ex["rows"] + 12.0 * B * N
            a = byts / ((ex["count_ms"] + ex["fill_ms"]) * 1e-3) / 1e9
            roof["excl_lists_build"] = {"bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                        "frac": a / HBM_PEAK_GBS, "bytes": byts, "members": ex["members"],
                                        "levels": ex["levels"], "lookup_equals_ball_query": ex["lookup_ok"]}
        byts = 12.0 * B * N + 12.0 * B * n + 8.0 * B * N * KNN_K
        a = byts / (ms["knn_grid"] * 1e-3) / 1e9
        roof["knn_grid"] = {"bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": a / HBM_PEAK_GBS,
                            "bytes": byts, "radius": kg_radius,
                            "points_searched_by_brute_force": float(kg[1][2].sum().item()) / (B * N)}
        out["stages"].append({
            "N": N, "n": n, "radius": sg["radius"], "k": k, "plan_G_T_P": list(fp.plan(B, N)),
            "record_sampler": "mdps_sample_pruned" if sg["pruned_record"] else "mdps_sample",
            "kernel_ms": ms,
            # microseconds per sample of a launch (all clouds of the batch run side by side)
            "fps_exact_us_per_sample": ms["fps_exact"] * 1e3 / max(n - 1, 1) if "fps_exact" in ms else None,
            "mdps_sample_us_per_sample": ms["mdps_sample"] * 1e3 / max(n - 1, 1) if "mdps_sample" in ms else None,
            "mdps_coverage_ratio_max": float(ratio.max()), "mdps_coverage_ratio_mean": float(ratio.mean()),
            # the paper's quality figure (Table 1): mean distance from a sample to the nearest other
            # sample, MDPS relative to exact FPS
            "mdps_sample_spacing_ratio": sample_spacing(torch, fp, x, midx) / sample_spacing(torch, fp, x, idx),
            "mdps_fps_tail_fraction_mean": float(sum((n - i.et_index) / n for i in infos) / len(infos)),
            "mdps_prefix_fraction": float(infos[0].m / n),
            "mdps_rounds_mean": float(sum(i.rounds for i in infos) / len(infos)),
            # mean over the clouds of the time in each phase of Section 4.1 (device clock, the call
            # without radius recording): exact FPS first, estimator, threshold sampling, remainder FPS
            "mdps_phase_us": {name: float(sum(i.phase_ticks[j] for i in infos) / len(infos)) * 0.01
                              for j, name in enumerate(["prefix_fps", "estimator_thresholds",
                                                        "threshold_sampling", "remainder_fps"])},
            "mdps_last_level_exhausted": int(sum(1 for i in infos if i.et_index < n)),
            "mdps_speedup_vs_fps": ms.get("fps_exact", 0.0) / ms["mdps_sample+record"] if ms.get("mdps_sample+record") else None,
            "cached_ball_query_equals_brute": cached_equal,
            "mdps_mlp_estimator": mlp_detail,
            "mdps_paper_estimator": paper_detail,
            "mdps_scattered_order": scattered_detail,
            "roofline": roof})
    return out


def calibration_module():
    from paper_2507_23480_amd import calibration
    return calibration


def sample_spacing(torch, fp, x, sidx):
    """Mean over the clouds' samples of the distance to the nearest other sample (through fp_knn on
    the gathered samples: the nearest sample of a sample is itself, the second is the one wanted)."""
    xs = fp.gather_xyz(x, sidx).contiguous()
    B, n = sidx.shape[0], sidx.shape[1]
    if n < 2:
        return 1.0
    every = torch.arange(n, dtype=torch.int32, device=x.device).repeat(B, 1).contiguous()
    _, d2 = fp.knn(xs, every, 2)
    torch.cuda.synchronize()
    return float(d2[:, :, 1].double().sqrt().mean())


def time_call(torch, fn, reps=3):
    """(best ms of `reps` calls timed with events after one warm-up, last result)."""
    out = fn()
    torch.cuda.synchronize()
    best = None
    for _ in range(reps):
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        out = fn()
        b.record()
        torch.cuda.synchronize()
        t = a.elapsed_time(b)
        best = t if best is None else min(best, t)
    return best, out


def time_excl_lists(torch, fp, x, sg, infos, midx, mbq, reps=3):
    """Exclusion lists of a stage as a data structure (the list-building loops of Alg. 2): one level per MDPS
    threshold of each cloud plus the ball-query radius; count and fill passes timed apart, and
    the stage's ball query answered by lookup in the extra level.  Not part of the timed step.
    The count pass always runs (it sizes the member array).  When the members would take more than
    EXCL_MEMBER_BUDGET bytes the lists are not built: the result then says how many members there
    are and what they would need (the large single cloud: its first-level radius spans whole
    clusters)."""
    import numpy as np
    B, N = x.shape[0], x.shape[1]
    lib = fp.load()
    nseg = sg["prm"].nseg
    r2 = np.float32(sg["radius"]) * np.float32(sg["radius"])
    thr = torch.tensor([[i.thr2[l] for l in range(nseg)] + [float(r2)] for i in infos],
                       dtype=torch.float32, device=x.device)
    L = nseg + 1
    ws = torch.empty(lib.fp_excl_workspace_bytes(B, N, L), dtype=torch.uint8, device=x.device)
    off = torch.empty(L * B * N + 1, dtype=torch.int64, device=x.device)
    st = torch.cuda.current_stream().cuda_stream

    def count():
        if lib.fp_excl_count(x.data_ptr(), B, N, thr.data_ptr(), L, off.data_ptr(), ws.data_ptr(), ws.numel(), st):
            raise RuntimeError("fp_excl_count failed")

    def timed(fn):
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

    count()
    torch.cuda.synchronize()
    total = int(off[-1].item())
    if 4 * total > EXCL_MEMBER_BUDGET:
        return {"built": False, "count_ms": timed(count) if N <= 200000 else None, "members": total,
                "rows": L * B * N, "levels": L,
                "reason": "%d members would take %.1f GB, above the benchmark's budget of %.0f GB for this "
                          "structure" % (total, 4.0 * total / 1e9, EXCL_MEMBER_BUDGET / 1e9)}
    ent = torch.empty(max(total, 1), dtype=torch.int32, device=x.device)

    def fill():
        if lib.fp_excl_fill(x.data_ptr(), B, N, thr.data_ptr(), L, off.data_ptr(), ent.data_ptr(), total,
                            ws.data_ptr(), ws.numel(), st):
            raise RuntimeError("fp_excl_fill failed")

    res = {"built": True, "count_ms": timed(count), "fill_ms": timed(fill), "members": total, "rows": L * B * N,
           "levels": L}
    idx, cnt = fp.ball_query_lists(off, ent, B, N, L, nseg, midx, sg["k"])
    torch.cuda.synchronize()
    res["lookup_ok"] = bool(torch.equal(idx, mbq[0]) and torch.equal(cnt, mbq[1]))
    if not res["lookup_ok"]:
        raise RuntimeError("ball query by lookup differs from the cache reader's result")
    return res


def time_knn(torch, fp, x, sg, midx, reps=3):
    """k nearest MDPS samples of every point of a stage: brute force and through the recorded
    ball bitmaps (both give the same result; checked here).  Not part of the timed step."""
    res = {}
    kcache = sg["cache"]
    if sg["pruned_record"]:
        # the step's record is in cell order, which the k-NN search does not read: record once more
        # with the index-ordered sampler (its samples are those of the same constants with scan order 0)
        kcache = torch.empty_like(sg["cache"])
        midx = fp.mdps_sample(x, midx.shape[1], sg["prm"], bq_cache=kcache, bq_radius=sg["radius"])
    for kname, cache in (("knn_brute", None), ("knn_cached", kcache)):
        fp.knn(x, midx, KNN_K, bq_cache=cache)
        torch.cuda.synchronize()
        best = None
        for _ in range(reps):
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            a.record()
            out = fp.knn(x, midx, KNN_K, bq_cache=cache, want_deferred=cache is not None)
            b.record()
            torch.cuda.synchronize()
            t = a.elapsed_time(b)
            best = t if best is None else min(best, t)
        res[kname + "_ms"] = best
        res[kname] = out
    same = torch.equal(res["knn_brute"][0], res["knn_cached"][0]) and \
        torch.equal(res["knn_brute"][1], res["knn_cached"][1])
    if not same:
        raise RuntimeError("redundancy-free k-NN differs from the brute-force result")
    res["deferred_fraction"] = float(res["knn_cached"][2].sum().item()) / (x.shape[0] * x.shape[1])
    res["samples"] = midx
    res["cache"] = kcache
    return res


def cpu_baseline(inputs, name, budget_s=12.0):
    """The CPU oracle, as it stands, on the same workload (one thread).

    C1-C3: whole clouds through all stages until the time budget is used.  C4 and C5: the oracle
    would need minutes for one step, so a bounded sample is timed -- exact FPS and MDPS for the first
    CPU_SAMPLE_N samples and the ball query of CPU_SAMPLE_M centres on the first cloud at its full
    size -- and reported as rates; the step time is extrapolated from them (every pick folds all N
    points, every centre tests all N points) and says so."""
    import numpy as np
    from oracle import ref
    from paper_2507_23480_amd import calibration
    wl = inputs.WORKLOADS[name]
    batch = inputs.make_batch(name)

    def params(s):
        ent = calibration.table()[name][s]
        return ref.MdpsParams(p=calibration.P_RATIO, nseg=calibration.NSEG, exponent=ent["exponent"],
                              bias=ent["bias"], fit_window=calibration.FIT_WINDOW,
                              m_min=calibration.M_MIN, level_scale=ent["level_scale"])

    if name in ("C4", "C5"):
        st = wl.stages[0]
        x = batch[0]
        ns, ms = CPU_SAMPLE_N, CPU_SAMPLE_M
        t0 = time.perf_counter()
        idx, _ = ref.fps_exact(x, ns)
        t1 = time.perf_counter()
        ref.mdps_sample(x, ns, params(0))
        t2 = time.perf_counter()
        ref.ball_query(x, idx[:ms], st.radius, st.k)
        t3 = time.perf_counter()
        fps_rate = (ns - 1) * float(wl.N) / (t1 - t0)             # point-iterations per second
        mdps_rate = (ns - 1) * float(wl.N) / (t2 - t1)
        bq_rate = ms * float(wl.N) / (t3 - t2)                    # pair tests per second
        step_s = wl.B * ((st.n - 1) * float(wl.N) * (1.0 / fps_rate + 1.0 / mdps_rate) +
                         2.0 * st.n * float(wl.N) / bq_rate)
        return {"value": wl.B * wl.N / step_s / 1e6, "unit": "Mpoints/s", "cores": 1, "kind": "oracle",
                "sample": "RATES, not a full run: cloud 0 of %s at full N, first %d samples of fps_exact "
                          "(%.1f s) and mdps_sample (%.1f s), ball query of %d centres (%.1f s); step "
                          "extrapolated linearly in samples and centres" % (name, ns, t1 - t0, t2 - t1, ms, t3 - t2),
                "fps_point_iterations_per_s": round(fps_rate), "mdps_point_iterations_per_s": round(mdps_rate),
                "ball_query_pair_tests_per_s": round(bq_rate), "ms_per_step_extrapolated": round(step_s * 1e3)}

    done_points = 0
    clouds = 0
    t0 = time.perf_counter()
    while True:
        for b in range(wl.B):
            x = batch[b]
            for s, st in enumerate(wl.stages):
                prm = params(s)
                idx, _ = ref.fps_exact(x, st.n)
                ref.ball_query(x, idx, st.radius, st.k)
                midx, _ = ref.mdps_sample(x, st.n, prm)
                ref.ball_query(x, midx, st.radius, st.k)
                if s + 1 < len(wl.stages):
                    x = ref.gather_xyz(x, idx)
            done_points += wl.N
            clouds += 1
            if time.perf_counter() - t0 > budget_s:
                break
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    return {"value": done_points / dt / 1e6, "unit": "Mpoints/s", "cores": 1, "kind": "oracle",
            "sample": "%d clouds of workload %s (all stages, same step as the GPU: fps_exact, ball_query, "
                      "mdps_sample, ball_query) in %.1f s" % (clouds, name, dt),
            "ms_per_batch_equivalent": dt * 1e3 / clouds * wl.B}


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives, "
              "no sharding across devices in this library)" % args.gpus, file=sys.stderr)
        return 2
    os.makedirs(os.path.dirname(os.path.abspath(args.detail_file)), exist_ok=True)
    extra = {} if args.no_extra else other_workloads(args.workload, args.detail_file)
    clock_reader = None if args.no_extra else start_clock_reader()
    import torch
    from paper_2507_23480_amd import binding as fp, inputs, calibration
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    fp.load()
    if args.plain_launch:
        fp.set_cooperative_launch(False)
    return run(args, torch, fp, inputs, calibration, extra, clock_reader)


def start_clock_reader():
    """A child process that reads the device's clocks once it is told to.  Started before this
    process touches the GPU (afterwards it starts no programs)."""
    import subprocess
    try:
        return subprocess.Popen(["sh", "-c", "read go; exec rocm-smi --showclocks --json"],
                                stdin=subprocess.PIPE, stdout=subprocess.PIPE, stderr=subprocess.DEVNULL)
    except Exception:
        return None


def clocks_under_load(torch, fp, reader):
    """Engine and memory clock (MHz) read by rocm-smi while a plain fp32 kernel of about a
    second keeps every compute unit busy; None where rocm-smi gives no answer."""
    if reader is None:
        return None
    try:
        out = torch.empty(8192 * 256, dtype=torch.float32, device="cuda")
        if fp.load().fp_probe_fp32_rate(8192, 1500000, out.data_ptr(), None) != 0:
            raise RuntimeError("probe")
        time.sleep(0.3)
        text = reader.communicate(b"go\n", timeout=30)[0].decode()
        torch.cuda.synchronize()
        card = next(iter(json.loads(text[text.index("{"):]).values()))
        mhz = lambda key: int("".join(ch for ch in card[key] if ch.isdigit()))
        return {"sclk_mhz": mhz("sclk clock speed:"), "mclk_mhz": mhz("mclk clock speed:"),
                "source": "rocm-smi --showclocks during a one-second fp32 kernel on all compute units"}
    except Exception:
        try:
            reader.kill()
            torch.cuda.synchronize()
        except Exception:
            pass
        return None


def other_workloads(name, detail_file):
    """The other workloads, each measured by a process of its own (started before this one
    touches the GPU): cooperative launches and graph replays with a second stream slow each
    other's launches down by tens of microseconds once both have run in one process.  Returns
    {workload: its short summary}; each child writes its own detail file next to `detail_file`."""
    import subprocess
    extra = {}
    stem, ext = os.path.splitext(detail_file)
    for other in ["C1", "C2", "C3", "C4", "C5"]:
        if other == name:
            continue
        k = 3 if other in ("C4", "C5") else 10
        cmd = [sys.executable, os.path.abspath(__file__), "--workload", other, "--no-extra", "--no-cpu",
               "--steps", str(k), "--warmup", "1", "--detail-file", "%s_%s%s" % (stem, other, ext)]
        try:
            out = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, timeout=240,
                                 check=True).stdout.decode()
            d = json.loads(out.strip().splitlines()[-1])
            extra[other] = d["workloads"][other]
        except Exception as exc:                 # reported, not fatal: the headline line still prints
            extra[other] = {"error": repr(exc)[:120]}
    return extra


def path_summary(wl, detail, ms_per_step, launch_mode, roof):
    """The short entry of one workload: time of the exact path (fps_exact + brute-force ball query
    [+ gather of the next stage's input]) and of the FastPoint path (mdps_sample recording the
    radius tests + ball query from the record), summed over the stages, each kernel timed alone."""
    exact = fast = fast_grid = best = 0.0
    for st in detail["stages"]:
        ms = st["kernel_ms"]
        exact += ms["fps_exact"] + ms["ball_query_brute"] + ms.get("gather", 0.0)
        fast += ms["mdps_sample+record"] + ms["ball_query_cached"]
        # the same samples and neighbours without the record: plain MDPS, then the grid ball query
        fast_grid += ms["mdps_sample"] + ms["ball_query_grid"]
        # the fastest sampler and ball query per stage: MDPS with either scan order, with or without
        # pruned updates, then the grid ball query on its samples (or the record where that wins)
        best += min(min(ms["mdps_sample"], ms["mdps_sample_pruned"]) + ms["ball_query_grid"],
                    min(ms["mdps_sample_scattered"], ms["mdps_sample_pruned_scattered"]) + ms["ball_query_grid_scattered"],
                    ms["mdps_sample+record_index_order"] + ms["ball_query_cached_after+record_index_order"],
                    ms["mdps_sample_pruned+record"] + ms["ball_query_cached_after_pruned+record"],
                    ms["mdps_sample_pruned+record_scattered"] + ms["ball_query_cached_after_pruned+record_scattered"])
    pts = wl.B * wl.N / 1e6
    s0 = detail["stages"][0]
    return {"ms_per_step": round(ms_per_step, 4), "launch": "graph" if launch_mode == GRAPH else "eager",
            "exact_path_ms": round(exact, 4), "fastpoint_path_ms": round(fast, 4),
            "mdps_plus_grid_query_ms": round(fast_grid, 4), "best_mdps_path_ms": round(best, 4),
            "exact_Mpoints_s": round(pts / (exact * 1e-3), 2), "fastpoint_Mpoints_s": round(pts / (fast * 1e-3), 2),
            "mdps_coverage_ratio_max": round(max(st["mdps_coverage_ratio_max"] for st in detail["stages"]), 4),
            # the estimator as the paper defines it (level_scale = 1): worst coverage ratio, share of the
            # samples left to the exact iterations after early termination (stage 0)
            "paper_est_coverage_max": round(max(st["mdps_paper_estimator"]["coverage_ratio_max"]
                                                for st in detail["stages"]), 4),
            "paper_est_fps_tail": round(s0["mdps_paper_estimator"]["fps_tail_fraction_mean"], 4),
            "fps_tail": round(s0["mdps_fps_tail_fraction_mean"], 4),
            "mdps_over_fps_time": round(s0["kernel_ms"]["mdps_sample"] / s0["kernel_ms"]["fps_exact"], 3),
            # the fastest MDPS variant of stage 0 (scan order, pruning) against fps_exact, and its coverage
            "best_mdps_over_fps_time": round(min(s0["kernel_ms"][v] for v in (
                "mdps_sample", "mdps_sample_pruned", "mdps_sample_scattered", "mdps_sample_pruned_scattered"))
                / s0["kernel_ms"]["fps_exact"], 3),
            "scattered_coverage_max": round(max(st["mdps_scattered_order"]["coverage_ratio_max"]
                                                for st in detail["stages"]), 4),
            "dominant_kernel": roof["kernel"].replace(" (stage 0)", ""), "dominant_frac": round(roof["frac"], 4)}


def run(args, torch, fp, inputs, calibration, extra, clock_reader=None):
    name = args.workload
    ctx = make_context(torch, fp, inputs, calibration, name)
    seq_ms, kernel_ms, kernel_min_median = measure_eager(torch, fp, ctx, args.steps, args.warmup)
    wl = ctx["wl"]
    detail = quality_and_rooflines(torch, fp, ctx, kernel_ms)
    for s, stage in enumerate(detail["stages"]):
        # the timed step's kernels over the timed steps: (min, median) beside the mean in kernel_ms
        stage["kernel_ms_min_median"] = {key.split("/")[0]: [round(v[0], 6), round(v[1], 6)]
                                         for key, v in kernel_min_median.items() if key.endswith("/s%d" % s)}
    props = torch.cuda.get_device_properties(ctx["xyz"].device)
    detail["device"] = {"name": props.name, "compute_units": int(props.multi_processor_count),
                        "memory_gib": round(props.total_memory / 2.0 ** 30, 1)}
    clocks = clocks_under_load(torch, fp, clock_reader)
    if clocks:
        detail["device"]["clocks_under_load"] = clocks
    s0 = detail["stages"][0]
    # dominant kernel of the step: the one with the largest share of the time
    in_step = [kname for kname in s0["roofline"]
               if kname in ("fps_exact", "mdps_sample+record", "ball_query_brute", "ball_query_cached")]
    dom = max(in_step, key=lambda kname: s0["kernel_ms"].get(kname, 0.0))
    roof = dict(s0["roofline"][dom])
    roof["kernel"] = dom + " (stage 0)"
    roof["ms_per_launch"] = s0["kernel_ms"][dom]
    roof["traffic"] = TRAFFIC_BYTES.get(name, {}).get(dom)
    if roof.get("bound") == "alu":
        # the published peak needs packed binary32 instructions, which this path may not use (every
        # operation rounds on its own); the rate the device reaches without them, measured here
        probe = fp.probe_fp32_rate(ctx["xyz"].device) / 1e12
        roof["plain_fp32_rate_measured"] = probe
        roof["frac_of_plain_fp32_rate"] = roof["achieved"] / probe
    if dom in ("fps_exact", "mdps_sample+record"):
        # the sampler runs a cloud on plan.G workgroups, one per compute unit: what share of the
        # device the launch can occupy at all, and the fraction of those units' peak
        G = ctx["stages"][0]["G"]
        units = min(256, wl.B * G)
        roof["compute_units_in_use"] = units
        roof["frac_of_units_in_use"] = roof["frac"] * 256.0 / units
    # graph replay after all eager measurements of this process (see measure_graph)
    ms_per_step, launch_mode = seq_ms, EAGER
    if one_workgroup_per_cloud(ctx):
        ms_per_step, launch_mode = measure_graph(torch, fp, ctx, args.steps, args.warmup), GRAPH
    summary = path_summary(wl, detail, ms_per_step, launch_mode, roof)
    workloads = dict(extra)
    workloads[name] = summary
    short_roof = {key: (round(roof[key], 5) if isinstance(roof[key], float) else roof[key])
                  for key in ("bound", "achieved", "peak", "unit", "frac", "traffic", "kernel", "ms_per_launch",
                              "plain_fp32_rate_measured", "frac_of_plain_fp32_rate", "compute_units_in_use", "bytes")
                  if key in roof}
    line = {
        "metric": "FPS+ball-query latency per batch (ms) and Mpoints/s; achieved HBM GB/s vs peak",
        "value": wl.B * wl.N / (ms_per_step * 1e-3) / 1e6, "unit": "Mpoints/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: %s" % (name, wl.description), "B": wl.B, "N": wl.N,
                   "stages": [{"n": st.n, "radius": st.radius, "k": st.k} for st in wl.stages],
                   "step": "per stage: fps_exact + ball_query(brute) [+ gather]; "
                           "%s(+record) + ball_query(from record)"
                           % ("mdps_sample_pruned[scan order 1]" if ctx["stages"][0]["pruned_record"] else "mdps_sample"),
                   "launch": launch_mode, "mdps": {"p": calibration.P_RATIO, "nseg": calibration.NSEG}},
        "paths": {"exact_path_ms": summary["exact_path_ms"], "fastpoint_path_ms": summary["fastpoint_path_ms"],
                  "exact_Mpoints_s": summary["exact_Mpoints_s"],
                  "fastpoint_Mpoints_s": summary["fastpoint_Mpoints_s"]},
        "roofline": short_roof,
    }
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(inputs, name)
    line["workloads"] = {key: workloads[key] for key in sorted(workloads)}
    line["detail_file"] = os.path.relpath(args.detail_file, ROOT)
    if args.copy_probe:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    full = dict(line)
    full["roofline"] = roof
    full["config"] = dict(line["config"], ms_per_step_one_stream_eager=seq_ms)
    full["detail"] = detail
    with open(args.detail_file, "w") as f:
        json.dump(full, f, indent=1)
        f.write("\n")
    text = json.dumps(line)
    if len(text) > 3900:                       # the driver reads the tail of stdout: keep the line short
        for key in ("detail_file",):
            line.pop(key, None)
        for w in line["workloads"].values():
            for key in ("dominant_kernel", "exact_Mpoints_s", "fastpoint_Mpoints_s", "launch"):
                w.pop(key, None)
        text = json.dumps(line)
    sys.stdout.flush()
    print(text, flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
