"""Pins for the oracle's MDPS (Algorithm 2, Section 4.1, Appendix A.1/A.3).

MDPS is an approximation, so there is no plain definition of its output.  What
pins it: hand-worked examples, the estimator's closed form on exact power-law
curves, the equality of the running-min-distance form with the explicit
exclusion-list/bitmap form, the special cases that reduce to exact FPS or to a
plain index scan, and the invariants the paper states (spacing lower bound per
segment, coverage at exhaustion, early termination continuing as exact FPS).
"""
import math
import os

import numpy as np
import pytest

from oracle import ref
from paper_2507_23480_amd import inputs
from test_oracle_fps import d2_matrix, line9

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
FLT_MIN = np.float32(1.17549435e-38)


# ------------------------------------------------------------------ hand examples
def test_line_examples_match_hand_derivation():
    for l in open(os.path.join(GOLDEN, "mdps_line9.txt")):
        if l.startswith("#") or not l.strip():
            continue
        head, want, et = [s.split() for s in l.split("|")]
        n, nseg = int(head[1]), int(head[2])
        thr = [float(v) for v in head[3:]]
        prm = ref.MdpsParams(p=0.2, nseg=nseg, m_min=1, thr_override=thr)
        for fn in (ref.mdps_sample, ref.mdps_literal):
            idx, info = fn(line9(), n, prm)
            assert info.m == 1
            assert idx.tolist() == [int(v) for v in want], (head[0], fn.__name__)
            assert info.et_index == int(et[0])


# ------------------------------------------------------------------ estimator
def test_series_power_function_agrees_with_libm():
    # the fixed-order series is pinned to the library routine it replaces
    rng = np.random.Generator(np.random.PCG64(7))
    xs = [1, 2, 3, 5, 7, 8, 9, 10, 63, 64, 65, 1000, 65535, 65536, 10 ** 6, 2 ** 31 - 1]
    xs += rng.integers(1, 2 ** 31, 200).tolist()
    for x in xs:
        for e in (-1.5, -0.3, 0.0, 0.5, 2.0 / 3.0, 0.8586, 1.0, 1.2069, 2.0, 3.25):
            got = ref.pow_int_base(x, e)
            want = math.pow(float(x), e)
            assert abs(got - want) <= 2e-14 * want, (x, e, got, want)
    assert ref.pow_int_base(1, 0.77) == 1.0
    assert ref.pow_int_base(4, 1.0) == 4.0


@pytest.mark.parametrize("e", [1.0, 0.5, 0.75])
def test_estimator_recovers_exact_power_law(e):
    # If the measured prefix IS a power law a0/x^e, the predicted curve is that law.
    n, m, a0 = 4000, 400, 3.7
    i = np.arange(0, m + 1, dtype=np.float64)
    mdc = np.empty(m + 1, np.float32)
    mdc[0] = np.inf
    mdc[1:] = (a0 * i[1:] ** (-e)).astype(np.float32)
    for bias in (1.0, 1.25):
        prm = ref.MdpsParams(p=0.1, nseg=6, exponent=e, bias=bias, fit_window=32)
        thr = ref.mdps_thresholds(mdc, n, m, prm)
        b = np.array([min(max(n * l // 6, 1), n - 1) for l in range(1, 7)], np.float64)
        want = bias * bias * a0 * b ** (-e)
        # the prefix values carry one binary32 rounding each (2^-24 relative)
        assert np.allclose(thr, want, rtol=3e-7, atol=0)
        assert np.all(thr[:-1] >= thr[1:])


def test_level_scale_multiplies_the_predicted_squared_value():
    n, m, a0, e = 3000, 300, 2.0, 1.0
    mdc = np.empty(m + 1, np.float32)
    mdc[0] = np.inf
    mdc[1:] = (a0 / np.arange(1, m + 1)).astype(np.float32)
    scale = [1.0, 0.9, 0.8, 0.7, 0.6, 0.5]
    thr = ref.mdps_thresholds(mdc, n, m, ref.MdpsParams(exponent=e, bias=1.1, level_scale=scale))
    b = np.array([min(n * l // 6, n - 1) for l in range(1, 7)], np.float64)
    assert np.allclose(thr, 1.21 * np.array(scale) * a0 / b, rtol=3e-7)


def test_thresholds_inside_the_prefix_are_the_measured_values():
    # boundaries b_l <= m take the measured curve (the estimator call of Alg. 2: measured prefix and
    # estimate are concatenated)
    n, m = 120, 60
    mdc = np.empty(m + 1, np.float32)
    mdc[0] = np.inf
    mdc[1:] = (50.0 / np.arange(1, m + 1)).astype(np.float32)
    prm = ref.MdpsParams(p=0.5, nseg=6, exponent=1.0)
    thr = ref.mdps_thresholds(mdc, n, m, prm)
    assert thr[0] == mdc[20] and thr[1] == mdc[40] and thr[2] == mdc[60]
    assert np.allclose(thr[3:], 50.0 / np.array([80, 100, 119]), rtol=3e-7)


def test_threshold_clamps():
    n, m = 100, 10
    mdc = np.zeros(m + 1, np.float32)         # degenerate curve: all zero
    mdc[0] = np.inf
    thr = ref.mdps_thresholds(mdc, n, m, ref.MdpsParams(nseg=4, exponent=1.0))
    assert np.all(thr == FLT_MIN)
    # an increasing "prediction" (negative exponent) is flattened to non-increasing
    mdc[1:] = 1.0
    thr = ref.mdps_thresholds(mdc, n, m, ref.MdpsParams(nseg=4, exponent=-1.0))
    assert np.all(thr[:-1] >= thr[1:])


def test_prefix_length_rule():
    assert ref.mdps_prefix_len(ref.MdpsParams(p=0.1, m_min=8), 6000) == 600
    assert ref.mdps_prefix_len(ref.MdpsParams(p=0.1, m_min=8), 94) == 9
    assert ref.mdps_prefix_len(ref.MdpsParams(p=0.1, m_min=8), 50) == 8
    assert ref.mdps_prefix_len(ref.MdpsParams(p=0.25, m_min=1), 1023) == 255


# ------------------------------------------------------------------ two forms agree
CASES = [
    # seed, N, n, nseg, exponent, bias, generator
    (1, 400, 100, 6, 0.8, 1.0, "cube"),
    (2, 400, 100, 6, 0.8, 1.3, "cube"),      # over-estimate: early termination
    (3, 400, 100, 6, 0.8, 0.7, "cube"),      # under-estimate: quota-driven, no exhaustion
    (4, 600, 200, 3, 1.0, 1.1, "cube"),
    (5, 300, 150, 1, 0.7, 1.0, "cube"),
    (6, 500, 125, 16, 0.9, 1.05, "cube"),
    (7, 300, 100, 6, 0.8, 1.0, "lattice"),   # ties and duplicate points
    (8, 300, 100, 4, 0.8, 1.4, "lattice"),
]


def _cloud(kind, seed, N):
    return inputs.uniform_cube(seed, N) if kind == "cube" else inputs.lattice_with_ties(seed, N, 5)


@pytest.mark.parametrize("seed,N,n,nseg,e,bias,kind", CASES)
def test_running_form_equals_explicit_lists_and_bitmaps(seed, N, n, nseg, e, bias, kind):
    xyz = _cloud(kind, seed, N)
    prm = ref.MdpsParams(nseg=nseg, exponent=e, bias=bias)
    a, ia = ref.mdps_sample(xyz, n, prm, start=seed % N)
    b, ib = ref.mdps_literal(xyz, n, prm, start=seed % N)
    assert np.array_equal(a, b)
    assert ia.m == ib.m and ia.et_index == ib.et_index
    assert np.array_equal(ia.level_start, ib.level_start)
    assert np.array_equal(ia.level_exhausted, ib.level_exhausted)
    assert np.array_equal(ia.thr2, ib.thr2)


def test_case_list_exercises_both_endings():
    ends = set()
    for seed, N, n, nseg, e, bias, kind in CASES:
        _, info = ref.mdps_sample(_cloud(kind, seed, N), n, ref.MdpsParams(nseg=nseg, exponent=e, bias=bias),
                                  start=seed % N)
        ends.add(info.et_index < n)
    assert ends == {True, False}


# ------------------------------------------------------------------ special cases
@pytest.mark.parametrize("kind", ["cube", "lattice"])
def test_infinite_thresholds_reduce_to_exact_fps(kind):
    # nothing is ever available: every level exhausts at once, the rest is exact FPS
    xyz = _cloud(kind, 61, 350)
    prm = ref.MdpsParams(nseg=3, thr_override=[np.inf] * 3)
    idx, info = ref.mdps_sample(xyz, 120, prm)
    fps, _ = ref.fps_exact(xyz, 120)
    assert np.array_equal(idx, fps)
    assert info.et_index == info.m + 1


def test_tiny_threshold_scans_indices_in_order():
    # with R^2 = FLT_MIN every point that is not a duplicate of a sample is available,
    # so after the prefix the picks are the lowest unsampled indices in ascending order
    xyz = inputs.uniform_cube(62, 200)
    prm = ref.MdpsParams(nseg=1, thr_override=[float(FLT_MIN)])
    idx, info = ref.mdps_sample(xyz, 60, prm)
    m = info.m
    prefix = set(idx[:m + 1].tolist())
    want = [j for j in range(200) if j not in prefix][:60 - (m + 1)]
    assert idx[m + 1:].tolist() == want
    assert info.et_index == 60


def test_small_n_is_all_exact_fps():
    xyz = inputs.uniform_cube(63, 100)
    idx, info = ref.mdps_sample(xyz, 9, ref.MdpsParams())      # m = max(0, 8) = 8 = n-1
    fps, _ = ref.fps_exact(xyz, 9)
    assert np.array_equal(idx, fps)


# ------------------------------------------------------------------ invariants
def _levels_of_picks(info, n, nseg):
    """level (1-based) at which every threshold-phase sample index was picked"""
    lv = np.zeros(n, np.int32)
    starts = [int(s) for s in info.level_start]
    for i in range(info.m + 1, info.et_index):
        cur = 0
        for l in range(nseg):
            if starts[l] >= 0 and starts[l] <= i:
                cur = l + 1
        lv[i] = cur
    return lv


@pytest.mark.parametrize("name,b,n,e,bias", [("C1", 0, 1024, 0.86, 1.0), ("C1", 0, 1024, 0.86, 1.08),
                                              ("C2", 3, 512, 1.19, 1.04), ("C2", 5, 256, 1.19, 0.9)])
def test_prefix_spacing_coverage_and_tail_invariants(name, b, n, e, bias):
    xyz = inputs.make_cloud(name, b)
    N = xyz.shape[0]
    prm = ref.MdpsParams(exponent=e, bias=bias)
    idx, info = ref.mdps_sample(xyz, n, prm)
    fps, mdc = ref.fps_exact(xyz, n)
    D = d2_matrix(xyz)
    m = info.m
    # the prefix is exact FPS and its curve feeds the thresholds
    assert np.array_equal(idx[:m + 1], fps[:m + 1])
    assert np.array_equal(info.thr2, ref.mdps_thresholds(mdc, n, m, prm))
    # Section 4.1 step 3: inside segment l the spacing is at least R_l
    lv = _levels_of_picks(info, n, prm.nseg)
    for i in range(m + 1, info.et_index):
        assert lv[i] >= 1
        assert D[idx[i], idx[:i]].min() >= info.thr2[lv[i] - 1]
        # ... and it is the LOWEST index that satisfies it
        mind = D[idx[:i]].min(axis=0)
        assert idx[i] == int(np.flatnonzero(mind >= info.thr2[lv[i] - 1])[0])
    # a level that ran out left every point closer than R_l to some sample
    for l in range(prm.nseg):
        if info.level_exhausted[l]:
            upto = info.level_start[l + 1] if l + 1 < prm.nseg else info.et_index
            assert D[idx[:upto]].min(axis=0).max() < info.thr2[l]
    # Section 4.1 step 4: after the last level the rest is exact FPS from the true state
    for i in range(info.et_index, n):
        mind = D[idx[:i]].min(axis=0)
        assert idx[i] == int(np.flatnonzero(mind == mind.max())[0])


def test_calibrated_sampling_quality_is_close_to_fps():
    # Table 1 reports 98.4-99.5 % of the FPS spacing; a fitted exponent lands in that range
    xyz = inputs.make_cloud("C1", 0)
    idx, info = ref.mdps_sample(xyz, 1024, ref.MdpsParams(exponent=0.8586, bias=1.04))
    fps, _ = ref.fps_exact(xyz, 1024)
    assert info.level_exhausted[-1] == 1
    assert ref.coverage_radius(xyz, idx) <= 1.05 * ref.coverage_radius(xyz, fps)
    assert ref.mean_spacing(xyz, idx) >= 0.97 * ref.mean_spacing(xyz, fps)


# ------------------------------------------------------------------ scattered scan order
def test_scattered_order_hand_examples():
    for l in open(os.path.join(GOLDEN, "mdps_line9_scattered.txt")):
        if l.startswith("#") or not l.strip():
            continue
        head, want, et = [s.split() for s in l.split("|")]
        n, nseg = int(head[1]), int(head[2])
        thr = [float(v) for v in head[3:]]
        prm = ref.MdpsParams(p=0.2, nseg=nseg, m_min=1, thr_override=thr, scan_order=1)
        for fn in (ref.mdps_sample, ref.mdps_literal):
            idx, info = fn(line9(), n, prm)
            assert idx.tolist() == [int(v) for v in want], (head[0], fn.__name__)
            assert info.et_index == int(et[0])


def test_scan_stride_gives_a_walk_over_every_point():
    assert ref.scan_stride(9) == 5 and ref.scan_stride(1) == 1 and ref.scan_stride(2) == 1
    assert ref.scan_stride(10) == 7            # floor(6.18) = 6 shares the divisor 2 with 10
    for N in list(range(1, 200)) + [1024, 4096, 24000, 120000, 1000000, 999983, 2 ** 21]:
        A = ref.scan_stride(N)
        assert A >= max(1, math.floor(0.6180339887498949 * N)) and math.gcd(A, N) == 1
        assert A - math.floor(0.6180339887498949 * N) < 40          # the next coprime number is near
        if N <= 4096:
            walk = (np.arange(N, dtype=np.int64) * A) % N
            assert np.array_equal(np.sort(walk), np.arange(N))


@pytest.mark.parametrize("seed,N,n,nseg", [(3, 300, 120, 3), (4, 500, 200, 6), (5, 257, 257, 2)])
def test_scattered_order_pick_is_the_first_available_of_the_walk(seed, N, n, nseg):
    """Every sample of the threshold phase, recomputed from a distance matrix: it is available at the
    level in force (no earlier sample closer than R_l), and no point earlier in the walk is."""
    xyz = inputs.uniform_cube(seed, N)
    prm = ref.MdpsParams(nseg=nseg, exponent=0.8, bias=1.1, scan_order=1)
    idx, info = ref.mdps_sample(xyz, n, prm)
    D = d2_matrix(xyz)
    A = ref.scan_stride(N)
    walk = (np.arange(N, dtype=np.int64) * A) % N
    starts = [int(s) for s in info.level_start]
    for i in range(info.m + 1, info.et_index):
        level = max(l for l in range(nseg) if 0 <= starts[l] <= i)
        mind = D[:, idx[:i]].min(axis=1)
        avail = mind >= info.thr2[level]
        assert avail[idx[i]], "sample %d is not available" % i
        first = walk[np.flatnonzero(avail[walk])[0]]
        assert first == idx[i], "sample %d is not the first available point of the walk" % i
    assert len(set(idx.tolist())) == n or info.et_index < n


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_scattered_order_literal_form_agrees(seed):
    xyz = inputs.uniform_cube(seed, 400 + 37 * seed)
    for nseg, bias in ((1, 1.0), (4, 1.05), (6, 1.3)):
        prm = ref.MdpsParams(nseg=nseg, exponent=0.85, bias=bias, scan_order=1)
        a, ia = ref.mdps_sample(xyz, 150, prm)
        b, ib = ref.mdps_literal(xyz, 150, prm)
        assert np.array_equal(a, b) and ia.et_index == ib.et_index
        assert np.array_equal(ia.level_start, ib.level_start)
    # the order only matters in the threshold phase: thresholds no point meets give exact FPS
    prm = ref.MdpsParams(nseg=2, thr_override=[np.inf, np.inf], scan_order=1)
    assert np.array_equal(ref.mdps_sample(xyz, 150, prm)[0], ref.fps_exact(xyz, 150)[0])
    # ... and a different order gives different samples than the index order where it can
    p0 = ref.MdpsParams(nseg=4, exponent=0.85, bias=1.05)
    p1 = ref.MdpsParams(nseg=4, exponent=0.85, bias=1.05, scan_order=1)
    assert not np.array_equal(ref.mdps_sample(xyz, 150, p0)[0], ref.mdps_sample(xyz, 150, p1)[0])
