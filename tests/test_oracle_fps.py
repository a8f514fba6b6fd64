"""Pins for the oracle's exact farthest point sampling (Algorithm 1, Section 3.3).

The checks restate the DEFINITION of each pick (it maximises the minimum distance
to the already selected set, lowest index among equals) from scratch with numpy
binary32 arithmetic, plus a hand-worked example, invariants and special cases.
"""
import os

import numpy as np
import pytest

from oracle import ref
from paper_2507_23480_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def d2_matrix(xyz):
    """All-pairs squared distances, binary32, ((dx*dx)+(dy*dy))+(dz*dz)."""
    a = xyz.astype(np.float32)
    dx = a[:, None, 0] - a[None, :, 0]
    dy = a[:, None, 1] - a[None, :, 1]
    dz = a[:, None, 2] - a[None, :, 2]
    t = dx * dx
    t = t + dy * dy
    t = t + dz * dz
    assert t.dtype == np.float32
    return t


def check_fps_definition(xyz, idx, mdc, start):
    """Every pick attains max_j min_{s<i} d2(P[s],P[j]) and is the lowest such index."""
    D = d2_matrix(xyz)
    assert idx[0] == start and np.isinf(mdc[0])
    for i in range(1, len(idx)):
        mind = D[idx[:i]].min(axis=0)          # recomputed from scratch each time
        best = mind.max()
        assert mind[idx[i]] == best, "pick %d does not attain the maximum" % i
        assert idx[i] == int(np.flatnonzero(mind == best)[0]), "pick %d is not the lowest index" % i
        assert mdc[i] == best


def line9():
    pts = np.zeros((9, 3), np.float32)
    pts[:, 0] = np.arange(9)
    return pts


def test_line_example_matches_hand_derivation():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "fps_line9.txt")) if not l.startswith("#")]
    want_idx = np.array([int(r[1]) for r in rows], np.int32)
    want_mdc = np.array([float(r[2]) for r in rows], np.float32)
    idx, mdc = ref.fps_exact(line9(), 9)
    assert np.array_equal(idx, want_idx)
    assert np.array_equal(mdc, want_mdc)


@pytest.mark.parametrize("seed,N,n,start", [(1, 64, 64, 0), (2, 257, 100, 5), (3, 512, 128, 511),
                                            (4, 300, 300, 17)])
def test_picks_match_definition_on_random_clouds(seed, N, n, start):
    xyz = inputs.uniform_cube(seed, N)
    idx, mdc = ref.fps_exact(xyz, n, start)
    check_fps_definition(xyz, idx, mdc, start)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_ties_and_duplicates_take_lowest_index(seed):
    xyz = inputs.lattice_with_ties(seed, 200, cells=4)     # many equal distances, duplicate points
    idx, mdc = ref.fps_exact(xyz, 120, 3)
    check_fps_definition(xyz, idx, mdc, 3)


def test_curve_is_non_increasing():
    # Section 4: the maximised minimum distance decreases as sampling proceeds
    for name in ("C1", "C2"):
        xyz = inputs.make_cloud(name, 0)
        _, mdc = ref.fps_exact(xyz, xyz.shape[0] // 2)
        assert np.all(mdc[1:-1] >= mdc[2:])


def test_full_sampling_is_a_permutation_of_distinct_points():
    xyz = inputs.uniform_cube(21, 333)
    idx, mdc = ref.fps_exact(xyz, 333, 7)
    assert sorted(idx.tolist()) == list(range(333))
    assert np.all(mdc[1:] > 0)


def test_all_points_identical_repeats_index_zero():
    xyz = np.ones((10, 3), np.float32)
    idx, mdc = ref.fps_exact(xyz, 5, 4)
    # every distance is 0: the argmax of an all-zero array is index 0
    assert idx.tolist() == [4, 0, 0, 0, 0]
    assert mdc[1:].tolist() == [0.0] * 4


def test_relabelling_points_relabels_the_picks():
    # generic points have no ties, so the picks do not depend on the labelling
    xyz = inputs.uniform_cube(31, 400)
    perm = np.random.Generator(np.random.PCG64(99)).permutation(400)
    idx, mdc = ref.fps_exact(xyz, 100, 0)
    inv = np.empty(400, np.int64)
    inv[perm] = np.arange(400)
    idx_p, mdc_p = ref.fps_exact(xyz[perm], 100, int(inv[0]))
    assert np.array_equal(perm[idx_p], idx)
    assert np.array_equal(mdc_p, mdc)


def test_prefix_property():
    xyz = inputs.uniform_cube(41, 500)
    a, _ = ref.fps_exact(xyz, 200)
    b, _ = ref.fps_exact(xyz, 50)
    assert np.array_equal(a[:50], b)


def test_single_sample_and_bad_arguments():
    xyz = inputs.uniform_cube(51, 10)
    idx, mdc = ref.fps_exact(xyz, 1, 9)
    assert idx.tolist() == [9]
    with pytest.raises(ValueError):
        ref.fps_exact(xyz, 11)
    with pytest.raises(ValueError):
        ref.fps_exact(xyz, 5, 10)


def test_gather_and_quality_metrics_closed_forms():
    pts = line9()
    g = ref.gather_xyz(pts, np.array([8, 0, 4], np.int32))
    assert g[:, 0].tolist() == [8.0, 0.0, 4.0]
    # samples {0,8}: the farthest point from its nearest sample is j=4 at distance 4
    assert ref.coverage_radius(pts, np.array([0, 8], np.int32)) == 4.0
    # samples {0,4,8}: nearest other sample at 4 for each; coverage 2 (points 2 and 6)
    assert ref.mean_spacing(pts, np.array([0, 4, 8], np.int32)) == 4.0
    assert ref.coverage_radius(pts, np.array([0, 4, 8], np.int32)) == 2.0
    # samples {0,1,8}: spacings 1,1,7
    assert ref.mean_spacing(pts, np.array([0, 1, 8], np.int32)) == 3.0
