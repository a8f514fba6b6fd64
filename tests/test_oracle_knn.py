"""Pins for the oracle's k nearest samples (Section 3.1, feature propagation step 1; the
redundancy-free form of Section 4.2 must return the same result).

The definition is a sort of all n distances of a point; the checks restate it with numpy
(stable argsort on clouds whose distances are exact integers, so ties are decided by the
position alone), with scipy's k-d tree on clouds without ties, with a hand-worked
example, and through the sampler: the nearest-sample distance is the running minimum
exact FPS keeps.
"""
import os

import numpy as np
import pytest
from scipy.spatial import cKDTree

from oracle import ref
from paper_2507_23480_amd import inputs
from test_oracle_fps import line9

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def d2_to_samples(xyz, sidx):
    """binary32 ((dx*dx)+(dy*dy))+(dz*dz) of every point to every sample, [N][n]."""
    a = np.asarray(xyz, dtype=np.float32)
    s = a[np.asarray(sidx)]
    dx = a[:, None, 0] - s[None, :, 0]
    dy = a[:, None, 1] - s[None, :, 1]
    dz = a[:, None, 2] - s[None, :, 2]
    return (dx * dx + dy * dy) + dz * dz


def test_line_example_matches_hand_derivation():
    pos, d2 = ref.knn(line9(), [0, 8, 4, 2, 6], 3)
    for l in open(os.path.join(GOLDEN, "knn_line9.txt")):
        if l.startswith("#") or not l.strip():
            continue
        j, wp, wd = [s.split() for s in l.split("|")]
        assert pos[int(j[0])].tolist() == [int(v) for v in wp]
        assert d2[int(j[0])].tolist() == [float(v) for v in wd]


def test_line_example_uses_the_fps_order():
    # the sample list of the fixture is what Algorithm 1 returns on these points
    idx, _ = ref.fps_exact(line9(), 5)
    assert idx.tolist() == [0, 8, 4, 2, 6]


@pytest.mark.parametrize("seed,N,n,k", [(11, 400, 60, 3), (12, 333, 333, 8), (13, 200, 5, 5),
                                        (14, 150, 40, 1)])
def test_equals_stable_sort_on_lattice(seed, N, n, k):
    # integer coordinates: every squared distance is exact, many are equal
    xyz = inputs.lattice_with_ties(seed, N, 5)
    sidx = np.random.Generator(np.random.PCG64(seed)).integers(0, N, n).astype(np.int32)
    D = d2_to_samples(xyz, sidx)
    want = np.argsort(D, axis=1, kind="stable")[:, :k]
    pos, d2 = ref.knn(xyz, sidx, k)
    assert np.array_equal(pos, want)
    assert np.array_equal(d2, np.take_along_axis(D, want, axis=1))


@pytest.mark.parametrize("seed,N,n,k", [(21, 1000, 250, 3), (22, 700, 64, 6)])
def test_equals_kd_tree_without_ties(seed, N, n, k):
    xyz = inputs.uniform_cube(seed, N)
    sidx, _ = ref.fps_exact(xyz, n)
    dist, want = cKDTree(xyz[sidx].astype(np.float64)).query(xyz.astype(np.float64), k=k)
    pos, d2 = ref.knn(xyz, sidx, k)
    gaps = np.diff(dist, axis=1)
    clear = np.all(gaps > 1e-6, axis=1)             # rows whose order no rounding can change
    assert clear.mean() > 0.95
    assert np.array_equal(pos[clear], want.reshape(N, k)[clear])
    assert np.allclose(np.sqrt(d2.astype(np.float64)), dist.reshape(N, k), rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("seed,N,n,k", [(31, 500, 100, 3), (32, 257, 33, 4)])
def test_definition_properties(seed, N, n, k):
    xyz = inputs.uniform_cube(seed, N)
    sidx = np.random.Generator(np.random.PCG64(seed)).permutation(N)[:n].astype(np.int32)
    D = d2_to_samples(xyz, sidx)
    pos, d2 = ref.knn(xyz, sidx, k)
    for j in range(N):
        assert len(set(pos[j].tolist())) == k
        assert np.array_equal(d2[j], D[j, pos[j]])
        key = list(zip(d2[j].tolist(), pos[j].tolist()))
        assert key == sorted(key)                                   # nearest first, then position
        rest = np.delete(D[j], pos[j])
        rest_q = np.delete(np.arange(n), pos[j])
        worst = (d2[j, -1], pos[j, -1])
        assert all((dv, qv) > worst for dv, qv in zip(rest.tolist(), rest_q.tolist()))


def test_a_sample_finds_itself_first_and_duplicates_keep_position_order():
    xyz = inputs.uniform_cube(41, 120)
    sidx = np.array([7, 30, 7, 99, 30], dtype=np.int32)           # repeated samples
    pos, d2 = ref.knn(xyz, sidx, 3)
    assert pos[7, :2].tolist() == [0, 2] and d2[7, 0] == 0.0 and d2[7, 1] == 0.0
    assert pos[30, :2].tolist() == [1, 4]
    assert pos[99, 0] == 3 and d2[99, 0] == 0.0


def test_nearest_sample_distance_is_the_running_minimum_of_fps():
    # after n picks of Algorithm 1 the distance array holds min_q dist2(P_j, S_q): the next
    # pick's value is its maximum, which the 1-NN distances must reproduce
    xyz = inputs.uniform_cube(51, 600)
    n = 80
    idx, mdc = ref.fps_exact(xyz, n + 1)
    _, d2 = ref.knn(xyz, idx[:n], 1)
    assert d2[:, 0].max() == mdc[n]
    assert int(np.argmax(d2[:, 0])) == int(idx[n])
    assert abs(np.sqrt(float(d2[:, 0].max())) - ref.coverage_radius(xyz, idx[:n])) < 1e-6


def test_point_subset_is_the_rows_of_the_full_result():
    xyz = inputs.uniform_cube(71, 300)
    sidx, _ = ref.fps_exact(xyz, 50)
    pos, d2 = ref.knn(xyz, sidx, 4)
    pts = np.array([299, 0, 17, 17, 123])
    spos, sd2 = ref.knn(xyz, sidx, 4, points=pts)
    assert np.array_equal(spos, pos[pts]) and np.array_equal(sd2, d2[pts])


def test_rejects_bad_arguments():
    xyz = inputs.uniform_cube(61, 50)
    with pytest.raises(ValueError):
        ref.knn(xyz, [1, 2], 3)                # k > n
    with pytest.raises(ValueError):
        ref.knn(xyz, [1, 50, 3], 2)            # sample index out of range
