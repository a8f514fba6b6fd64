"""Pins for the oracle's exclusion lists (the list-building loops of Alg. 2, Section 4.1 step 2; the extra
list at the ball-query radius, Section 4.2) and the ball query by lookup in them.

The lists are a plain definition; the pins are a hand-worked example, a restatement with a
numpy binary32 distance matrix, structure that the definition forces (symmetry, nesting,
self-membership, row sizes), a k-d tree on integer lattices (where binary32 distances are
exact) and the already pinned brute-force ball query.
"""
import os

import numpy as np
import pytest
from scipy.spatial import cKDTree

from oracle import ref
from paper_2507_23480_amd import inputs
from test_oracle_fps import d2_matrix, line9

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rows(off, ent, N, L):
    return [[ent[off[l * N + i]:off[l * N + i + 1]].tolist() for i in range(N)] for l in range(L)]


def test_line_example_matches_hand_derivation():
    off, ent = ref.excl_lists(line9(), [10.0, 2.0, 6.25])
    got = rows(off, ent, 9, 3)
    seen = 0
    for l in open(os.path.join(GOLDEN, "excl_line9.txt")):
        if l.startswith("#") or not l.strip():
            continue
        lev, pt, members = [s.split() for s in l.split("|")]
        assert got[int(lev[0])][int(pt[0])] == [int(v) for v in members]
        seen += 1
    assert seen == 9
    # total members: sum over i of #{j: |i-j| <= w}, w = 3, 1, 2
    assert off[-1] == (9 * 7 - 12) + (9 * 3 - 2) + (9 * 5 - 6)


@pytest.mark.parametrize("seed,N,thr", [(1, 200, [0.09, 0.04, 0.01]), (2, 333, [0.02, 0.3]),
                                        (3, 64, [1e-12]), (4, 129, [4.0, 0.0625, 0.0625])])
def test_matches_definition(seed, N, thr):
    xyz = inputs.uniform_cube(seed, N)
    off, ent = ref.excl_lists(xyz, thr)
    D = d2_matrix(xyz)
    got = rows(off, ent, N, len(thr))
    for l, t in enumerate(thr):
        for i in range(N):
            assert got[l][i] == np.flatnonzero(D[i] < np.float32(t)).tolist()


def test_structure_forced_by_the_definition():
    xyz = inputs.uniform_cube(7, 300)
    thr = [0.08, 0.03, 0.05, 0.002]
    off, ent = ref.excl_lists(xyz, thr)
    got = rows(off, ent, 300, 4)
    order = np.argsort(thr)[::-1]                       # levels by decreasing radius
    for l in range(4):
        member = [set(r) for r in got[l]]
        for i in range(300):
            assert i in member[i]                        # dist2(i, i) = 0 < thr
            assert got[l][i] == sorted(got[l][i])        # the loop over j appends in ascending order
            for j in got[l][i]:
                assert i in member[j]                    # the distance is symmetric bit for bit
    for a, b in zip(order[:-1], order[1:]):              # a smaller radius gives a sub-list
        for i in range(300):
            assert set(got[b][i]) <= set(got[a][i])
    assert np.all(np.diff(off) >= 0) and off[0] == 0 and off[-1] == len(ent)


def test_lattice_against_kd_tree():
    # integer coordinates: squared distances are exact in binary32, so a radius strictly
    # between two attainable values leaves no rounding question for the k-d tree either
    xyz = inputs.lattice_with_ties(11, 400, 4)
    thr = [2.5, 0.5, 5.5]
    off, ent = ref.excl_lists(xyz, thr)
    got = rows(off, ent, 400, 3)
    tree = cKDTree(xyz.astype(np.float64))
    for l, t in enumerate(thr):
        want = tree.query_ball_point(xyz.astype(np.float64), np.sqrt(t))
        for i in range(400):
            assert got[l][i] == sorted(want[i])


def test_zero_and_negative_radius_give_empty_rows():
    off, ent = ref.excl_lists(line9(), [0.0, -1.0])
    assert off[-1] == 0 and len(ent) == 0


@pytest.mark.parametrize("k", [1, 4, 32])
def test_lookup_equals_brute_force_ball_query(k):
    xyz = inputs.uniform_cube(5, 500)
    radius = 0.17
    r2 = np.float32(radius) * np.float32(radius)
    off, ent = ref.excl_lists(xyz, [0.5, r2])
    centers = np.random.Generator(np.random.PCG64(3)).integers(0, 500, 200).astype(np.int32)
    idx, cnt = ref.ball_query_lists(off, ent, 500, 1, centers, k)
    bidx, bcnt = ref.ball_query(xyz, centers, radius, k)
    assert np.array_equal(idx, bidx) and np.array_equal(cnt, bcnt)


def test_lookup_of_an_empty_row():
    off, ent = ref.excl_lists(line9(), [0.0])
    idx, cnt = ref.ball_query_lists(off, ent, 9, 0, [3], 4)
    assert idx.tolist() == [[-1, -1, -1, -1]] and cnt.tolist() == [0]
