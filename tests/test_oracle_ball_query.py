"""Pins for the oracle's ball query (Section 3.1 step 2; redundancy-free form Section 4.2).

Brute force IS the definition; the checks restate it with numpy binary32
arithmetic, plus a hand-worked example and the structural properties of the
output format (first k hits by index, strict <, padded with the first hit).
"""
import os

import numpy as np
import pytest

from oracle import ref
from paper_2507_23480_amd import inputs
from test_oracle_fps import d2_matrix, line9

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def check_ball_query(xyz, centers, radius, k, idx, cnt):
    D = d2_matrix(xyz)
    r2 = np.float32(radius) * np.float32(radius)
    for q, c in enumerate(centers):
        hits = np.flatnonzero(D[c] < r2)
        assert cnt[q] == min(len(hits), k)
        assert idx[q, :cnt[q]].tolist() == hits[:k].tolist()
        assert np.all(idx[q, cnt[q]:] == hits[0])
        assert c in hits


def test_line_example_matches_hand_derivation():
    for l in open(os.path.join(GOLDEN, "ball_line9.txt")):
        if l.startswith("#") or not l.strip():
            continue
        c, want, cnt = [s.split() for s in l.split("|")]
        idx, got = ref.ball_query(line9(), [int(c[0])], 2.5, 4)
        assert idx[0].tolist() == [int(v) for v in want]
        assert got[0] == int(cnt[0])


@pytest.mark.parametrize("seed,N,M,radius,k", [(1, 300, 300, 0.2, 8), (2, 500, 64, 0.35, 32),
                                               (3, 257, 100, 0.05, 4), (4, 128, 128, 2.0, 16)])
def test_matches_definition(seed, N, M, radius, k):
    xyz = inputs.uniform_cube(seed, N)
    centers = np.random.Generator(np.random.PCG64(seed)).integers(0, N, M).astype(np.int32)
    idx, cnt = ref.ball_query(xyz, centers, radius, k)
    check_ball_query(xyz, centers, radius, k, idx, cnt)


def test_boundary_is_strict():
    # neighbours at squared distance exactly r^2 are outside (Alg. 2 builds its lists with "<")
    pts = line9()
    idx, cnt = ref.ball_query(pts, [4], 2.0, 8)
    assert cnt[0] == 3 and idx[0, :3].tolist() == [3, 4, 5]


def test_duplicates_and_ties_keep_index_order():
    xyz = inputs.lattice_with_ties(5, 200, 3)
    centers = np.arange(0, 200, 7, dtype=np.int32)
    idx, cnt = ref.ball_query(xyz, centers, 1.5, 16)
    check_ball_query(xyz, centers, 1.5, 16, idx, cnt)


def test_bad_arguments():
    with pytest.raises(ValueError):
        ref.ball_query(line9(), [9], 1.0, 4)
    with pytest.raises(ValueError):
        ref.ball_query(line9(), [0], 0.0, 4)
    with pytest.raises(ValueError):
        ref.ball_query(line9(), [0], 1.0, 0)
