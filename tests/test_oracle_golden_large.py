"""The stored oracle results of the two large workloads (tests/golden/c4_full.npz, c5_full.npz)
are what the oracle, as it stands, computes: one C4 cloud is recomputed in full and the start of
the C5 run is recomputed, and the invariants of Algorithm 1 / Algorithm 2 that hold at any size
are checked on all of it (a curve that never rises, distinct samples, the MDPS run starting with
the exact-FPS samples, the recorded distance of sampled picks recomputed from the coordinates)."""
import json
import os

import numpy as np
import pytest

from oracle import ref
from paper_2507_23480_amd import inputs

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load(name):
    with np.load(os.path.join(GOLDEN, name.lower() + "_full.npz")) as z:
        return {k: z[k] for k in z.files}


def params(gold, v):
    return ref.MdpsParams(**json.loads(str(gold["params_" + v])))


@pytest.mark.parametrize("name", ["C4", "C5"])
def test_invariants_of_the_stored_results(name):
    wl = inputs.WORKLOADS[name]
    n = wl.stages[0].n
    gold = load(name)
    batch = inputs.make_batch(name)
    rng = np.random.Generator(np.random.PCG64(11))
    for b in range(wl.B):
        idx, mdc = gold["fps_idx"][b], gold["fps_mdc"][b]
        assert idx.shape == (n,) and idx[0] == 0 and np.isinf(mdc[0])
        assert len(np.unique(idx)) == n and idx.min() >= 0 and idx.max() < wl.N
        assert np.all(mdc[1:-1] >= mdc[2:])
        pts = batch[b].astype(np.float32)
        for i in rng.integers(1, n, 24):
            d = pts[idx[i]] - pts[idx[:i]]
            t = d[:, 0] * d[:, 0]
            t = t + d[:, 1] * d[:, 1]
            t = t + d[:, 2] * d[:, 2]
            assert mdc[i] == t.min()
        for v in [k[len("params_"):] for k in gold if k.startswith("params_")]:
            midx, m = gold["mdps_idx_" + v][b], int(gold["m_" + v][b])
            assert len(np.unique(midx)) == n
            assert np.array_equal(midx[:m + 1], idx[:m + 1])
            thr = gold["thr2_" + v][b]
            assert np.all(thr[:-1] >= thr[1:]) and np.all(thr > 0)


def test_one_lidar_cloud_recomputed_in_full():
    gold = load("C4")
    n = inputs.WORKLOADS["C4"].stages[0].n
    cloud = inputs.make_cloud("C4", 3)
    midx, info = ref.mdps_sample(cloud, n, params(gold, "calibrated"))
    assert np.array_equal(midx, gold["mdps_idx_calibrated"][3])
    assert info.et_index == gold["et_index_calibrated"][3] and info.m == gold["m_calibrated"][3]
    assert np.array_equal(info.thr2, gold["thr2_calibrated"][3])
    assert np.array_equal(info.level_start, gold["level_start_calibrated"][3])


def test_start_of_the_million_point_run_recomputed():
    gold = load("C5")
    cloud = inputs.make_cloud("C5", 0)
    idx, mdc = ref.fps_exact(cloud, 200)
    assert np.array_equal(idx, gold["fps_idx"][0, :200]) and np.array_equal(mdc, gold["fps_mdc"][0, :200])
