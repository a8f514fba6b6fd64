"""Seeded random shapes and parameters through every sampler entry point against the CPU oracle,
through the C ABI: sizes around the wave and workgroup boundaries, forced numbers of workgroups
per cloud, every number of segments, biases that end levels by quota or by exhaustion, clouds
with duplicates and equal distances.  Indices and level bookkeeping bit-exact."""
import sys

import numpy as np
import pytest

from oracle import ref
from paper_2507_23480_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fp():
    from paper_2507_23480_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load()
    binding.set_wg_per_cloud(0)
    yield binding
    binding.set_wg_per_cloud(0)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def make_cloud(rng, kind, N):
    if kind == 0:
        return rng.uniform(0, 1, (N, 3)).astype(np.float32)
    if kind == 1:                                         # clusters of very different density
        c = rng.uniform(-1, 1, (5, 3))
        w = rng.integers(0, 5, N)
        return (c[w] + rng.normal(0, 1, (N, 3)) * rng.uniform(0.002, 0.2, 5)[w, None]).astype(np.float32)
    if kind == 2:                                         # small integer lattice: ties and duplicates
        return rng.integers(0, 6, (N, 3)).astype(np.float32)
    pts = rng.uniform(0, 1, (N, 3)).astype(np.float32)    # sorted along x: index order follows space
    return pts[np.argsort(pts[:, 0], kind="stable")]


def case(seed):
    rng = np.random.Generator(np.random.PCG64(1000 + seed))
    N = int(rng.choice([1, 2, 63, 64, 65, 127, 129, 511, 513, 1023, 1025, 2047, 2500, 4097, 6000]))
    if seed % 3 == 0:
        N = int(rng.integers(1, 5000))
    n = int(rng.integers(1, N + 1)) if N < 200 or seed % 4 == 0 else int(rng.integers(1, max(2, N // 3)))
    B = int(rng.choice([1, 1, 2, 3]))
    G = int(rng.choice([0, 0, 1, 2, 3, 5])) if N >= 1500 else 0     # forced splits need points for every workgroup
    return rng, B, N, n, G


@pytest.mark.parametrize("seed", range(40))
def test_samplers_match_the_oracle(fp, seed):
    rng, B, N, n, G = case(seed)
    kind = seed % 4
    batch = np.stack([make_cloud(rng, kind, N) for _ in range(B)])
    starts = [int(rng.integers(0, N)) for _ in range(B)]
    nseg = int(rng.integers(1, 17))
    prm_kw = dict(p=float(rng.choice([0.05, 0.1, 0.2, 0.4])), nseg=nseg, exponent=float(rng.uniform(0.6, 1.4)),
                  bias=float(rng.choice([0.7, 0.9, 1.0, 1.05, 1.3])), m_min=int(rng.choice([1, 4, 8])),
                  fit_window=int(rng.choice([1, 8, 32, 64])))
    say("seed %d kind %d B %d N %d n %d G %d %s" % (seed, kind, B, N, n, G, prm_kw))
    prm, rprm = fp.MdpsParams(**prm_kw), ref.MdpsParams(**prm_kw)
    x = dev(batch)
    fp.set_wg_per_cloud(G)
    try:
        idx, mdc = fp.fps_exact(x, n, start_idx=starts, want_mdc=True)
        pidx, pmdc = fp.fps_exact_pruned(x, n, start_idx=starts, want_mdc=True)
        midx, minfo = fp.mdps_sample(x, n, prm, start_idx=starts, want_info=True)
        qidx, qinfo = fp.mdps_sample_pruned(x, n, prm, start_idx=starts, want_info=True)
        radius = float(rng.choice([0.05, 0.3, 2.0]))
        k = int(rng.choice([1, 7, 32, 100]))
        cache = fp.new_bq_cache(x, n)
        ridx = fp.mdps_sample(x, n, prm, start_idx=starts, bq_cache=cache, bq_radius=radius)
        cbq = fp.ball_query(x, ridx, radius, k, bq_cache=cache)
        bbq = fp.ball_query(x, ridx, radius, k)
        gbq = fp.ball_query_grid(x, ridx, radius, k)
        torch.cuda.synchronize()
    finally:
        fp.set_wg_per_cloud(0)
    assert torch.equal(pidx, idx) and torch.equal(pmdc, mdc)
    assert torch.equal(qidx, midx) and torch.equal(ridx, midx)
    for other in (cbq, gbq):
        assert torch.equal(other[0], bbq[0]) and torch.equal(other[1], bbq[1])
    mi, qi = fp.parse_info(minfo), fp.parse_info(qinfo)
    for b in range(B):
        want = ref.fps_exact(batch[b], n, starts[b])
        assert np.array_equal(idx[b].cpu().numpy(), want[0]) and np.array_equal(mdc[b].cpu().numpy(), want[1])
        widx, winfo = ref.mdps_sample(batch[b], n, rprm, starts[b])
        assert np.array_equal(midx[b].cpu().numpy(), widx), "mdps cloud %d" % b
        for gi in (mi[b], qi[b]):
            assert gi.status == 0 and gi.m == winfo.m and gi.et_index == winfo.et_index
            if gi.m < n - 1:
                assert np.array_equal(np.array(gi.thr2[:nseg], np.float32), winfo.thr2)
                assert list(gi.level_start[:nseg]) == winfo.level_start.tolist()
                assert list(gi.level_exhausted[:nseg]) == winfo.level_exhausted.tolist()
        wbq, wcnt = ref.ball_query(batch[b], widx, radius, k)
        assert np.array_equal(bbq[0][b].cpu().numpy(), wbq) and np.array_equal(bbq[1][b].cpu().numpy(), wcnt)
