"""GPU parity of MDPS with the MLP curve estimator (Appendix A.3) against the CPU oracle,
through the C ABI: the binary32 thresholds bit for bit (binary64 network arithmetic in the same
fixed order on both sides), and with them the indices and the bookkeeping."""
import sys

import numpy as np
import pytest

from oracle import ref
from paper_2507_23480_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

SIZES = [(32, 128), (128,), (128, 128), (128,), (128, 64), (64,)]


@pytest.fixture(scope="module")
def fp():
    from paper_2507_23480_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load()
    binding.set_wg_per_cloud(0)
    yield binding
    binding.set_wg_per_cloud(0)


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def random_weights(seed, scale=0.05, fall=1.5):
    rng = np.random.Generator(np.random.PCG64(seed))
    parts = [rng.normal(0, scale, s).astype(np.float32) for s in SIZES]
    parts[5][:] = (-np.linspace(0.05, fall, 64) + rng.normal(0, 0.02, 64)).astype(np.float32)
    return np.concatenate([p.reshape(-1) for p in parts])


def check(fp, batch, n, w, G=0, nseg=6, bias=1.05, p=0.1, m_min=8, scale=None):
    fp.set_wg_per_cloud(G)
    try:
        wd = torch.from_numpy(w).cuda()
        prm = fp.MdpsParams(p=p, nseg=nseg, bias=bias, m_min=m_min, level_scale=scale, mlp=wd)
        rp = ref.MdpsParams(p=p, nseg=nseg, bias=bias, m_min=m_min, level_scale=scale, mlp=w)
        idx, info = fp.mdps_sample(torch.from_numpy(np.ascontiguousarray(batch)).cuda(), n, prm, want_info=True)
        torch.cuda.synchronize()
        idx = idx.cpu().numpy()
        infos = fp.parse_info(info)
        for b in range(batch.shape[0]):
            widx, winfo = ref.mdps_sample(batch[b], n, rp)
            gi = infos[b]
            assert gi.status == 0
            assert np.array_equal(np.array(gi.thr2[:nseg], dtype=np.float32), winfo.thr2[:nseg]), "thresholds %d" % b
            assert np.array_equal(idx[b], widx), "indices cloud %d" % b
            assert gi.m == winfo.m and gi.et_index == winfo.et_index
    finally:
        fp.set_wg_per_cloud(0)


@pytest.mark.parametrize("N,n", [(300, 94), (1024, 512), (2049, 700), (6000, 1500), (9000, 3000)])
def test_random_networks(fp, N, n):
    say("mlp estimator N=%d n=%d" % (N, n))
    check(fp, inputs.uniform_cube(400 + N, N)[None], n, random_weights(N))


def test_batch_and_several_workgroups(fp):
    batch = np.stack([inputs.uniform_cube(10 + b, 5000) for b in range(3)])
    for G in (1, 3, 8):
        check(fp, batch, 1200, random_weights(G), G=G)


def test_wild_networks_still_agree(fp):
    # large weights: outputs far outside any sensible range, clamps and the monotone rule at work
    cloud = inputs.uniform_cube(5, 2000)[None]
    check(fp, cloud, 500, random_weights(1, scale=3.0, fall=400.0))
    check(fp, cloud, 500, random_weights(2, scale=1.0, fall=-50.0))       # a "rising" prediction
    w = random_weights(3)
    w[:] = 0.0                                                            # curve stays at mdc[m]
    check(fp, cloud, 500, w)


def test_short_prefix_repeats_inputs(fp):
    # m < 32: several of the 32 inputs read the same curve position
    check(fp, inputs.uniform_cube(8, 700)[None], 90, random_weights(4), nseg=4)
    check(fp, inputs.uniform_cube(9, 700)[None], 120, random_weights(5), p=0.3, m_min=3, nseg=5)


def test_level_scale_and_bias_apply(fp):
    check(fp, inputs.uniform_cube(6, 3000)[None], 800, random_weights(6), bias=1.2,
          scale=[1.0, 1.1, 0.9, 1.05, 1.0, 0.95])


def test_duplicates(fp):
    check(fp, inputs.lattice_with_ties(3, 1500, 4)[None], 600, random_weights(7))


COVERAGE_BOUND = 1.05


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_trained_estimators_at_the_workloads_match_the_oracle(fp, name):
    """Every stage, every cloud, with the committed weights: parity element by element and
    the sampling-quality bound."""
    from concurrent.futures import ThreadPoolExecutor
    from paper_2507_23480_amd import mlp_estimator
    say("trained mlp estimator at workload", name)
    wl = inputs.WORKLOADS[name]
    batch = inputs.make_batch(name)
    x = torch.from_numpy(batch).cuda()
    host = [batch[b] for b in range(wl.B)]
    for s, st in enumerate(wl.stages):
        prm = mlp_estimator.params_for(name, s)
        w = mlp_estimator.weights()["%s/%d" % (name, s)]
        rp = ref.MdpsParams(p=prm.p, nseg=prm.nseg, bias=prm.bias, m_min=prm.m_min, mlp=w)
        idx, info = fp.mdps_sample(x, st.n, prm, want_info=True)
        fidx = fp.fps_exact(x, st.n)
        ratio = (fp.coverage2(x, idx).sqrt() / fp.coverage2(x, fidx).sqrt())
        torch.cuda.synchronize()
        assert float(ratio.max()) <= COVERAGE_BOUND, "coverage ratio %.4f" % float(ratio.max())
        infos = fp.parse_info(info)
        with ThreadPoolExecutor(max_workers=8) as ex:
            want = list(ex.map(lambda c: ref.mdps_sample(c, st.n, rp), host))
        got = idx.cpu().numpy()
        for b in range(wl.B):
            assert np.array_equal(got[b], want[b][0]), "stage %d cloud %d" % (s, b)
            assert np.array_equal(np.array(infos[b].thr2[:prm.nseg], dtype=np.float32), want[b][1].thr2[:prm.nseg])
        if s + 1 < len(wl.stages):
            host = [ref.gather_xyz(host[b], ref.fps_exact(host[b], st.n)[0]) for b in range(wl.B)]
            x = fp.gather_xyz(x, fidx).contiguous()


@pytest.mark.parametrize("name", ["C4", "C5"])
def test_trained_estimators_at_the_large_workloads(fp, name):
    """Full size: thresholds bit for bit against the oracle's estimator fed with the curve of
    the prefix (which the exact-FPS tests pin), the spacing bound of every level on sampled
    picks, and the sampling-quality bound."""
    from paper_2507_23480_amd import mlp_estimator
    say("trained mlp estimator at workload", name)
    wl = inputs.WORKLOADS[name]
    st = wl.stages[0]
    batch = inputs.make_batch(name)
    x = torch.from_numpy(batch).cuda()
    prm = mlp_estimator.params_for(name, 0)
    w = mlp_estimator.weights()["%s/0" % name]
    rp = ref.MdpsParams(p=prm.p, nseg=prm.nseg, bias=prm.bias, m_min=prm.m_min, mlp=w)
    idx, info = fp.mdps_sample(x, st.n, prm, want_info=True)
    fidx, mdc = fp.fps_exact(x, st.n, want_mdc=True)
    ratio = (fp.coverage2(x, idx).sqrt() / fp.coverage2(x, fidx).sqrt())
    torch.cuda.synchronize()
    assert float(ratio.max()) <= COVERAGE_BOUND
    infos = fp.parse_info(info)
    got = idx.cpu().numpy()
    curve = mdc.cpu().numpy()
    rng = np.random.Generator(np.random.PCG64(1))
    for b in range(wl.B):
        gi = infos[b]
        thr = ref.mdps_thresholds(curve[b], st.n, gi.m, rp)
        assert np.array_equal(np.array(gi.thr2[:prm.nseg], dtype=np.float32), thr)
        assert np.array_equal(got[b, :gi.m + 1], fidx[b, :gi.m + 1].cpu().numpy())
        assert len(np.unique(got[b])) == st.n
        # a pick of level l keeps at least R_l to every earlier sample (Section 4.1 step 3)
        starts = [v for v in gi.level_start[:prm.nseg]]
        for pos in rng.integers(gi.m + 1, gi.et_index, 12):
            lvl = max(l for l in range(prm.nseg) if 0 <= starts[l] <= pos)
            p = batch[b, got[b, pos]].astype(np.float32)
            q = batch[b, got[b, :pos]].astype(np.float32)
            d = (p - q)
            d2 = (d[:, 0] * d[:, 0] + d[:, 1] * d[:, 1]) + d[:, 2] * d[:, 2]
            assert d2.min() >= gi.thr2[lvl]
