"""GPU parity of MDPS with pruned distance updates (fp_mdps_sample_pruned) against the CPU oracle
of Algorithm 2, through the C ABI: indices, thresholds and level bookkeeping bit-exact.  The
pruned sampler holds the cloud in cell order and finds "the lowest available index" through a
window of indices, so the cases stress what depends on that: clouds whose index order follows
space and clouds where it does not, equal distances, windows that come up empty or too full,
levels that end by quota and by exhaustion, several workgroups per cloud.  Every case runs with both
scan orders of the threshold phase: the lowest available index, and the first available point of the
scattered walk (there the windows run over a point's place in the walk instead of its index)."""
import dataclasses
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


@pytest.fixture(params=[0, 1], ids=["index_order", "scattered_order"])
def order(request):
    return request.param


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def rparams(prm):
    return ref.MdpsParams(p=prm.p, nseg=prm.nseg, exponent=prm.exponent, bias=prm.bias,
                          fit_window=prm.fit_window, m_min=prm.m_min, thr_override=prm.thr_override,
                          level_scale=prm.level_scale, scan_order=prm.scan_order)


def check(fp, batch, n, prm, start=None, G=0, order=0):
    prm = dataclasses.replace(prm, scan_order=order)
    fp.set_wg_per_cloud(G)
    try:
        B = batch.shape[0]
        starts = [0] * B if start is None else list(start)
        idx, info = fp.mdps_sample_pruned(dev(batch), n, prm, start_idx=None if start is None else starts,
                                          want_info=True)
        torch.cuda.synchronize()
        idx = idx.cpu().numpy()
        infos = fp.parse_info(info)
        rp = rparams(prm)
        for b in range(B):
            widx, winfo = ref.mdps_sample(batch[b], n, rp, starts[b])
            gi = infos[b]
            assert gi.status == 0
            assert np.array_equal(np.array(gi.thr2[:prm.nseg], np.float32), winfo.thr2) or gi.m >= n - 1, \
                "thresholds cloud %d" % b
            assert np.array_equal(idx[b], widx), "idx cloud %d" % b
            assert gi.m == winfo.m and gi.et_index == winfo.et_index
            if gi.m < n - 1:
                assert list(gi.level_start[:prm.nseg]) == winfo.level_start.tolist()
                assert list(gi.level_exhausted[:prm.nseg]) == winfo.level_exhausted.tolist()
    finally:
        fp.set_wg_per_cloud(0)


def test_line_examples_and_overrides(fp, order):
    line = np.zeros((1, 9, 3), np.float32)
    line[0, :, 0] = np.arange(9)
    check(fp, line, 5, fp.MdpsParams(p=0.2, nseg=1, m_min=1, thr_override=[3.0]), order=order)
    check(fp, line, 5, fp.MdpsParams(p=0.2, nseg=1, m_min=1, thr_override=[4.0]), order=order)
    check(fp, line, 6, fp.MdpsParams(p=0.2, nseg=2, m_min=1, thr_override=[10.0, 2.0]), order=order)


@pytest.mark.parametrize("N,n,G,nseg,e,bias", [
    (400, 100, 0, 6, 0.8, 1.0), (400, 100, 0, 6, 0.8, 1.3), (400, 100, 0, 6, 0.8, 0.7),
    (4096, 1024, 0, 6, 0.8586, 1.04), (4096, 1024, 0, 1, 0.8586, 1.0), (4096, 1024, 0, 16, 0.8586, 1.1),
    (4097, 700, 0, 6, 0.8, 1.0), (9000, 2000, 2, 6, 0.8, 1.05), (9000, 2000, 3, 6, 0.8, 0.9),
    (20000, 5000, 0, 6, 0.8, 1.04), (20000, 5000, 7, 4, 0.8, 1.2), (300, 9, 0, 6, 1.0, 1.0)])
def test_uniform_cube(fp, order, N, n, G, nseg, e, bias):
    say("pruned mdps order=%d N=%d n=%d G=%d nseg=%d e=%g bias=%g" % (order, N, n, G, nseg, e, bias))
    batch = inputs.uniform_cube(200 + N, N)[None]
    check(fp, batch, n, fp.MdpsParams(nseg=nseg, exponent=e, bias=bias), G=G, order=order)


def test_index_order_follows_space(fp, order):
    # points sorted along x: a window of indices is a slab of space, so windows come up
    # full near unsampled slabs and empty elsewhere
    say("pruned mdps, cloud sorted along x")
    cloud = inputs.uniform_cube(71, 6000)
    cloud = cloud[np.argsort(cloud[:, 0], kind="stable")]
    check(fp, cloud[None], 1500, fp.MdpsParams(exponent=0.8, bias=1.04), order=order)
    check(fp, cloud[None], 1500, fp.MdpsParams(exponent=0.8, bias=1.04), start=[5999], G=4, order=order)


def test_equal_distances_and_duplicates(fp, order):
    lat = inputs.lattice_with_ties(7, 600, 5)[None]
    check(fp, lat, 200, fp.MdpsParams(exponent=0.8, bias=1.0), start=[5], order=order)
    check(fp, lat, 200, fp.MdpsParams(nseg=3, thr_override=[float("inf")] * 3), order=order)   # == exact FPS
    check(fp, lat, 200, fp.MdpsParams(nseg=1, thr_override=[1.17549435e-38]), order=order)      # everything stays available
    batch = np.stack([inputs.lattice_with_ties(20 + b, 1500, 5) for b in range(3)])
    check(fp, batch, 500, fp.MdpsParams(exponent=0.8, bias=1.0), G=2, order=order)


def test_clustered_cloud(fp, order):
    # dense clusters and a sparse background: availability per index window varies widely
    rng = np.random.Generator(np.random.PCG64(77))
    parts = [rng.normal(c, 0.01, (1500, 3)) for c in rng.uniform(-1, 1, (4, 3))]
    parts.append(rng.uniform(-1, 1, (2000, 3)))
    cloud = np.concatenate(parts).astype(np.float32)          # index order: cluster by cluster
    check(fp, cloud[None], 2000, fp.MdpsParams(exponent=0.8, bias=1.04), order=order)
    check(fp, cloud[rng.permutation(cloud.shape[0])][None], 2000, fp.MdpsParams(exponent=0.8, bias=1.04), G=3, order=order)


def test_batches_and_start_indices(fp, order):
    say("pruned mdps C2 batch")
    batch = inputs.make_batch("C2")
    check(fp, batch, 512, fp.MdpsParams(exponent=1.2069, bias=1.1), order=order)
    check(fp, batch, 512, fp.MdpsParams(exponent=1.2069, bias=1.0), start=[(91 * b) % 1024 for b in range(16)], order=order)


def test_mlp_estimator(fp):
    from paper_2507_23480_amd import mlp_estimator
    x = inputs.make_batch("C1")
    prm = mlp_estimator.params_for("C1", 0)
    a = fp.mdps_sample(dev(x), 1024, prm)
    b = fp.mdps_sample_pruned(dev(x), 1024, prm)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_argument_checks(fp):
    lib = fp.load()
    x = dev(inputs.uniform_cube(3, 300)[None])
    out = torch.empty((1, 10), dtype=torch.int32, device="cuda")
    ws = torch.empty(lib.fp_fps_pruned_workspace_bytes(1, 300), dtype=torch.uint8, device="cuda")
    import ctypes
    c = fp.MdpsParams().to_c()
    call = lambda xp, n, p, wsb: lib.fp_mdps_sample_pruned(xp, 1, 300, n, None, p, out.data_ptr(), None,
                                                            None, 0, 0.0, ws.data_ptr(), wsb, None)
    assert call(x.data_ptr(), 10, None, ws.numel()) == -1
    assert call(None, 10, ctypes.byref(c), ws.numel()) == -1
    assert call(x.data_ptr(), 301, ctypes.byref(c), ws.numel()) == -2
    assert call(x.data_ptr(), 10, ctypes.byref(c), lib.fp_workspace_bytes(1, 300)) == -4
    assert call(x.data_ptr(), 10, ctypes.byref(c), ws.numel()) == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_workloads_equal_mdps_sample(fp, order, name):
    """Full size, the configuration bench.py times: identical to mdps_sample (which the workload
    tests pin to the oracle), level bookkeeping included."""
    from paper_2507_23480_amd import calibration
    say("pruned mdps at workload", name, "scan order", order)
    wl = inputs.WORKLOADS[name]
    st = wl.stages[0]
    x = dev(inputs.make_batch(name))
    prm = dataclasses.replace(calibration.params_for(name, 0), scan_order=order)
    a, ainfo = fp.mdps_sample(x, st.n, prm, want_info=True)
    b, binfo = fp.mdps_sample_pruned(x, st.n, prm, want_info=True)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    for ia, ib in zip(fp.parse_info(ainfo), fp.parse_info(binfo)):
        assert ib.status == 0 and ia.m == ib.m and ia.et_index == ib.et_index
        assert list(ia.level_start[:prm.nseg]) == list(ib.level_start[:prm.nseg])
        assert list(ia.level_exhausted[:prm.nseg]) == list(ib.level_exhausted[:prm.nseg])
        assert list(ia.thr2[:prm.nseg]) == list(ib.thr2[:prm.nseg])
