"""Edge cases of the C ABI on the GPU: degenerate and maximum sizes, batches larger than the
device holds at once, and the error codes of the argument checks (nothing is enqueued on an
error).  Results against the CPU oracle, bit-exact."""
import ctypes
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
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("N,n", [(1, 1), (2, 1), (2, 2), (3, 3), (1000, 1), (1000, 2)])
def test_smallest_shapes(fp, N, n):
    cloud = inputs.uniform_cube(N, N)
    x = dev(cloud[None])
    want = ref.fps_exact(cloud, n)
    idx, mdc = fp.fps_exact(x, n, want_mdc=True)
    pidx = fp.fps_exact_pruned(x, n)
    midx = fp.mdps_sample(x, n, fp.MdpsParams())            # n this small is exact FPS by definition
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy()[0], want[0]) and np.array_equal(mdc.cpu().numpy()[0], want[1])
    assert np.array_equal(pidx.cpu().numpy()[0], want[0])
    assert np.array_equal(midx.cpu().numpy()[0], ref.mdps_sample(cloud, n, ref.MdpsParams())[0])
    bq, cnt = fp.ball_query(x, idx, 0.5, 3)
    torch.cuda.synchronize()
    wbq, wcnt = ref.ball_query(cloud, want[0], 0.5, 3)
    assert np.array_equal(bq.cpu().numpy()[0], wbq) and np.array_equal(cnt.cpu().numpy()[0], wcnt)


@pytest.mark.parametrize("N,n", [(1, 1), (2, 2), (3, 3), (10, 10), (63, 40), (64, 64), (65, 65), (129, 100),
                                 (257, 257), (1000, 2)])
def test_smallest_shapes_with_a_threshold_phase(fp, N, n):
    """Small clouds with a prefix of one or two exact iterations, so that nearly every sample comes from
    the threshold phase or its early termination: both scan orders, the cloud as given and in cell
    order, with and without a record, n up to N (every point is sampled)."""
    cloud = inputs.uniform_cube(900 + N, N)
    x = dev(cloud[None])
    for order in (0, 1):
        for thr in ([0.05, 0.01], [1e-30, 1e-30], [float("inf"), 4.0]):
            prm = fp.MdpsParams(p=0.01, nseg=2, m_min=1, thr_override=thr, scan_order=order)
            rp = ref.MdpsParams(p=0.01, nseg=2, m_min=1, thr_override=thr, scan_order=order)
            want, winfo = ref.mdps_sample(cloud, n, rp)
            a, ainfo = fp.mdps_sample(x, n, prm, want_info=True)
            b, binfo = fp.mdps_sample_pruned(x, n, prm, want_info=True)
            cache = fp.new_bq_cache(x, n, entries_per_cloud=n * ((N + 63) // 64) + N + 128)
            c = fp.mdps_sample_pruned(x, n, prm, bq_cache=cache, bq_radius=0.3)
            bq, cnt = fp.ball_query(x, c, 0.3, 5, bq_cache=cache)
            torch.cuda.synchronize()
            for got, info in ((a, ainfo), (b, binfo), (c, None)):
                assert np.array_equal(got.cpu().numpy()[0], want), "N=%d n=%d order=%d thr=%s" % (N, n, order, thr)
                if info is not None:
                    gi = fp.parse_info(info)[0]
                    assert gi.status == 0 and gi.m == winfo.m and gi.et_index == winfo.et_index
            wbq, wcnt = ref.ball_query(cloud, want, 0.3, 5)
            assert np.array_equal(bq.cpu().numpy()[0], wbq) and np.array_equal(cnt.cpu().numpy()[0], wcnt)


def test_more_clouds_than_the_device_holds_at_once(fp):
    # 300 clouds: the workgroups take further clouds in turn
    B, N, n = 300, 500, 120
    batch = np.stack([inputs.uniform_cube(7000 + b, N) for b in range(B)])
    x = dev(batch)
    prm = fp.MdpsParams(exponent=0.9, bias=1.1)
    rp = ref.MdpsParams(exponent=0.9, bias=1.1)
    idx = fp.fps_exact(x, n).cpu().numpy()
    pidx = fp.fps_exact_pruned(x, n).cpu().numpy()
    cache = fp.new_bq_cache(x, n)
    midx_t = fp.mdps_sample(x, n, prm, bq_cache=cache, bq_radius=0.2)
    bq, cnt = fp.ball_query(x, midx_t, 0.2, 8, bq_cache=cache)
    torch.cuda.synchronize()
    midx = midx_t.cpu().numpy()
    for b in range(B):
        want = ref.fps_exact(batch[b], n)[0]
        assert np.array_equal(idx[b], want), "fps cloud %d" % b
        assert np.array_equal(pidx[b], want), "pruned fps cloud %d" % b
        wm = ref.mdps_sample(batch[b], n, rp)[0]
        assert np.array_equal(midx[b], wm), "mdps cloud %d" % b
    for b in (0, 131, 299):
        wbq, wcnt = ref.ball_query(batch[b], midx[b], 0.2, 8)
        assert np.array_equal(bq[b].cpu().numpy(), wbq) and np.array_equal(cnt[b].cpu().numpy(), wcnt)


def test_largest_cloud_the_sampler_takes(fp):
    # 256 workgroups x 8192 points; one more point is refused
    N = 256 * 8192
    say("largest cloud", N)
    rng = np.random.Generator(np.random.PCG64(99))
    cloud = rng.uniform(0, 1, (N, 3)).astype(np.float32)
    x = dev(cloud[None])
    n = 48
    want = ref.fps_exact(cloud, n)
    idx, mdc = fp.fps_exact(x, n, want_mdc=True)
    pidx = fp.fps_exact_pruned(x, n)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy()[0], want[0]) and np.array_equal(mdc.cpu().numpy()[0], want[1])
    assert np.array_equal(pidx.cpu().numpy()[0], want[0])
    lib = fp.load()
    g, t, p = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    assert lib.fp_plan(1, N, ctypes.byref(g), ctypes.byref(t), ctypes.byref(p)) == 0 and g.value == 256
    assert lib.fp_plan(1, N + 1, ctypes.byref(g), ctypes.byref(t), ctypes.byref(p)) == -2
    big = torch.empty((1, N + 1, 3), dtype=torch.float32, device="cuda")
    out = torch.empty((1, n), dtype=torch.int32, device="cuda")
    ws = fp.new_workspace(x.device, 1, N)
    assert lib.fp_fps_exact(big.data_ptr(), 1, N + 1, n, None, out.data_ptr(), None, None, None, 0, 0.0,
                            ws.data_ptr(), ws.numel(), None) == -2


def test_ball_query_limits(fp):
    cloud = inputs.uniform_cube(4, 300)
    x = dev(cloud[None])
    centres = np.arange(0, 300, 3, dtype=np.int32)
    for radius, k in ((10.0, 254), (10.0, 1), (1e-6, 254), (0.3, 200)):
        bq, cnt = fp.ball_query(x, dev(centres[None]), radius, k)
        torch.cuda.synchronize()
        wbq, wcnt = ref.ball_query(cloud, centres, radius, k)
        assert np.array_equal(bq.cpu().numpy()[0], wbq) and np.array_equal(cnt.cpu().numpy()[0], wcnt)
    empty = torch.empty((1, 0), dtype=torch.int32, device="cuda")
    bq, cnt = fp.ball_query(x, empty, 0.1, 4)
    torch.cuda.synchronize()
    assert bq.shape == (1, 0, 4) and cnt.shape == (1, 0)


def test_error_codes(fp):
    lib = fp.load()
    x = dev(inputs.uniform_cube(1, 200)[None])
    out = torch.empty((1, 50), dtype=torch.int32, device="cuda")
    ws = fp.new_workspace(x.device, 1, 200)
    f = lambda *a: lib.fp_fps_exact(*a)
    ok = (x.data_ptr(), 1, 200, 50, None, out.data_ptr(), None, None, None, 0, 0.0, ws.data_ptr(), ws.numel(), None)
    assert f(*ok) == 0
    assert f(None, *ok[1:]) == -1                                     # xyz
    assert f(*ok[:5], None, *ok[6:]) == -1                            # out_idx
    assert f(*ok[:3], 201, *ok[4:]) == -2                             # n > N
    assert f(*ok[:3], 0, *ok[4:]) == -2                               # n < 1
    assert f(*ok[:1], 0, *ok[2:]) == -2                               # B < 1
    assert f(*ok[:11], None, 0, None) == -4                           # no workspace
    assert f(*ok[:11], ws.data_ptr() + 8, ws.numel() - 8, None) == -4  # misaligned
    assert f(*ok[:12], 1024, None) == -4                              # too small
    cache = fp.new_bq_cache(x, 50)
    assert f(*ok[:8], cache.data_ptr(), cache.numel(), 0.0, *ok[11:]) == -3          # cache without a radius
    assert f(*ok[:8], cache.data_ptr() + 4, cache.numel() - 4, 0.1, *ok[11:]) == -4  # misaligned cache
    assert f(*ok[:8], cache.data_ptr(), 1024, 0.1, *ok[11:]) == -4                   # cache too small for any entry
    assert 2 * 200 + 16 * 50 <= lib.fp_bq_cache_entries(cache.numel(), 1, 200, 50) < 2 * 200 + 16 * 50 + 32
    assert lib.fp_bq_cache_bytes(1, 200, 50, 0) == cache.numel()
    assert lib.fp_bq_cache_entries(lib.fp_bq_cache_bytes(1, 200, 50, 12345), 1, 200, 50) >= 12345
    torch.cuda.synchronize()

    def mdps(**kw):
        prm = fp.MdpsParams(**{k: v for k, v in kw.items() if k not in ("raw",)}).to_c()
        for k, v in kw.get("raw", {}).items():
            setattr(prm, k, v)
        return lib.fp_mdps_sample(x.data_ptr(), 1, 200, 50, None, ctypes.byref(prm), out.data_ptr(), None, None,
                                  0, 0.0, ws.data_ptr(), ws.numel(), None)
    assert mdps() == 0
    assert mdps(raw={"p": 0.0}) == -3 and mdps(raw={"p": 1.0}) == -3
    assert mdps(raw={"nseg": 0}) == -3 and mdps(raw={"nseg": 17}) == -3
    assert mdps(raw={"bias": 0.0}) == -3 and mdps(raw={"fit_window": 65}) == -3 and mdps(raw={"m_min": 0}) == -3
    assert lib.fp_mdps_sample(x.data_ptr(), 1, 200, 50, None, None, out.data_ptr(), None, None, 0, 0.0,
                              ws.data_ptr(), ws.numel(), None) == -1
    torch.cuda.synchronize()

    c = dev(np.zeros((1, 4), dtype=np.int32))
    bo = torch.empty((1, 4, 8), dtype=torch.int32, device="cuda")
    bq = lambda r, k: lib.fp_ball_query(x.data_ptr(), 1, 200, c.data_ptr(), 4, r, k, bo.data_ptr(), None, None, None)
    assert bq(0.1, 8) == 0
    assert bq(0.0, 8) == -3 and bq(-1.0, 8) == -3 and bq(float("inf"), 8) == -3 and bq(float("nan"), 8) == -3
    assert bq(0.1, 0) == -2 and bq(0.1, 255) == -2
    torch.cuda.synchronize()
    assert lib.fp_status_string(0) == b"ok" and len(lib.fp_status_string(-3)) > 0


def test_phase_times_are_reported(fp):
    """info.phase_ticks: the four phases of MDPS add up to less than the call, exact FPS has one."""
    from paper_2507_23480_amd import calibration
    x = dev(inputs.make_batch("C2"))
    _, info = fp.mdps_sample(x, 512, calibration.params_for("C2", 0), want_info=True)
    _, finfo = fp.fps_exact(x, 512, want_info=True)
    torch.cuda.synchronize()
    for i in fp.parse_info(info):
        t = list(i.phase_ticks)
        assert all(v >= 0 for v in t) and t[0] > 0 and t[2] > 0
        assert sum(t) < 100 * 1000 * 100          # well under a second (10 ns ticks)
    for i in fp.parse_info(finfo):
        t = list(i.phase_ticks)
        assert t[0] > 0 and t[1] == 0 and t[2] == 0 and t[3] == 0


def test_recording_with_sixteen_points_per_thread(fp):
    """The largest kernel shape with radius recording (its radius-test rows take 64 KB of LDS):
    the cache reader must give the brute-force bytes, the samples the oracle's."""
    N, n, G = 150000, 96, 20                      # 7500 points per workgroup -> 16 per thread
    say("recording, P=16", N)
    cloud = np.random.Generator(np.random.PCG64(5)).uniform(0, 1, (N, 3)).astype(np.float32)
    x = dev(cloud[None])
    fp.set_wg_per_cloud(G)
    try:
        assert fp.plan(1, N) == (G, 512, 16)
        cache = fp.new_bq_cache(x, n)
        idx = fp.fps_exact(x, n, bq_cache=cache, bq_radius=0.05)
        cbq = fp.ball_query(x, idx, 0.05, 16, bq_cache=cache)
        cache2 = fp.new_bq_cache(x, n)
        midx = fp.mdps_sample(x, n, fp.MdpsParams(exponent=0.7, bias=1.05), bq_cache=cache2, bq_radius=0.05)
        mbq = fp.ball_query(x, midx, 0.05, 16, bq_cache=cache2)
        torch.cuda.synchronize()
    finally:
        fp.set_wg_per_cloud(0)
    assert np.array_equal(idx.cpu().numpy()[0], ref.fps_exact(cloud, n)[0])
    assert np.array_equal(midx.cpu().numpy()[0], ref.mdps_sample(cloud, n, ref.MdpsParams(exponent=0.7, bias=1.05))[0])
    for got, centres in ((cbq, idx), (mbq, midx)):
        want = fp.ball_query(x, centres, 0.05, 16)
        torch.cuda.synchronize()
        assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1])


@pytest.mark.parametrize("G", [65, 100, 130, 192, 200])
def test_clouds_over_two_to_four_waves_of_workgroup_counts(fp, G):
    """The candidate exchange adds up the workgroups' counts in as many waves as hold them (64 counts
    each): workgroup counts that need two, three and four of them, every sampler, a few hundred
    points per workgroup so that most rounds take candidates from many workgroups."""
    N, n = 48000, 1500
    say("exchange over", G, "workgroups")
    cloud = inputs.uniform_cube(900 + G, N)
    x = dev(cloud[None])
    prm = dict(exponent=0.8, bias=1.04)
    fp.set_wg_per_cloud(G)
    try:
        assert fp.plan(1, N)[0] == G
        idx = fp.fps_exact(x, n)
        pidx = fp.fps_exact_pruned(x, n)
        midx = fp.mdps_sample(x, n, fp.MdpsParams(**prm))
        mpidx = fp.mdps_sample_pruned(x, n, fp.MdpsParams(**prm))
        m1idx = fp.mdps_sample(x, n, fp.MdpsParams(scan_order=1, **prm))
        mp1idx = fp.mdps_sample_pruned(x, n, fp.MdpsParams(scan_order=1, **prm))
        torch.cuda.synchronize()
    finally:
        fp.set_wg_per_cloud(0)
    want = ref.fps_exact(cloud, n)[0]
    assert np.array_equal(idx.cpu().numpy()[0], want) and np.array_equal(pidx.cpu().numpy()[0], want)
    want = ref.mdps_sample(cloud, n, ref.MdpsParams(**prm))[0]
    assert np.array_equal(midx.cpu().numpy()[0], want) and np.array_equal(mpidx.cpu().numpy()[0], want)
    want = ref.mdps_sample(cloud, n, ref.MdpsParams(scan_order=1, **prm))[0]
    assert np.array_equal(m1idx.cpu().numpy()[0], want) and np.array_equal(mp1idx.cpu().numpy()[0], want)


def test_plain_fp32_rate_probe(fp):
    """The measurement aid runs and lands near 256 compute units x 64 lanes x the clock."""
    rate = fp.probe_fp32_rate(torch.device("cuda:0"), blocks=4096, iterations=2048)
    assert 5e12 < rate < 80e12
    lib = fp.load()
    out = torch.empty(256, dtype=torch.float32, device="cuda")
    assert lib.fp_probe_fp32_rate(1, 0, out.data_ptr(), None) == -2
    assert lib.fp_probe_fp32_rate(0, 10, out.data_ptr(), None) == -2
    assert lib.fp_probe_fp32_rate(1, 10, None, None) == -1
