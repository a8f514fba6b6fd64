"""GPU parity of the exclusion lists (the list-building loops of Alg. 2 with the extra ball-query level of
Section 4.2) and of the ball query by lookup, through the C ABI, against the CPU oracle:
offsets and members bit-exact (the lists are index sets decided by binary32 comparisons)."""
import ctypes
import os
import sys
from concurrent.futures import ThreadPoolExecutor

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


def oracle_rows(batch, thr):
    """Offsets and members in the library's row order (level, cloud, point)."""
    B, N = batch.shape[0], batch.shape[1]
    L = thr.shape[1]
    with ThreadPoolExecutor(max_workers=8) as ex:            # ctypes calls drop the GIL
        per = list(ex.map(lambda b: ref.excl_lists(batch[b], thr[b]), range(B)))
    sizes = np.zeros(L * B * N, dtype=np.int64)
    chunks = []
    for l in range(L):
        for b in range(B):
            off, ent = per[b]
            sizes[(l * B + b) * N:(l * B + b + 1) * N] = np.diff(off[l * N:(l + 1) * N + 1])
            chunks.append(ent[off[l * N]:off[(l + 1) * N]])
    offsets = np.concatenate([[0], np.cumsum(sizes)])
    return offsets, (np.concatenate(chunks) if chunks else np.zeros(0, np.int32))


def check_lists(fp, batch, thr):
    batch = np.ascontiguousarray(batch, dtype=np.float32)
    thr = np.ascontiguousarray(thr, dtype=np.float32)
    off, ent = fp.excl_lists(dev(batch), dev(thr))
    torch.cuda.synchronize()
    woff, went = oracle_rows(batch, thr)
    assert np.array_equal(off.cpu().numpy(), woff), "offsets"
    assert np.array_equal(ent.cpu().numpy(), went), "members"
    return off, ent


def line9():
    return np.stack([np.arange(9), np.zeros(9), np.zeros(9)], axis=1).astype(np.float32)


def test_line_example(fp):
    check_lists(fp, line9()[None], np.array([[10.0, 2.0, 6.25]]))


@pytest.mark.parametrize("N,thr", [(1, [0.5]), (63, [0.1, 0.01]), (64, [0.3]), (65, [0.02, 0.2, 0.07]),
                                   (300, [0.09, 0.04, 0.01, 0.0025]), (1000, [0.01] * 17),
                                   (2049, [0.004, 0.001, 0.002, 0.0005, 0.003, 0.00025, 0.0001])])
def test_uniform_cube(fp, N, thr):
    say("excl lists N=%d L=%d" % (N, len(thr)))
    check_lists(fp, inputs.uniform_cube(1200 + N, N)[None], np.array([thr]))


def test_batch_with_a_radius_set_per_cloud(fp):
    batch = np.stack([inputs.uniform_cube(40 + b, 700) * (1.0 + b) for b in range(4)])
    thr = np.array([[0.02, 0.005], [0.3, 0.0001], [1e-9, 0.05], [0.5, 0.5]], dtype=np.float32)
    check_lists(fp, batch, thr)


def test_batch_with_long_rows(fp):
    # several clouds whose rows are longer than what the sorting kernel takes, radii per cloud
    rng = np.random.Generator(np.random.PCG64(8))
    batch = np.stack([np.concatenate([rng.normal(0.0, 0.02 * (b + 1), (1200, 3)),
                                      rng.uniform(-1.0, 1.0, (800, 3))])[rng.permutation(2000)]
                      for b in range(3)]).astype(np.float32)
    thr = np.array([[0.01, 0.0004], [0.0009, 0.04], [0.09, 0.09]], dtype=np.float32)
    off, _ = check_lists(fp, batch, thr)
    sizes = np.diff(off.cpu().numpy()).reshape(2, 3, 2000)
    assert (sizes.max(axis=(0, 2)) > 600).all()           # every cloud has rows for the bitmap kernel


def test_ties_and_duplicates(fp):
    batch = np.stack([inputs.lattice_with_ties(60 + b, 900, 4) for b in range(2)])
    # radii on attainable squared distances (strict <) and between them
    check_lists(fp, batch, np.array([[2.0, 1.0, 3.5, 0.5]] * 2))


@pytest.mark.parametrize("N", [2048, 2100, 3000])
def test_radius_beyond_the_cloud(fp, N):
    # every point is in every list: the rows reach and pass the size one wave sorts in LDS
    say("excl lists, all points, N=%d" % N)
    check_lists(fp, inputs.uniform_cube(5, N)[None], np.array([[4.0, 0.01]]))


def test_rows_around_the_sort_capacity(fp):
    # clustered cloud: rows below, at and above the LDS capacity in one call
    rng = np.random.Generator(np.random.PCG64(12))
    dense = rng.normal(0.0, 0.01, (2500, 3))
    sparse = rng.uniform(-1.0, 1.0, (1500, 3))
    cloud = np.concatenate([dense, sparse]).astype(np.float32)
    cloud = cloud[rng.permutation(4000)]
    off, _ = check_lists(fp, cloud[None], np.array([[0.0009, 0.0001, 0.25]]))
    sizes = np.diff(off.cpu().numpy())
    assert sizes.max() > 2048 and sizes.min() >= 1


@pytest.mark.parametrize("N,cluster", [(70000, 2600), (70000, 300), (530000, 2600), (530000, 1100)])
def test_long_rows_over_several_index_slabs(fp, N, cluster):
    """Longer rows are built from a bitmap over slabs of 32768 or 65536 indices, shorter ones by
    sorting; where the border lies depends on the number of slabs (128 members per slab).  Clouds
    of more points than one slab, with a cluster whose members' indices lie in all of them:
    3 slabs with rows of 2600 (bitmap) and 300 (sorted), 9 slabs with rows of 2600 (bitmap) and
    1100 (sorted, the largest network).
    The all-pairs oracle would take minutes here; the rows of sampled points are checked against
    the oracle's ball query (first k members by index, k above the longest row; radii are powers
    of two, so radius * radius is the list's squared radius exactly), every row size against the
    number of rows that hold the point (the relation is symmetric)."""
    rng = np.random.Generator(np.random.PCG64(31 + cluster))
    dense = rng.normal(0.0, 0.002, (cluster, 3))
    sparse = rng.uniform(-8.0, 8.0, (N - cluster, 3))
    cloud = np.concatenate([dense, sparse]).astype(np.float32)
    cloud = cloud[rng.permutation(N)]
    radii = [2.0 ** -6, 2.0 ** -8]
    thr = np.array([[r * r for r in radii]], dtype=np.float32)
    say("excl lists, long rows over several slabs, N=%d, cluster of %d" % (N, cluster))
    off, ent = fp.excl_lists(dev(cloud[None]), dev(thr))
    torch.cuda.synchronize()
    off, ent = off.cpu().numpy(), ent.cpu().numpy()
    sizes = np.diff(off).reshape(2, N)
    assert sizes[0].max() > 0.95 * cluster and sizes.min() >= 1
    in_cluster = np.flatnonzero(sizes[0] > 0.5 * cluster)
    assert in_cluster.min() < 32768 and in_cluster.max() >= 65536 * ((N - 1) // 65536)
    picks = np.concatenate([in_cluster[:40], in_cluster[-40:], rng.integers(0, N, 60)]).astype(np.int32)
    for l, r in enumerate(radii):
        widx, wcnt = ref.ball_query(cloud, picks, r, 4096)
        for t, i in enumerate(picks):
            row = ent[off[l * N + i]:off[l * N + i + 1]]
            assert row.shape[0] == wcnt[t], "row size, level %d point %d" % (l, i)
            assert np.array_equal(row, widx[t, :wcnt[t]]), "row members, level %d point %d" % (l, i)
        # symmetry: i is in the row of j exactly when j is in the row of i
        assert np.array_equal(np.bincount(ent[off[l * N]:off[(l + 1) * N]], minlength=N), sizes[l])


def test_empty_levels(fp):
    thr = np.array([[0.0, -1.0, np.nan, 0.01]], dtype=np.float32)
    off, ent = check_lists(fp, inputs.uniform_cube(9, 500)[None], thr)
    assert int(off[3 * 500]) == 0
    off, ent = check_lists(fp, inputs.uniform_cube(9, 500)[None], np.array([[0.0, np.nan]], dtype=np.float32))
    assert ent.numel() == 0


def test_coincident_points(fp):
    cloud = np.zeros((300, 3), dtype=np.float32) + np.float32(0.25)
    check_lists(fp, cloud[None], np.array([[1e-30, 0.0]]))


def test_infinite_radius(fp):
    check_lists(fp, inputs.uniform_cube(3, 400)[None], np.array([[np.inf, 0.01]], dtype=np.float32))


def test_fill_respects_capacity(fp):
    lib = fp.load()
    cloud = dev(inputs.uniform_cube(21, 800)[None])
    thr = dev(np.array([[0.05, 0.01]], dtype=np.float32))
    off, ent = fp.excl_lists(cloud, thr)
    torch.cuda.synchronize()
    total = ent.numel()
    cap = total // 2
    ws = torch.empty(lib.fp_excl_workspace_bytes(1, 800, 2), dtype=torch.uint8, device="cuda")
    off2 = torch.empty_like(off)
    part = torch.full((total,), -5, dtype=torch.int32, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    assert lib.fp_excl_count(cloud.data_ptr(), 1, 800, thr.data_ptr(), 2, off2.data_ptr(), ws.data_ptr(),
                             ws.numel(), s) == 0
    assert lib.fp_excl_fill(cloud.data_ptr(), 1, 800, thr.data_ptr(), 2, off2.data_ptr(), part.data_ptr(),
                            ctypes.c_int64(cap), ws.data_ptr(), ws.numel(), s) == 0
    torch.cuda.synchronize()
    assert torch.equal(off2, off)
    assert torch.equal(part[:cap], ent[:cap]) and bool((part[cap:] == -5).all())


def test_argument_checks(fp):
    lib = fp.load()
    assert lib.fp_excl_workspace_bytes(1, 100, 18) == 0
    assert lib.fp_excl_workspace_bytes(0, 100, 2) == 0
    cloud = dev(inputs.uniform_cube(1, 100)[None])
    thr = dev(np.array([[0.1]], dtype=np.float32))
    off = torch.empty(101, dtype=torch.int64, device="cuda")
    ws = torch.empty(lib.fp_excl_workspace_bytes(1, 100, 1), dtype=torch.uint8, device="cuda")
    assert lib.fp_excl_count(cloud.data_ptr(), 1, 100, thr.data_ptr(), 1, off.data_ptr(), ws.data_ptr(), 16, None) == -4
    assert lib.fp_excl_count(None, 1, 100, thr.data_ptr(), 1, off.data_ptr(), ws.data_ptr(), ws.numel(), None) == -1
    assert lib.fp_excl_count(cloud.data_ptr(), 1, 100, thr.data_ptr(), 0, off.data_ptr(), ws.data_ptr(),
                             ws.numel(), None) == -2


@pytest.mark.parametrize("k", [1, 16, 64])
def test_lookup_equals_ball_query_for_any_centres(fp, k):
    # the list at the query radius answers the ball query of ANY centre set, samples or not
    B, N, M = 3, 1500, 333
    batch = np.stack([inputs.uniform_cube(80 + b, N) for b in range(B)])
    radius = 0.11
    r2 = np.float32(radius) * np.float32(radius)
    thr = np.array([[0.05, r2]] * B, dtype=np.float32)
    x = dev(batch)
    off, ent = fp.excl_lists(x, dev(thr))
    centres = np.random.Generator(np.random.PCG64(k)).integers(0, N, (B, M)).astype(np.int32)
    idx, cnt = fp.ball_query_lists(off, ent, B, N, 2, 1, dev(centres), k)
    bidx, bcnt = fp.ball_query(x, dev(centres), radius, k)
    torch.cuda.synchronize()
    assert torch.equal(idx, bidx) and torch.equal(cnt, bcnt)
    for b in range(B):
        widx, wcnt = ref.ball_query(batch[b], centres[b], radius, k)
        assert np.array_equal(idx[b].cpu().numpy(), widx) and np.array_equal(cnt[b].cpu().numpy(), wcnt)


def test_lookup_of_empty_rows_and_bad_centres(fp):
    cloud = inputs.uniform_cube(2, 200)[None]
    off, ent = fp.excl_lists(dev(cloud), dev(np.array([[0.0, 0.01]], dtype=np.float32)))
    centres = dev(np.array([[3, -1, 200, 7]], dtype=np.int32))
    idx, cnt = fp.ball_query_lists(off, ent, 1, 200, 2, 0, centres, 4)
    torch.cuda.synchronize()
    assert bool((idx == -1).all()) and bool((cnt == 0).all())
    idx, cnt = fp.ball_query_lists(off, ent, 1, 200, 2, 1, centres, 4)
    torch.cuda.synchronize()
    assert idx[0, 1].tolist() == [-1] * 4 and idx[0, 2].tolist() == [-1] * 4 and cnt[0].tolist()[1:3] == [0, 0]
    widx, wcnt = ref.ball_query(cloud[0], [3, 7], 0.1, 4)
    assert idx[0, 0].tolist() == widx[0].tolist() and idx[0, 3].tolist() == widx[1].tolist()


@pytest.mark.parametrize("name,clouds", [("C1", 1), ("C2", 4), ("C3", 2)])
def test_workload_shapes_with_the_thresholds_of_mdps(fp, name, clouds):
    """Stage 0 of a workload: levels = the nseg thresholds MDPS derived for each cloud (read
    from the sampler's info records on the device) and the ball-query radius."""
    from paper_2507_23480_amd import calibration
    say("excl lists at workload", name)
    wl = inputs.WORKLOADS[name]
    st = wl.stages[0]
    batch = inputs.make_batch(name)[:clouds]
    x = dev(batch)
    prm = calibration.params_for(name, 0)
    _, info = fp.mdps_sample(x, st.n, prm, want_info=True)
    torch.cuda.synchronize()
    recs = fp.parse_info(info)
    thr = np.array([[r.thr2[l] for l in range(prm.nseg)] + [np.float32(st.radius) * np.float32(st.radius)]
                    for r in recs], dtype=np.float32)
    off, ent = check_lists(fp, batch, thr)
    # the extra level answers the stage's ball query for the MDPS samples
    midx = fp.mdps_sample(x, st.n, prm)
    idx, cnt = fp.ball_query_lists(off, ent, clouds, wl.N, prm.nseg + 1, prm.nseg, midx, st.k)
    bidx, bcnt = fp.ball_query(x, midx, st.radius, st.k)
    torch.cuda.synchronize()
    assert torch.equal(idx, bidx) and torch.equal(cnt, bcnt)


def test_lidar_cloud_at_full_size(fp):
    """One full cloud of the LiDAR-like workload (120 000 points in ring-major order, rows of
    several thousand members near the sensor) with the levels of its own MDPS run and the
    ball-query radius.  The oracle's all-pairs pass gives the size of EVERY row (its count pass;
    about a minute on one core); the members of rows sampled over the whole index range, the
    longest rows among them, are compared with the oracle's ball query (a row is the ball of its
    point: first k members by index with k above the longest row); and the relation is checked
    to be symmetric on all rows."""
    from paper_2507_23480_amd import calibration
    wl = inputs.WORKLOADS["C4"]
    st = wl.stages[0]
    cloud = inputs.make_cloud("C4", 1)
    N = wl.N
    x = dev(cloud[None])
    prm = calibration.params_for("C4", 0)
    _, info = fp.mdps_sample(x, st.n, prm, want_info=True)
    torch.cuda.synchronize()
    rec = fp.parse_info(info)[0]
    radii2 = [rec.thr2[l] for l in range(prm.nseg)] + [np.float32(st.radius) * np.float32(st.radius)]
    thr = np.array([radii2], dtype=np.float32)
    L = thr.shape[1]
    say("excl lists, C4 cloud at full size: N=%d, %d levels" % (N, L))
    off, ent = fp.excl_lists(x, dev(thr))
    torch.cuda.synchronize()
    say("   %d members; oracle count pass over all pairs ..." % ent.numel())
    woff = np.empty(L * N + 1, dtype=np.int64)
    rc = ref.lib().ref_excl_lists(cloud.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), N,
                                  thr[0].ctypes.data_as(ctypes.POINTER(ctypes.c_float)), L,
                                  woff.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), None, 0)
    assert rc == 0
    assert np.array_equal(off.cpu().numpy(), woff), "row sizes differ from the oracle's"
    say("   all %d row sizes equal the oracle's" % (L * N))
    sizes = np.diff(woff).reshape(L, N)
    for l in range(L):      # symmetry on every row: i is in the row of j exactly when j is in the row of i
        counts = torch.bincount(ent[int(woff[l * N]):int(woff[(l + 1) * N])], minlength=N)
        assert np.array_equal(counts.cpu().numpy(), sizes[l])
    rng = np.random.Generator(np.random.PCG64(44))
    widest = int(np.argmax(radii2))
    picks = np.unique(np.concatenate([np.argsort(sizes[widest])[-150:], rng.integers(0, N, 1350),
                                      np.arange(0, N, N // 100)])).astype(np.int32)
    off_h = woff
    for l in range(L):
        kmax = int(sizes[l][picks].max()) + 1
        radius = float(np.sqrt(np.float64(radii2[l])))
        if np.float32(radius) * np.float32(radius) != np.float32(radii2[l]):
            continue        # the level's squared radius is not the square of a binary32 radius: no ball query gives it
        for c0 in range(0, len(picks), 128):
            chunk = picks[c0:c0 + 128]
            widx, wcnt = ref.ball_query(cloud, chunk, radius, kmax)
            for t, i in enumerate(chunk):
                a, b = int(off_h[l * N + i]), int(off_h[l * N + i + 1])
                assert b - a == wcnt[t]
                assert np.array_equal(ent[a:b].cpu().numpy(), widx[t, :wcnt[t]]), "members, level %d point %d" % (l, i)
        say("   level %d: members of %d sampled rows (longest %d) equal the oracle's" % (l, len(picks), kmax - 1))


def test_million_point_cloud_sampled_rows(fp):
    """The large single cloud (10^6 points, 200 clusters) with the levels of its own MDPS run and the
    ball-query radius: about 10^10 members (40 GB), which the device memory holds.  The all-pairs
    oracle is out of reach at this size; the rows of points sampled over the whole index range are
    compared with the oracle's ball query (a row is the ball of its point) on every level, and every
    row's size with the number of members the oracle finds."""
    gold = np.load(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "c5_full.npz"))
    wl = inputs.WORKLOADS["C5"]
    st = wl.stages[0]
    N = wl.N
    cloud = inputs.make_cloud("C5", 0)
    radii2 = [np.float32(v) for v in gold["thr2_calibrated"][0]] + [np.float32(st.radius) * np.float32(st.radius)]
    thr = np.array([radii2], dtype=np.float32)
    L = thr.shape[1]
    free, _ = torch.cuda.mem_get_info()
    x = dev(cloud[None])
    say("excl lists, C5 at full size: N=%d, %d levels" % (N, L))
    lib = fp.load()
    ws = torch.empty(lib.fp_excl_workspace_bytes(1, N, L), dtype=torch.uint8, device="cuda")
    off = torch.empty(L * N + 1, dtype=torch.int64, device="cuda")
    t = dev(thr)
    s = torch.cuda.current_stream().cuda_stream
    assert lib.fp_excl_count(x.data_ptr(), 1, N, t.data_ptr(), L, off.data_ptr(), ws.data_ptr(), ws.numel(), s) == 0
    torch.cuda.synchronize()
    total = int(off[-1].item())
    say("   %d members (%.1f GB)" % (total, 4.0 * total / 1e9))
    if 4 * total + (8 << 30) > free:
        pytest.skip("not enough free device memory for the members of this cloud")
    ent = torch.empty(total, dtype=torch.int32, device="cuda")
    assert lib.fp_excl_fill(x.data_ptr(), 1, N, t.data_ptr(), L, off.data_ptr(), ent.data_ptr(), ctypes.c_int64(total),
                            ws.data_ptr(), ws.numel(), s) == 0
    torch.cuda.synchronize()
    off_h = off.cpu().numpy()
    rng = np.random.Generator(np.random.PCG64(45))
    picks = np.unique(np.concatenate([rng.integers(0, N, 150), np.arange(0, N, N // 50)])).astype(np.int32)
    for l in range(L):
        radius = float(np.sqrt(np.float64(radii2[l])))
        if np.float32(radius) * np.float32(radius) != np.float32(radii2[l]):
            continue        # no binary32 radius squares to this level's value: no ball query gives the row
        sizes = off_h[l * N + picks + 1] - off_h[l * N + picks]
        kmax = int(sizes.max()) + 1
        for c0 in range(0, len(picks), 32):
            chunk = picks[c0:c0 + 32]
            widx, wcnt = ref.ball_query(cloud, chunk, radius, kmax)
            for tt, i in enumerate(chunk):
                a, b = int(off_h[l * N + i]), int(off_h[l * N + i + 1])
                assert b - a == wcnt[tt], "row size, level %d point %d" % (l, i)
                assert np.array_equal(ent[a:b].cpu().numpy(), widx[tt, :wcnt[tt]]), "members, level %d point %d" % (l, i)
        say("   level %d: %d sampled rows (longest %d) equal the oracle's" % (l, len(picks), kmax - 1))


def test_clouds_too_large_for_the_lists_are_refused(fp):
    """The list kernels address a cloud's points and rows with the limits the header states; a
    shape beyond them is refused on the host with FP_ERR_SHAPE and nothing is launched."""
    lib = fp.load()
    assert lib.fp_excl_workspace_bytes(1, 1 << 30, 17) == 0 or lib.fp_excl_workspace_bytes(70000, 1 << 20, 2) == 0
    assert lib.fp_excl_workspace_bytes(70000, 100, 2) == 0          # more clouds than the grid kernels index
    x = dev(inputs.uniform_cube(1, 100)[None])
    thr = dev(np.array([[0.1]], dtype=np.float32))
    off = torch.empty(101, dtype=torch.int64, device="cuda")
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda")
    assert lib.fp_excl_count(x.data_ptr(), 70000, 100, thr.data_ptr(), 1, off.data_ptr(), ws.data_ptr(), 4096, None) == -2
