"""GPU parity at the five workload shapes, in the launch configuration bench.py times
(automatic plan, calibrated MDPS constants).

C1-C3: every cloud, every stage, element by element against the oracle, run live.
C4, C5: the oracle needs minutes for the full job, so
  * full N and full n: every sample of exact FPS (index and curve value) and of MDPS (index,
    thresholds, prefix length, level starts, exhausted flags, early-termination position) is
    compared with the oracle's results stored in tests/golden/c4_full.npz and c5_full.npz
    (written by tests/golden/make_large_golden.py, which calls only the oracle; the MDPS constants
    it used are stored with them and fed to the GPU here);
  * ball-query and k-NN rows of a few thousand sampled centres / points, computed live by the
    oracle; cached == brute on every row; coverage bound; properties that hold at any size;
  * full N with a reduced sample count n once more live against the oracle.
"""
import dataclasses
import json
import os
import sys
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from oracle import ref
from paper_2507_23480_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

COVERAGE_BOUND = 1.05     # MDPS coverage radius relative to exact FPS
KNN_K = 3                 # neighbours of the up-sampling step (Section 3.1)


@pytest.fixture(scope="module")
def fp():
    from paper_2507_23480_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load()
    binding.set_wg_per_cloud(0)
    return binding


@pytest.fixture(scope="module")
def cal():
    from paper_2507_23480_amd import calibration
    return calibration


def say(*a):
    print(*a, flush=True)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def pmap(fn, items):
    with ThreadPoolExecutor(max_workers=8) as ex:       # ctypes calls drop the GIL
        return list(ex.map(fn, items))


def rparams(prm):
    return ref.MdpsParams(p=prm.p, nseg=prm.nseg, exponent=prm.exponent, bias=prm.bias,
                          fit_window=prm.fit_window, m_min=prm.m_min, level_scale=prm.level_scale,
                          scan_order=prm.scan_order)


def d2(a, b):
    """binary32 squared distances between point sets a [A][3] and b [B][3] -> [A][B]"""
    dx = a[:, None, 0] - b[None, :, 0]
    dy = a[:, None, 1] - b[None, :, 1]
    dz = a[:, None, 2] - b[None, :, 2]
    t = dx * dx
    t = t + dy * dy
    t = t + dz * dz
    return t


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_full_workload_matches_oracle(fp, cal, name):
    wl = inputs.WORKLOADS[name]
    batch = inputs.make_batch(name)
    for s, st in enumerate(wl.stages):
        say("%s stage %d: B=%d N=%d n=%d" % (name, s, wl.B, batch.shape[1], st.n))
        prm = cal.params_for(name, s)
        xyz = dev(batch)
        cache = fp.new_bq_cache(xyz, st.n)
        idx, mdc = fp.fps_exact(xyz, st.n, want_mdc=True)
        bq, cnt = fp.ball_query(xyz, idx, st.radius, st.k)
        midx, info = fp.mdps_sample(xyz, st.n, prm, want_info=True, bq_cache=cache, bq_radius=st.radius)
        mbq, mcnt = fp.ball_query(xyz, midx, st.radius, st.k, bq_cache=cache)
        cov_f, cov_m = fp.coverage2(xyz, idx).sqrt(), fp.coverage2(xyz, midx).sqrt()
        # the estimator exactly as Appendix A.3 defines it (no per-segment factors)
        pprm = cal.params_for(name, s, "paper")
        pidx, pinfo = fp.mdps_sample(xyz, st.n, pprm, want_info=True)
        cov_p = fp.coverage2(xyz, pidx).sqrt()
        # the scattered scan order of the threshold phase, on the cloud in walk order and in cell order
        sprm = dataclasses.replace(prm, scan_order=1)
        sidx, sinfo = fp.mdps_sample(xyz, st.n, sprm, want_info=True)
        spidx, spinfo = fp.mdps_sample_pruned(xyz, st.n, sprm, want_info=True)
        cov_s = fp.coverage2(xyz, sidx).sqrt()
        kpos, kd2 = fp.knn(xyz, idx, KNN_K)
        mkpos, mkd2, deferred = fp.knn(xyz, midx, KNN_K, bq_cache=cache, want_deferred=True)
        torch.cuda.synchronize()
        assert torch.equal(sidx, spidx)
        sidx, sinfos, spinfos = sidx.cpu().numpy(), fp.parse_info(sinfo), fp.parse_info(spinfo)
        rps = rparams(sprm)
        say("   k-NN points searched by brute force: %s of %d" % (deferred.cpu().tolist(), batch.shape[1]))
        kpos, kd2, mkpos, mkd2 = kpos.cpu().numpy(), kd2.cpu().numpy(), mkpos.cpu().numpy(), mkd2.cpu().numpy()
        idx, mdc, bq, cnt = idx.cpu().numpy(), mdc.cpu().numpy(), bq.cpu().numpy(), cnt.cpu().numpy()
        midx, mbq, mcnt = midx.cpu().numpy(), mbq.cpu().numpy(), mcnt.cpu().numpy()
        infos = fp.parse_info(info)
        pinfos = fp.parse_info(pinfo)
        pidx = pidx.cpu().numpy()
        rp = rparams(prm)
        rpp = rparams(pprm)

        def one(b):
            widx, wmdc = ref.fps_exact(batch[b], st.n)
            wbq, wcnt = ref.ball_query(batch[b], widx, st.radius, st.k)
            wmidx, winfo = ref.mdps_sample(batch[b], st.n, rp)
            wmbq, wmcnt = ref.ball_query(batch[b], wmidx, st.radius, st.k)
            return widx, wmdc, wbq, wcnt, wmidx, winfo, wmbq, wmcnt, ref.knn(batch[b], widx, KNN_K), \
                ref.knn(batch[b], wmidx, KNN_K), ref.mdps_sample(batch[b], st.n, rpp), \
                ref.mdps_sample(batch[b], st.n, rps)
        for b, (widx, wmdc, wbq, wcnt, wmidx, winfo, wmbq, wmcnt, wk, wmk, wp, ws) in enumerate(pmap(one, range(wl.B))):
            assert np.array_equal(sidx[b], ws[0]), "mdps with the scattered scan order, cloud %d" % b
            for gi in (sinfos[b], spinfos[b]):
                assert gi.status == 0 and gi.et_index == ws[1].et_index
                assert np.array_equal(np.array(gi.thr2[:prm.nseg], np.float32), ws[1].thr2)
                assert list(gi.level_start[:prm.nseg]) == ws[1].level_start.tolist()
                assert list(gi.level_exhausted[:prm.nseg]) == ws[1].level_exhausted.tolist()
            assert np.array_equal(pidx[b], wp[0]), "mdps with the pure power function, cloud %d" % b
            assert pinfos[b].status == 0 and pinfos[b].et_index == wp[1].et_index
            assert np.array_equal(np.array(pinfos[b].thr2[:pprm.nseg], np.float32), wp[1].thr2)
            assert np.array_equal(kpos[b], wk[0]) and np.array_equal(kd2[b], wk[1]), "brute k-NN cloud %d" % b
            assert np.array_equal(mkpos[b], wmk[0]) and np.array_equal(mkd2[b], wmk[1]), "cached k-NN cloud %d" % b
            assert np.array_equal(idx[b], widx) and np.array_equal(mdc[b], wmdc), "fps cloud %d" % b
            assert np.array_equal(bq[b], wbq) and np.array_equal(cnt[b], wcnt), "brute bq cloud %d" % b
            assert np.array_equal(midx[b], wmidx), "mdps cloud %d" % b
            assert infos[b].status == 0 and infos[b].et_index == winfo.et_index
            assert np.array_equal(np.array(infos[b].thr2[:prm.nseg], np.float32), winfo.thr2)
            assert np.array_equal(mbq[b], wmbq) and np.array_equal(mcnt[b], wmcnt), "cached bq cloud %d" % b
        ratio = (cov_m / cov_f).cpu().numpy()
        pratio = (cov_p / cov_f).cpu().numpy()
        say("   coverage ratio max %.4f; pure power function (bias %.2f): %.4f, FPS tail %.1f%% of the samples"
            % (ratio.max(), pprm.bias, pratio.max(), 100.0 * np.mean([(st.n - i.et_index) / st.n for i in pinfos])))
        sratio = (cov_s / cov_f).cpu().numpy()
        say("   scattered scan order: coverage ratio max %.4f" % sratio.max())
        assert ratio.max() <= COVERAGE_BOUND and pratio.max() <= COVERAGE_BOUND and sratio.max() <= COVERAGE_BOUND
        if s + 1 < len(wl.stages):
            batch = np.stack([ref.gather_xyz(batch[b], idx[b]) for b in range(wl.B)])


GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def check_against_stored_oracle(fp, name, xyz, idx, mdc):
    """Every sample of the full-size run against the oracle's stored results: exact FPS as given,
    MDPS run here with each stored set of estimator constants."""
    wl = inputs.WORKLOADS[name]
    n = wl.stages[0].n
    with np.load(os.path.join(GOLDEN, name.lower() + "_full.npz")) as z:
        gold = {k: z[k] for k in z.files}
    assert gold["fps_idx"].shape == (wl.B, n)
    assert np.array_equal(idx, gold["fps_idx"]), "%s exact FPS: samples differ from the stored oracle result" % name
    assert np.array_equal(mdc, gold["fps_mdc"]), "%s exact FPS: curve differs from the stored oracle result" % name
    variants = sorted(k[len("params_"):] for k in gold if k.startswith("params_"))
    assert "calibrated" in variants and "paper" in variants and "scattered" in variants
    for v in variants:
        p = json.loads(str(gold["params_" + v]))
        prm = fp.MdpsParams(p=p["p"], nseg=p["nseg"], exponent=p["exponent"], bias=p["bias"],
                            fit_window=p["fit_window"], m_min=p["m_min"], level_scale=p["level_scale"],
                            scan_order=p.get("scan_order", 0))
        # both entry points: the cloud as given (or in the order of the walk), and in cell order
        for entry in (fp.mdps_sample, fp.mdps_sample_pruned):
            midx, info = entry(xyz, n, prm, want_info=True)
            torch.cuda.synchronize()
            infos = fp.parse_info(info)
            assert np.array_equal(midx.cpu().numpy(), gold["mdps_idx_" + v]), \
                "%s %s (%s constants): samples differ from the stored oracle result" % (name, entry.__name__, v)
            for b, gi in enumerate(infos):
                assert gi.status == 0 and gi.m == gold["m_" + v][b] and gi.et_index == gold["et_index_" + v][b]
                assert np.array_equal(np.array(gi.thr2[:prm.nseg], np.float32), gold["thr2_" + v][b])
                assert np.array_equal(np.array(gi.level_start[:prm.nseg]), gold["level_start_" + v][b])
                assert np.array_equal(np.array(gi.level_exhausted[:prm.nseg]), gold["level_exhausted_" + v][b])
        cov = fp.coverage2(xyz, midx).sqrt() / fp.coverage2(xyz, torch.from_numpy(gold["fps_idx"]).cuda()).sqrt()
        torch.cuda.synchronize()
        say("   %s constants (bias %.2f): all %d x %d MDPS samples equal the stored oracle result, FPS tail %s, "
            "coverage ratio max %.4f" % (v, p["bias"], wl.B, n, [n - int(e) for e in gold["et_index_" + v]],
                                          float(cov.max())))
        assert float(cov.max()) <= COVERAGE_BOUND
    return gold


def check_large(fp, cal, name, n_small, bq_centres):
    wl = inputs.WORKLOADS[name]
    st = wl.stages[0]
    batch = inputs.make_batch(name)
    xyz = dev(batch)
    prm = cal.params_for(name, 0)
    rp = rparams(prm)
    B, N, n = wl.B, wl.N, st.n

    # ---- full N, reduced n: element by element
    say("%s: full N=%d, reduced n=%d" % (name, N, n_small))
    sidx, smdc = fp.fps_exact(xyz, n_small, want_mdc=True)
    smidx, sinfo = fp.mdps_sample(xyz, n_small, prm, want_info=True)
    torch.cuda.synchronize()
    sidx, smdc, smidx = sidx.cpu().numpy(), smdc.cpu().numpy(), smidx.cpu().numpy()
    sinfos = fp.parse_info(sinfo)
    want = pmap(lambda b: (ref.fps_exact(batch[b], n_small), ref.mdps_sample(batch[b], n_small, rp)),
                range(B))
    for b, ((widx, wmdc), (wmidx, winfo)) in enumerate(want):
        assert np.array_equal(sidx[b], widx) and np.array_equal(smdc[b], wmdc), "fps cloud %d" % b
        assert np.array_equal(smidx[b], wmidx), "mdps cloud %d" % b
        assert sinfos[b].et_index == winfo.et_index
        assert np.array_equal(np.array(sinfos[b].thr2[:prm.nseg], np.float32), winfo.thr2)

    # ---- full N, full n
    say("%s: full N=%d, full n=%d" % (name, N, n))
    cache = fp.new_bq_cache(xyz, n)
    idx, mdc = fp.fps_exact(xyz, n, want_mdc=True)
    midx, info = fp.mdps_sample(xyz, n, prm, want_info=True, bq_cache=cache, bq_radius=st.radius)
    bq, cnt = fp.ball_query(xyz, midx, st.radius, st.k)
    cbq, ccnt = fp.ball_query(xyz, midx, st.radius, st.k, bq_cache=cache)
    fbq, fcnt = fp.ball_query(xyz, idx, st.radius, st.k)
    cov = (fp.coverage2(xyz, midx).sqrt() / fp.coverage2(xyz, idx).sqrt())
    kpos, kd2 = fp.knn(xyz, midx, KNN_K)
    ckpos, ckd2, deferred = fp.knn(xyz, midx, KNN_K, bq_cache=cache, want_deferred=True)
    torch.cuda.synchronize()
    assert torch.equal(bq, cbq) and torch.equal(cnt, ccnt), "cached ball query differs from brute force"
    assert torch.equal(kpos, ckpos) and torch.equal(kd2, ckd2), "redundancy-free k-NN differs from brute force"
    # the cell-ordered recorder at full size, both scan orders: its samples are those of mdps_sample (compared
    # with the stored oracle results below), the ball query read from its record is the brute-force one
    # (sampled rows of which are compared with the oracle below), and the k-NN search, which does not
    # read such a record, still returns the brute-force result
    for order in (0, 1):
        oprm = dataclasses.replace(prm, scan_order=order)
        pcache = fp.new_bq_cache(xyz, n, 10 * N if name == "C4" else 0)
        pidx = fp.mdps_sample_pruned(xyz, n, oprm, bq_cache=pcache, bq_radius=st.radius)
        assert torch.equal(pidx, fp.mdps_sample(xyz, n, oprm))
        pbq, pcnt = fp.ball_query(xyz, pidx, st.radius, st.k, bq_cache=pcache)
        wbq, wcnt = (bq, cnt) if order == 0 else fp.ball_query(xyz, pidx, st.radius, st.k)
        torch.cuda.synchronize()
        assert not any(fp.bq_cache_stats(pcache)["incomplete"])
        assert torch.equal(pbq, wbq) and torch.equal(pcnt, wcnt), "ball query from the cell-ordered record, order %d" % order
        if order == 0:
            pk = fp.knn(xyz, pidx, KNN_K, bq_cache=pcache)
            torch.cuda.synchronize()
            assert torch.equal(pk[0], kpos) and torch.equal(pk[1], kd2)
        del pcache
    say("   k-NN points searched by brute force: %s of %d" % (deferred.cpu().tolist(), N))
    kpos, kd2 = kpos.cpu().numpy(), kd2.cpu().numpy()
    idx, mdc, midx = idx.cpu().numpy(), mdc.cpu().numpy(), midx.cpu().numpy()
    bq, cnt, fbq, fcnt = bq.cpu().numpy(), cnt.cpu().numpy(), fbq.cpu().numpy(), fcnt.cpu().numpy()
    infos = fp.parse_info(info)
    say("   coverage ratio max %.4f, FPS tail %s" % (float(cov.max()), [n - i.et_index for i in infos]))
    assert float(cov.max()) <= COVERAGE_BOUND
    gold = check_against_stored_oracle(fp, name, xyz, idx, mdc)
    if json.loads(str(gold["params_calibrated"]))["bias"] == prm.bias:
        # the recording run above used the stored constants: its samples are the stored ones too
        assert np.array_equal(midx, gold["mdps_idx_calibrated"])
    rng = np.random.Generator(np.random.PCG64(5))
    for b in range(B):
        pts = batch[b]
        # exact FPS: prefix property, curve non-increasing, curve values of sampled picks
        assert np.array_equal(idx[b, :n_small], sidx[b]) and np.array_equal(mdc[b, :n_small], smdc[b])
        assert np.all(mdc[b, 1:-1] >= mdc[b, 2:])
        assert len(np.unique(idx[b])) == n
        for i in rng.integers(1, n, 64):
            assert mdc[b, i] == d2(pts[idx[b, i:i + 1]], pts[idx[b, :i]]).min()
        # MDPS: same prefix as exact FPS, spacing bound of the level of sampled picks
        gi = infos[b]
        assert gi.status == 0 and np.array_equal(midx[b, :gi.m + 1], idx[b, :gi.m + 1])
        assert len(np.unique(midx[b])) == n
        starts = [s for s in gi.level_start[:prm.nseg]]
        for i in rng.integers(gi.m + 1, max(gi.et_index, gi.m + 2), 64):
            if i >= gi.et_index:
                continue
            lvl = max(l for l in range(prm.nseg) if 0 <= starts[l] <= i)
            assert d2(pts[midx[b, i:i + 1]], pts[midx[b, :i]]).min() >= gi.thr2[lvl]
        # ball-query rows of sampled centres, computed one by one by the oracle
        qs = rng.integers(0, n, bq_centres)
        wq, wc = ref.ball_query(pts, midx[b, qs], st.radius, st.k)
        assert np.array_equal(bq[b, qs], wq) and np.array_equal(cnt[b, qs], wc)
        wq, wc = ref.ball_query(pts, idx[b, qs], st.radius, st.k)
        assert np.array_equal(fbq[b, qs], wq) and np.array_equal(fcnt[b, qs], wc)
        # k-NN rows of sampled points
        js = rng.integers(0, N, bq_centres)
        wp, wd = ref.knn(pts, midx[b], KNN_K, points=js)
        assert np.array_equal(kpos[b, js], wp) and np.array_equal(kd2[b, js], wd)


def test_lidar_workload(fp, cal):
    check_large(fp, cal, "C4", n_small=2048, bq_centres=4096)


def test_million_point_workload(fp, cal):
    check_large(fp, cal, "C5", n_small=1024, bq_centres=2048)


@pytest.mark.parametrize("name", ["C3", "C4"])
def test_point_order_of_the_cloud(fp, cal, name):
    """The workloads whose points come in scanner order (surface by surface, ring by ring), run
    again with every cloud shuffled.  Exact FPS does not depend on the order of the points except
    through ties between equal distances: started from the same point it picks the same points
    (checked pick by pick while the two curves agree, which they do where no tie occurs).
    MDPS takes "the lowest available index", so its samples do depend on the order; the coverage
    bound has to hold in either order."""
    wl = inputs.WORKLOADS[name]
    st = wl.stages[0]
    batch = inputs.make_batch(name)
    B, N, n = wl.B, wl.N, st.n
    rng = np.random.Generator(np.random.PCG64(99))
    perms = [rng.permutation(N) for _ in range(B)]
    shuffled = np.stack([batch[b][perms[b]] for b in range(B)])
    starts = [int(np.flatnonzero(perms[b] == 0)[0]) for b in range(B)]       # where point 0 went
    prm = cal.params_for(name, 0)
    x, xs = dev(batch), dev(shuffled)
    say("%s: scanner order and shuffled" % name)
    idx, mdc = fp.fps_exact(x, n, want_mdc=True)
    sidx, smdc = fp.fps_exact(xs, n, start_idx=starts, want_mdc=True)
    midx = fp.mdps_sample(x, n, prm)
    smidx = fp.mdps_sample(xs, n, prm, start_idx=starts)
    cov = fp.coverage2(x, midx).sqrt() / fp.coverage2(x, idx).sqrt()
    scov = fp.coverage2(xs, smidx).sqrt() / fp.coverage2(xs, sidx).sqrt()
    torch.cuda.synchronize()
    say("   coverage ratio max: scanner order %.4f, shuffled %.4f" % (float(cov.max()), float(scov.max())))
    assert float(cov.max()) <= COVERAGE_BOUND and float(scov.max()) <= COVERAGE_BOUND
    idx, mdc, sidx, smdc = idx.cpu().numpy(), mdc.cpu().numpy(), sidx.cpu().numpy(), smdc.cpu().numpy()
    for b in range(B):
        back = perms[b][sidx[b]]                           # the shuffled run's picks as original indices
        same = back == idx[b]
        agree = int(n if same.all() else np.argmin(same))  # picks before the first difference
        assert np.array_equal(smdc[b, :agree], mdc[b, :agree])
        if agree < n:
            # the runs part at a tie: two points at the same distance, taken in index order
            assert smdc[b, agree] == mdc[b, agree], "cloud %d parts at pick %d without a tie" % (b, agree)
        say("   cloud %d: identical picks %d of %d" % (b, agree, n))
        assert agree > n // 20


def test_expired_wait_ends_the_kernel_cleanly(fp):
    # with a wait limit of zero a wait gives up after two empty polls: the kernel
    # must end on its own and report status 2 with an all -1 result (no hang, no fault)
    cloud = inputs.uniform_cube(77, 30000)[None]
    fp.set_wg_per_cloud(8)
    fp.set_wait_limit_us(0)
    try:
        idx, info = fp.fps_exact(dev(cloud), 4000, want_info=True)
        torch.cuda.synchronize()
    finally:
        fp.set_wait_limit_us(2000000)
        fp.set_wg_per_cloud(0)
    st = fp.parse_info(info)[0].status
    if st == 2:
        assert bool((idx == -1).all())
    else:       # every wait happened to be met within the limit: the result must then be right
        assert st == 0 and np.array_equal(idx.cpu().numpy()[0], ref.fps_exact(cloud[0], 4000)[0])
    again = fp.fps_exact(dev(cloud), 500)
    torch.cuda.synchronize()
    assert np.array_equal(again.cpu().numpy()[0], ref.fps_exact(cloud[0], 500)[0])
