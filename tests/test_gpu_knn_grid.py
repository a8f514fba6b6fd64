"""GPU parity of the k nearest samples through a grid over the samples (fp_knn_grid) against
the CPU oracle's definition and the brute-force kernel, through the C ABI: positions and squared
distances bit-exact, whatever share of the points the grid settles."""
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


def check(fp, batch, sidx, k, radius):
    x = dev(np.ascontiguousarray(batch, dtype=np.float32))
    s = dev(np.ascontiguousarray(sidx, dtype=np.int32))
    pos, d2, deferred = fp.knn_grid(x, s, k, radius, want_deferred=True)
    bpos, bd2 = fp.knn(x, s, k)
    torch.cuda.synchronize()
    assert torch.equal(pos, bpos) and torch.equal(d2, bd2), "grid differs from brute force"
    for b in range(batch.shape[0]):
        wp, wd = ref.knn(batch[b], sidx[b], k)
        assert np.array_equal(pos[b].cpu().numpy(), wp) and np.array_equal(d2[b].cpu().numpy(), wd)
    return deferred.cpu().numpy()


def test_line_example(fp):
    pts = np.stack([np.arange(9), np.zeros(9), np.zeros(9)], axis=1).astype(np.float32)
    for radius in (0.5, 2.5, 100.0):
        check(fp, pts[None], np.array([[0, 8, 4, 2, 6]]), 3, radius)


@pytest.mark.parametrize("N,n,k,radius", [(64, 64, 1, 0.3), (300, 40, 3, 0.4), (1000, 257, 8, 0.25), (2049, 513, 3, 0.1),
                                          (5000, 700, 5, 0.15), (700, 2, 2, 0.5), (3000, 900, 3, 1e-4),
                                          (3000, 900, 3, 50.0)])
def test_uniform_cube(fp, N, n, k, radius):
    say("grid knn N=%d n=%d k=%d r=%g" % (N, n, k, radius))
    cloud = inputs.uniform_cube(800 + N, N)
    sidx = np.random.Generator(np.random.PCG64(N)).permutation(N)[:n]
    deferred = check(fp, cloud[None], sidx[None], k, radius)
    if radius == 50.0:
        assert deferred[0] == 0            # every sample lies in the 27 cells of every point
    if radius == 1e-4:
        assert deferred[0] > 0             # only the samples themselves find anything that close


def test_ties_duplicates_and_batches(fp):
    batch = np.stack([inputs.lattice_with_ties(40 + b, 900, 5) for b in range(3)])
    sidx = np.random.Generator(np.random.PCG64(3)).integers(0, 900, (3, 300))
    for k in (3, 8):
        check(fp, batch, sidx, k, 2.5)


def test_invalid_samples_are_never_neighbours(fp):
    cloud = inputs.uniform_cube(33, 500)[None]
    sidx = np.array([[5, -1, 17, 500, 40, 3]], dtype=np.int32)
    pos, d2 = fp.knn_grid(dev(cloud), dev(sidx), 3, 0.6)
    torch.cuda.synchronize()
    valid = np.array([0, 2, 4, 5])
    wp, wd = ref.knn(cloud[0], sidx[0, valid], 3)
    assert np.array_equal(pos.cpu().numpy()[0], valid[wp]) and np.array_equal(d2.cpu().numpy()[0], wd)


def test_argument_checks(fp):
    lib = fp.load()
    assert lib.fp_knn_grid_workspace_bytes(1, 100, 0) == 0
    x = dev(inputs.uniform_cube(1, 100)[None])
    s = dev(np.arange(10, dtype=np.int32)[None])
    pos = torch.empty((1, 100, 3), dtype=torch.int32, device="cuda")
    d2 = torch.empty((1, 100, 3), dtype=torch.float32, device="cuda")
    ws = torch.empty(lib.fp_knn_grid_workspace_bytes(1, 100, 10), dtype=torch.uint8, device="cuda")
    call = lambda k, r, wsb: lib.fp_knn_grid(x.data_ptr(), 1, 100, s.data_ptr(), 10, k, r, pos.data_ptr(),
                                             d2.data_ptr(), None, ws.data_ptr(), wsb, None)
    assert call(3, 0.2, ws.numel()) == 0
    assert call(9, 0.2, ws.numel()) == -2 and call(3, 0.0, ws.numel()) == -3 and call(3, 0.2, 128) == -4
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_workloads_equal_the_brute_force_kernel(fp, name):
    """Stage 0 at full size, the three nearest exact-FPS samples of every point, search radius
    three times the samples' coverage radius: the bytes of fp_knn without a cache (which the
    workload tests pin to the oracle), and nearly every point settled in the grid."""
    say("grid knn at workload", name)
    wl = inputs.WORKLOADS[name]
    st = wl.stages[0]
    x = dev(inputs.make_batch(name))
    sidx = fp.fps_exact(x, st.n)
    radius = 3.0 * float(fp.coverage2(x, sidx).max().sqrt())
    pos, d2, deferred = fp.knn_grid(x, sidx, 3, radius, want_deferred=True)
    bpos, bd2 = fp.knn(x, sidx, 3)
    torch.cuda.synchronize()
    assert torch.equal(pos, bpos) and torch.equal(d2, bd2)
    say("  deferred share %.4f" % (float(deferred.sum()) / (wl.B * wl.N)))
