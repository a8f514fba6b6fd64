"""GPU parity of the ball query through a uniform grid (fp_ball_query_grid) against the CPU
oracle's definition and against the brute-force kernel, through the C ABI: identical bytes."""
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


def check(fp, batch, centres, radius, k):
    x = dev(np.ascontiguousarray(batch, dtype=np.float32))
    c = dev(np.ascontiguousarray(centres, dtype=np.int32))
    idx, cnt = fp.ball_query_grid(x, c, radius, k)
    bidx, bcnt = fp.ball_query(x, c, radius, k)
    torch.cuda.synchronize()
    assert torch.equal(idx, bidx) and torch.equal(cnt, bcnt), "grid differs from brute force"
    for b in range(batch.shape[0]):
        widx, wcnt = ref.ball_query(batch[b], centres[b], radius, k)
        assert np.array_equal(idx[b].cpu().numpy(), widx) and np.array_equal(cnt[b].cpu().numpy(), wcnt)


def test_line_example(fp):
    pts = np.stack([np.arange(9), np.zeros(9), np.zeros(9)], axis=1).astype(np.float32)
    check(fp, pts[None], np.array([[0, 4, 8]]), 2.5, 4)
    check(fp, pts[None], np.array([[4]]), 2.0, 8)                 # strict <


@pytest.mark.parametrize("N,M,radius,k", [(1, 1, 0.5, 3), (63, 63, 0.3, 8), (300, 300, 0.2, 8), (1000, 77, 0.15, 32),
                                          (2049, 500, 0.05, 4), (5000, 333, 0.08, 64), (3000, 100, 10.0, 254),
                                          (3000, 100, 1e-7, 5), (700, 700, 0.4, 1)])
def test_uniform_cube(fp, N, M, radius, k):
    say("grid ball query N=%d M=%d r=%g k=%d" % (N, M, radius, k))
    cloud = inputs.uniform_cube(500 + N, N)
    centres = np.random.Generator(np.random.PCG64(N)).integers(0, N, M)
    check(fp, cloud[None], centres[None], radius, k)


def test_dense_and_sparse_balls_in_one_call(fp):
    # balls of a few hits and of thousands (several selections of the k lowest per centre)
    rng = np.random.Generator(np.random.PCG64(5))
    cloud = np.concatenate([rng.normal(0, 0.01, (3500, 3)), rng.uniform(-1, 1, (2500, 3))]).astype(np.float32)
    cloud = cloud[rng.permutation(6000)]
    centres = rng.integers(0, 6000, 400)
    for k in (16, 254):
        check(fp, cloud[None], centres[None], 0.05, k)


def test_batches_ties_and_invalid_centres(fp):
    batch = np.stack([inputs.lattice_with_ties(30 + b, 1200, 4) for b in range(3)])
    centres = np.random.Generator(np.random.PCG64(2)).integers(0, 1200, (3, 200))
    check(fp, batch, centres, 1.5, 16)
    x = dev(batch)
    c = dev(np.array([[5, -1, 1200, 7]] * 3, dtype=np.int32))
    idx, cnt = fp.ball_query_grid(x, c, 1.5, 6)
    torch.cuda.synchronize()
    assert bool((idx[:, 1:3] == -1).all()) and bool((cnt[:, 1:3] == 0).all())
    w, wc = ref.ball_query(batch[1], [5, 7], 1.5, 6)
    assert np.array_equal(idx[1, [0, 3]].cpu().numpy(), w) and np.array_equal(cnt[1, [0, 3]].cpu().numpy(), wc)


def test_no_centres_and_argument_checks(fp):
    lib = fp.load()
    x = dev(inputs.uniform_cube(1, 100)[None])
    idx, cnt = fp.ball_query_grid(x, torch.empty((1, 0), dtype=torch.int32, device="cuda"), 0.1, 4)
    assert idx.shape == (1, 0, 4)
    c = dev(np.zeros((1, 2), dtype=np.int32))
    out = torch.empty((1, 2, 4), dtype=torch.int32, device="cuda")
    ws = torch.empty(lib.fp_ball_query_grid_workspace_bytes(1, 100), dtype=torch.uint8, device="cuda")
    call = lambda r, k, wsb: lib.fp_ball_query_grid(x.data_ptr(), 1, 100, c.data_ptr(), 2, r, k, out.data_ptr(), None,
                                                    ws.data_ptr(), wsb, None)
    assert call(0.1, 4, ws.numel()) == 0
    assert call(0.0, 4, ws.numel()) == -3 and call(0.1, 255, ws.numel()) == -2 and call(0.1, 4, 64) == -4
    torch.cuda.synchronize()
    assert lib.fp_ball_query_grid_workspace_bytes(0, 5) == 0


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_workloads_equal_the_brute_force_kernel(fp, name):
    """Stage 0 at full size over the exact-FPS samples: the bytes of fp_ball_query, which the
    workload tests pin to the oracle."""
    say("grid ball query at workload", name)
    wl = inputs.WORKLOADS[name]
    st = wl.stages[0]
    x = dev(inputs.make_batch(name))
    centres = fp.fps_exact(x, st.n)
    idx, cnt = fp.ball_query_grid(x, centres, st.radius, st.k)
    bidx, bcnt = fp.ball_query(x, centres, st.radius, st.k)
    torch.cuda.synchronize()
    assert torch.equal(idx, bidx) and torch.equal(cnt, bcnt)
