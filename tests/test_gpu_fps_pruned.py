"""GPU parity of exact FPS with pruned distance updates (fp_fps_exact_pruned) against the CPU
oracle of Algorithm 1, through the C ABI: indices and the binary32 curve bit-exact.  The pruned
sampler works on a reordered copy of the cloud, so the cases stress what could depend on the
order: equal distances (lattices, duplicates), several workgroups per cloud, ragged sizes."""
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


def check(fp, batch, n, start=None, G=0):
    fp.set_wg_per_cloud(G)
    try:
        B = batch.shape[0]
        starts = [0] * B if start is None else list(start)
        idx, mdc, info = fp.fps_exact_pruned(dev(batch), n, start_idx=None if start is None else starts,
                                             want_mdc=True, want_info=True)
        torch.cuda.synchronize()
        idx, mdc = idx.cpu().numpy(), mdc.cpu().numpy()
        infos = fp.parse_info(info)
        for b in range(B):
            want = ref.fps_exact(batch[b], n, starts[b])
            assert infos[b].status == 0
            assert np.array_equal(idx[b], want[0]), "idx cloud %d" % b
            assert np.array_equal(mdc[b], want[1]), "curve cloud %d" % b
    finally:
        fp.set_wg_per_cloud(0)


def test_line_example(fp):
    pts = np.stack([np.arange(9), np.zeros(9), np.zeros(9)], axis=1).astype(np.float32)
    check(fp, pts[None], 9)


@pytest.mark.parametrize("N,n", [(1, 1), (2, 2), (63, 20), (64, 64), (65, 33), (1000, 250), (1025, 1025),
                                 (4097, 700), (9000, 1200)])
def test_uniform_cube(fp, N, n):
    say("pruned fps N=%d n=%d" % (N, n))
    check(fp, inputs.uniform_cube(300 + N, N)[None], n)


@pytest.mark.parametrize("G", [0, 1, 2, 5, 12])
def test_several_workgroups_per_cloud(fp, G):
    say("pruned fps G=%d" % G)
    batch = np.stack([inputs.uniform_cube(50 + b, 6000) for b in range(3)])
    check(fp, batch, 900, start=[0, 5999, 1234], G=G)


def test_equal_distances_take_the_lowest_index(fp):
    # integer lattices with repeated points: most arg-max decisions are ties, and the order of
    # the reordered copy is not the order of the indices
    batch = np.stack([inputs.lattice_with_ties(20 + b, 1500, 5) for b in range(4)])
    check(fp, batch, 1500)
    check(fp, batch, 400, G=3)


def test_all_points_coincide(fp):
    cloud = np.full((500, 3), 0.75, dtype=np.float32)
    check(fp, cloud[None], 40)


def test_clustered_cloud(fp):
    # dense clusters and a sparse background: cells of very different occupancy
    rng = np.random.Generator(np.random.PCG64(77))
    parts = [rng.normal(c, 0.01, (1500, 3)) for c in rng.uniform(-1, 1, (4, 3))]
    parts.append(rng.uniform(-1, 1, (2000, 3)))
    cloud = np.concatenate(parts).astype(np.float32)
    cloud = cloud[rng.permutation(cloud.shape[0])]
    check(fp, cloud[None], 2000)


def test_bad_start_index(fp):
    x = dev(inputs.uniform_cube(3, 300)[None])
    idx, info = fp.fps_exact_pruned(x, 10, start_idx=[300], want_info=True)
    torch.cuda.synchronize()
    assert bool((idx == -1).all()) and fp.parse_info(info)[0].status == 1


def test_argument_checks(fp):
    lib = fp.load()
    assert lib.fp_fps_pruned_workspace_bytes(0, 10) == 0
    x = dev(inputs.uniform_cube(3, 300)[None])
    out = torch.empty((1, 10), dtype=torch.int32, device="cuda")
    ws = torch.empty(lib.fp_fps_pruned_workspace_bytes(1, 300), dtype=torch.uint8, device="cuda")
    assert lib.fp_fps_exact_pruned(x.data_ptr(), 1, 300, 10, None, out.data_ptr(), None, None, ws.data_ptr(),
                                   lib.fp_workspace_bytes(1, 300), None) == -4
    assert lib.fp_fps_exact_pruned(x.data_ptr(), 1, 300, 301, None, out.data_ptr(), None, None, ws.data_ptr(),
                                   ws.numel(), None) == -2
    assert lib.fp_fps_exact_pruned(None, 1, 300, 10, None, out.data_ptr(), None, None, ws.data_ptr(),
                                   ws.numel(), None) == -1


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_workloads_equal_fps_exact(fp, name):
    """Full size, the configuration bench.py times: identical to fps_exact (which the workload
    tests pin to the oracle), and sampled curve values recomputed by the oracle's definition."""
    say("pruned fps at workload", name)
    wl = inputs.WORKLOADS[name]
    st = wl.stages[0]
    x = dev(inputs.make_batch(name))
    a, amdc = fp.fps_exact(x, st.n, want_mdc=True)
    b, bmdc, info = fp.fps_exact_pruned(x, st.n, want_mdc=True, want_info=True)
    torch.cuda.synchronize()
    assert all(i.status == 0 for i in fp.parse_info(info))
    assert torch.equal(a, b)
    assert torch.equal(amdc, bmdc)
