"""fp_fps_exact_static -- the entry point for callers that cannot allocate (its scratch memory is
a static device array inside the library) -- against fp_fps_exact on the same inputs, through the
C ABI: samples and curve bit for bit, on two calls in a row, the second with a smaller input (the
array keeps the first call's contents, which the second must not see).  All buffers are allocated
before the first call; the calls themselves get plain pointers."""
import ctypes

import numpy as np
import pytest

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


def test_static_scratch_entry_point_equals_fps_exact_on_two_calls_in_a_row(fp):
    lib = fp.load()
    shapes = [(2, 60000, 3000), (3, 9000, 700)]          # 59 and 9 workgroups per cloud, then smaller
    bufs = []
    for B, N, n in shapes:                                # everything is allocated up front
        batch = np.stack([inputs.uniform_cube(900 + 10 * N + b, N) for b in range(B)])
        xyz = torch.from_numpy(batch).cuda()
        start = torch.tensor([(7 * b + 1) % N for b in range(B)], dtype=torch.int32, device="cuda")
        bufs.append((xyz, start, torch.full((B, n), -7, dtype=torch.int32, device="cuda"),
                     torch.full((B, n), -7.0, dtype=torch.float32, device="cuda")))
        assert fp.plan(B, N)[0] > 1
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream().cuda_stream
    for (B, N, n), (xyz, start, idx, mdc) in zip(shapes, bufs):
        print("fp_fps_exact_static B=%d N=%d n=%d" % (B, N, n), flush=True)
        rc = lib.fp_fps_exact_static(xyz.data_ptr(), B, N, n, start.data_ptr(), idx.data_ptr(), mdc.data_ptr(), stream)
        assert rc == 0, lib.fp_status_string(rc)
    torch.cuda.synchronize()
    for (B, N, n), (xyz, start, idx, mdc) in zip(shapes, bufs):
        widx, wmdc = fp.fps_exact(xyz, n, start_idx=start, want_mdc=True)
        torch.cuda.synchronize()
        assert torch.equal(idx, widx), "samples differ from fp_fps_exact (B=%d N=%d)" % (B, N)
        assert torch.equal(mdc, wmdc), "curve differs from fp_fps_exact (B=%d N=%d)" % (B, N)


def test_static_scratch_entry_point_checks_its_arguments(fp):
    lib = fp.load()
    x = torch.zeros((1, 16, 3), dtype=torch.float32, device="cuda")
    out = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    assert lib.fp_fps_exact_static(None, 1, 16, 4, None, out.data_ptr(), None, None) == -1
    assert lib.fp_fps_exact_static(x.data_ptr(), 1, 16, 17, None, out.data_ptr(), None, None) == -2
    # more points than the static array's exchange slots serve: refused with a message of its own
    assert lib.fp_fps_exact_static(x.data_ptr(), 1, 2097153, 4, None, out.data_ptr(), None, None) == -6
    assert b"static scratch" in lib.fp_status_string(-6)
