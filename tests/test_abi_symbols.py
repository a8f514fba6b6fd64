"""The C-ABI library loads on a machine without a GPU and exports every symbol that
include/fastpoint.h declares (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fastpoint.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fp_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2507_23480_amd import binding
    lib = binding.load()
    names = declared_functions()
    assert "fp_fps_exact" in names and "fp_mdps_sample" in names and "fp_ball_query" in names
    for name in names:
        assert hasattr(lib, name), "missing export: " + name
    assert sorted(binding.EXPORTS) == names


def test_struct_layouts_match_the_header():
    from paper_2507_23480_amd import binding
    # fp_mdps_params: float,int32,double,float,int32,int32,int32,float[16],float[16],pointer; info: 2+16+16+16+2 words
    assert ctypes.sizeof(binding.FpMdpsParams) == 176
    assert ctypes.sizeof(binding.FpMdpsInfo) == 4 * (2 + 16 + 16 + 16 + 2 + 4)


def test_host_side_argument_checks_need_no_gpu():
    from paper_2507_23480_amd import binding
    lib = binding.load()
    assert lib.fp_workspace_bytes(0, 10) == 0
    assert lib.fp_workspace_bytes(1, 10) > 0
    assert lib.fp_bq_cache_bytes(1, 100, 101, 0) == 0
    assert lib.fp_bq_cache_bytes(2, 1000, 10, 0) >= 256 + 2 * 10 * 4 + 2 * (2 * 1000 + 16 * 10) * (16 + 12)
    assert lib.fp_status_string(0) == b"ok"
    assert lib.fp_status_string(-2) == b"shape out of range"
    # NULL pointers are rejected before anything touches a device
    assert lib.fp_ball_query(None, 1, 10, None, 1, 1.0, 4, None, None, None, None) == -1
    assert lib.fp_gather_xyz(None, 1, 10, None, 1, None, None) == -1


def test_plan_covers_the_workload_shapes():
    from paper_2507_23480_amd import binding, inputs
    for wl in inputs.WORKLOADS.values():
        g, t, p = binding.plan(wl.B, wl.N)
        assert g * t * p >= wl.N and g >= 1 and wl.B * g <= 256 or wl.B > 256
    with pytest.raises(RuntimeError):
        binding.plan(1, 256 * 8192 + 1)       # larger than the resident capacity of one cloud
