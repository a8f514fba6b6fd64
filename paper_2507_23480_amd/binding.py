"""Thin Python binding of the C ABI in include/fastpoint.h.

Argument marshalling only: tensors in, tensors out, every step of the path runs
in the HIP library.  PyTorch supplies device memory and the current stream.
There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
from typing import Optional, Sequence, Tuple

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libfastpoint_hip.so")
MAX_SEG = 16

EXPORTS = ["fp_mdps_scattered_workspace_bytes", "fp_bq_cache_entries", "fp_fps_exact_static", "fp_fps_pruned_workspace_bytes", "fp_fps_exact_pruned", "fp_mdps_sample_pruned", "fp_workspace_bytes", "fp_bq_cache_bytes", "fp_fps_exact", "fp_mdps_sample",
           "fp_ball_query", "fp_ball_query_grid_workspace_bytes", "fp_ball_query_grid", "fp_knn_workspace_bytes", "fp_knn", "fp_knn_grid_workspace_bytes", "fp_knn_grid", "fp_excl_workspace_bytes", "fp_excl_count",
           "fp_excl_fill", "fp_ball_query_lists", "fp_gather_xyz", "fp_coverage", "fp_probe_fp32_rate", "fp_plan", "fp_set_wg_per_cloud",
           "fp_set_wait_limit_us", "fp_set_cooperative_launch", "fp_status_string"]


class FpMdpsParams(ctypes.Structure):
    _fields_ = [("p", ctypes.c_float), ("nseg", ctypes.c_int32), ("exponent", ctypes.c_double),
                ("bias", ctypes.c_float), ("fit_window", ctypes.c_int32), ("m_min", ctypes.c_int32),
                ("use_override", ctypes.c_int32), ("thr_override", ctypes.c_float * MAX_SEG),
                ("level_scale", ctypes.c_float * MAX_SEG), ("mlp_weights", ctypes.c_void_p),
                ("scan_order", ctypes.c_int32), ("reserved0", ctypes.c_int32)]


MLP_WEIGHTS = 32 * 128 + 128 + 128 * 128 + 128 + 128 * 64 + 64


class FpMdpsInfo(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int32), ("et_index", ctypes.c_int32),
                ("level_start", ctypes.c_int32 * MAX_SEG),
                ("level_exhausted", ctypes.c_int32 * MAX_SEG),
                ("thr2", ctypes.c_float * MAX_SEG),
                ("rounds", ctypes.c_int32), ("status", ctypes.c_int32),
                ("phase_ticks", ctypes.c_int32 * 4)]


INFO_BYTES = ctypes.sizeof(FpMdpsInfo)


@dataclasses.dataclass
class MdpsParams:
    """MDPS hyper-parameters (paper defaults p = 0.1, nseg = 6; exponent and bias are
    fitted per workload, see calibration.py)."""
    p: float = 0.1
    nseg: int = 6
    exponent: float = 1.0
    bias: float = 1.0
    fit_window: int = 32
    m_min: int = 8
    thr_override: Optional[Sequence[float]] = None
    level_scale: Optional[Sequence[float]] = None
    mlp: Optional[torch.Tensor] = None    # MLP_WEIGHTS float32 weights on the device: the MLP estimator
    scan_order: int = 0                   # threshold phase: 0 lowest available index, 1 scattered walk

    def to_c(self) -> FpMdpsParams:
        c = FpMdpsParams()
        if self.mlp is not None:
            if not (self.mlp.is_cuda and self.mlp.dtype == torch.float32 and self.mlp.is_contiguous()
                    and self.mlp.numel() == MLP_WEIGHTS):
                raise ValueError("mlp must be a contiguous CUDA float32 tensor of MLP_WEIGHTS values")
            c.mlp_weights = self.mlp.data_ptr()
        for i in range(MAX_SEG):
            c.level_scale[i] = 1.0
        if self.level_scale is not None:
            if len(self.level_scale) != self.nseg:
                raise ValueError("level_scale needs nseg values")
            for i, v in enumerate(self.level_scale):
                c.level_scale[i] = v
        c.p, c.nseg, c.exponent, c.bias = self.p, self.nseg, self.exponent, self.bias
        c.fit_window, c.m_min = self.fit_window, self.m_min
        c.scan_order = int(self.scan_order)
        c.use_override = 0
        if self.thr_override is not None:
            if len(self.thr_override) != self.nseg:
                raise ValueError("thr_override needs nseg values")
            c.use_override = 1
            for i, v in enumerate(self.thr_override):
                c.thr_override[i] = v
        return c


_lib = None


def load() -> ctypes.CDLL:
    """Loads libfastpoint_hip.so (built by build.py); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("HIP library not built: %s is missing (run paper_2507_23480_amd/build.py)"
                           % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
    lib.fp_workspace_bytes.argtypes = [i32, i32]
    lib.fp_workspace_bytes.restype = ctypes.c_size_t
    lib.fp_bq_cache_bytes.argtypes = [i32, i32, i32, ctypes.c_int64]
    lib.fp_bq_cache_bytes.restype = ctypes.c_size_t
    lib.fp_bq_cache_entries.argtypes = [ctypes.c_size_t, i32, i32, i32]
    lib.fp_bq_cache_entries.restype = ctypes.c_int64
    lib.fp_fps_exact.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, ctypes.c_size_t, f32, vp, ctypes.c_size_t, vp]
    lib.fp_fps_exact.restype = i32
    lib.fp_fps_exact_static.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp]
    lib.fp_fps_exact_static.restype = i32
    lib.fp_fps_pruned_workspace_bytes.argtypes = [i32, i32]
    lib.fp_fps_pruned_workspace_bytes.restype = ctypes.c_size_t
    lib.fp_mdps_scattered_workspace_bytes.argtypes = [i32, i32]
    lib.fp_mdps_scattered_workspace_bytes.restype = ctypes.c_size_t
    lib.fp_fps_exact_pruned.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.fp_fps_exact_pruned.restype = i32
    lib.fp_mdps_sample_pruned.argtypes = [vp, i32, i32, i32, vp, ctypes.POINTER(FpMdpsParams), vp, vp, vp,
                                          ctypes.c_size_t, f32, vp, ctypes.c_size_t, vp]
    lib.fp_mdps_sample_pruned.restype = i32
    lib.fp_mdps_sample.argtypes = [vp, i32, i32, i32, vp, ctypes.POINTER(FpMdpsParams), vp, vp, vp,
                                   ctypes.c_size_t, f32, vp, ctypes.c_size_t, vp]
    lib.fp_mdps_sample.restype = i32
    lib.fp_ball_query.argtypes = [vp, i32, i32, vp, i32, f32, i32, vp, vp, vp, vp]
    lib.fp_ball_query.restype = i32
    lib.fp_ball_query_grid_workspace_bytes.argtypes = [i32, i32]
    lib.fp_ball_query_grid_workspace_bytes.restype = ctypes.c_size_t
    lib.fp_ball_query_grid.argtypes = [vp, i32, i32, vp, i32, f32, i32, vp, vp, vp, ctypes.c_size_t, vp]
    lib.fp_ball_query_grid.restype = i32
    lib.fp_knn_workspace_bytes.argtypes = [i32, i32, ctypes.c_int64]
    lib.fp_knn_workspace_bytes.restype = ctypes.c_size_t
    lib.fp_knn.argtypes = [vp, i32, i32, vp, i32, i32, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.fp_knn.restype = i32
    lib.fp_knn_grid_workspace_bytes.argtypes = [i32, i32, i32]
    lib.fp_knn_grid_workspace_bytes.restype = ctypes.c_size_t
    lib.fp_knn_grid.argtypes = [vp, i32, i32, vp, i32, i32, f32, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.fp_knn_grid.restype = i32
    lib.fp_excl_workspace_bytes.argtypes = [i32, i32, i32]
    lib.fp_excl_workspace_bytes.restype = ctypes.c_size_t
    lib.fp_excl_count.argtypes = [vp, i32, i32, vp, i32, vp, vp, ctypes.c_size_t, vp]
    lib.fp_excl_count.restype = i32
    lib.fp_excl_fill.argtypes = [vp, i32, i32, vp, i32, vp, vp, ctypes.c_int64, vp, ctypes.c_size_t, vp]
    lib.fp_excl_fill.restype = i32
    lib.fp_ball_query_lists.argtypes = [vp, vp, i32, i32, i32, i32, vp, i32, i32, vp, vp, vp]
    lib.fp_ball_query_lists.restype = i32
    lib.fp_gather_xyz.argtypes = [vp, i32, i32, vp, i32, vp, vp]
    lib.fp_gather_xyz.restype = i32
    lib.fp_coverage.argtypes = [vp, i32, i32, vp, i32, vp, vp]
    lib.fp_coverage.restype = i32
    lib.fp_probe_fp32_rate.argtypes = [i32, i32, vp, vp]
    lib.fp_probe_fp32_rate.restype = i32
    lib.fp_plan.argtypes = [i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.fp_plan.restype = i32
    lib.fp_set_wg_per_cloud.argtypes = [i32]
    lib.fp_set_wg_per_cloud.restype = None
    lib.fp_set_cooperative_launch.argtypes = [i32]
    lib.fp_set_cooperative_launch.restype = None
    lib.fp_set_wait_limit_us.argtypes = [ctypes.c_int64]
    lib.fp_set_wait_limit_us.restype = None
    lib.fp_status_string.argtypes = [i32]
    lib.fp_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(status: int, what: str) -> None:
    if status != 0:
        raise RuntimeError("%s failed: %s" % (what, load().fp_status_string(status).decode()))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _xyz(xyz: torch.Tensor) -> Tuple[int, int]:
    if not (xyz.is_cuda and xyz.dtype == torch.float32 and xyz.dim() == 3 and xyz.shape[2] == 3
            and xyz.is_contiguous()):
        raise ValueError("xyz must be a contiguous CUDA float32 tensor [B][N][3]")
    return int(xyz.shape[0]), int(xyz.shape[1])


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def plan(B: int, N: int) -> Tuple[int, int, int]:
    """(workgroups per cloud, threads per workgroup, points per thread) for B clouds of N points."""
    g, t, p = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(load().fp_plan(B, N, ctypes.byref(g), ctypes.byref(t), ctypes.byref(p)), "fp_plan")
    return g.value, t.value, p.value


def set_wg_per_cloud(g: int) -> None:
    load().fp_set_wg_per_cloud(int(g))


def probe_fp32_rate(device: torch.device, blocks: int = 8192, iterations: int = 4096, reps: int = 3) -> float:
    """Plain binary32 operations per second (multiplications and additions rounded one by one, as
    the distance update does them) that the device reaches with this build."""
    out = torch.empty(blocks * 256, dtype=torch.float32, device=device)
    best = None
    for _ in range(reps + 1):
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        _check(load().fp_probe_fp32_rate(blocks, iterations, out.data_ptr(), _stream()), "fp_probe_fp32_rate")
        b.record()
        torch.cuda.synchronize()
        t = a.elapsed_time(b)
        best = t if best is None else min(best, t)
    return blocks * 256.0 * iterations * 16.0 / (best * 1e-3)


def set_cooperative_launch(on: bool) -> None:
    load().fp_set_cooperative_launch(1 if on else 0)


def set_wait_limit_us(us: int) -> None:
    load().fp_set_wait_limit_us(int(us))


_workspaces = {}


def workspace(device: torch.device, B: int, N: int) -> torch.Tensor:
    """A cached per-device workspace tensor (calls on one device must not overlap)."""
    need = int(load().fp_workspace_bytes(B, N))
    key = (device.type, device.index)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < need:
        ws = torch.empty(need, dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def new_workspace(device: torch.device, B: int, N: int) -> torch.Tensor:
    """A workspace of its own, for sampler calls that run at the same time as others on the
    device (another stream) or inside a captured graph."""
    need = int(load().fp_workspace_bytes(B, N))
    if need == 0:
        raise ValueError("shape (B=%d, N=%d) not supported" % (B, N))
    return torch.empty(need, dtype=torch.uint8, device=device)


def new_bq_cache(xyz: torch.Tensor, n: int, entries_per_cloud: int = 0) -> torch.Tensor:
    """A ball-query cache for n samples of xyz; entries_per_cloud = 0 takes the default capacity
    (2 N + 16 n non-empty blocks of 64 radius tests per cloud)."""
    B, N = _xyz(xyz)
    need = int(load().fp_bq_cache_bytes(B, N, n, int(entries_per_cloud)))
    if need == 0:
        raise ValueError("bad shape for a ball-query cache")
    return torch.empty(need, dtype=torch.uint8, device=xyz.device)


def bq_cache_stats(cache: torch.Tensor) -> dict:
    """What a recorded ball-query cache holds (reads its header and counters back to the host):
    entries per cloud it has room for, chunks of 64 entries the sampler's wavefronts took, whether a
    cloud's record is incomplete, entries per cloud after grouping.  For sizing a cache."""
    import struct
    head = cache[:256].cpu().numpy().tobytes()
    magic, B, N, n, blocks, valid, r2_bits, order = struct.unpack_from("<Iiiiiiii", head, 0)
    cap, idx_off, cur_off, ovf_off, rowcnt_off, fill_off, rowoff_off, raw_off, rows_off, map_off, nbytes = \
        struct.unpack_from("<11q", head, 32)
    if magic != 0x46504232 or valid != 1:
        raise ValueError("not a recorded ball-query cache")
    u32 = lambda off, count: cache[off:off + 4 * count].cpu().numpy().view("uint32")
    rowoff = u32(rowoff_off, B * (n + 1)).reshape(B, n + 1)
    return {"B": B, "N": N, "n": n, "entries_capacity": int(cap), "chunks_taken": u32(cur_off, B).tolist(),
            "incomplete": [bool(v) for v in u32(ovf_off, B)], "entries": [int(v) for v in rowoff[:, n]],
            "bytes": int(nbytes), "cell_order": bool(order)}


def _start(start_idx, B, device) -> Optional[torch.Tensor]:
    if start_idx is None:
        return None
    if isinstance(start_idx, torch.Tensor):
        t = start_idx.to(device=device, dtype=torch.int32).contiguous()
    else:
        t = torch.as_tensor(start_idx, dtype=torch.int32, device=device).reshape(-1).contiguous()
    if t.numel() != B:
        raise ValueError("start_idx needs one entry per cloud")
    return t


def fps_exact(xyz: torch.Tensor, n: int, start_idx=None, want_mdc: bool = False,
              want_info: bool = False, bq_cache: Optional[torch.Tensor] = None,
              bq_radius: float = 0.0, ws: Optional[torch.Tensor] = None):
    """Exact farthest point sampling.  Returns idx [B][n] int32 (and mdc [B][n] float32,
    info bytes [B][INFO_BYTES] uint8 when asked for).  `ws`: a workspace from new_workspace
    (default: the device's shared one)."""
    B, N = _xyz(xyz)
    st = _start(start_idx, B, xyz.device)
    idx = torch.empty((B, n), dtype=torch.int32, device=xyz.device)
    mdc = torch.empty((B, n), dtype=torch.float32, device=xyz.device) if want_mdc else None
    info = torch.zeros((B, INFO_BYTES), dtype=torch.uint8, device=xyz.device) if want_info else None
    if ws is None:
        ws = workspace(xyz.device, B, N)
    _check(load().fp_fps_exact(xyz.data_ptr(), B, N, n, _ptr(st), idx.data_ptr(), _ptr(mdc), _ptr(info),
                               _ptr(bq_cache), 0 if bq_cache is None else bq_cache.numel(), float(bq_radius),
                               ws.data_ptr(), ws.numel(), _stream()),
           "fp_fps_exact")
    out = [idx]
    if want_mdc:
        out.append(mdc)
    if want_info:
        out.append(info)
    return out[0] if len(out) == 1 else tuple(out)


def fps_exact_static(xyz: torch.Tensor, n: int, out_idx: torch.Tensor, out_mdc: Optional[torch.Tensor] = None,
                     start_idx: Optional[torch.Tensor] = None) -> None:
    """fp_fps_exact_static: exact FPS into outputs the caller has allocated, the scratch memory
    being the library's own static device array (the call allocates nothing).  out_idx [B][n]
    int32, out_mdc [B][n] float32 or None, start_idx [B] int32 on the device or None."""
    B, N = _xyz(xyz)
    for t, dt in ((out_idx, torch.int32), (out_mdc, torch.float32)):
        if t is not None and not (t.is_cuda and t.dtype == dt and t.is_contiguous() and tuple(t.shape) == (B, n)):
            raise ValueError("outputs must be contiguous CUDA tensors [B][n]")
    if start_idx is not None and not (start_idx.is_cuda and start_idx.dtype == torch.int32
                                      and start_idx.is_contiguous() and start_idx.numel() == B):
        raise ValueError("start_idx must be a contiguous CUDA int32 tensor [B]")
    _check(load().fp_fps_exact_static(xyz.data_ptr(), B, N, n, _ptr(start_idx), out_idx.data_ptr(),
                                      _ptr(out_mdc), _stream()), "fp_fps_exact_static")


def fps_exact_pruned(xyz: torch.Tensor, n: int, start_idx=None, want_mdc: bool = False,
                     want_info: bool = False, ws: Optional[torch.Tensor] = None):
    """Exact farthest point sampling with pruned distance updates: the outputs of fps_exact."""
    B, N = _xyz(xyz)
    st = _start(start_idx, B, xyz.device)
    idx = torch.empty((B, n), dtype=torch.int32, device=xyz.device)
    mdc = torch.empty((B, n), dtype=torch.float32, device=xyz.device) if want_mdc else None
    info = torch.zeros((B, INFO_BYTES), dtype=torch.uint8, device=xyz.device) if want_info else None
    ws = _pruned_workspace(xyz, B, N, ws)
    _check(load().fp_fps_exact_pruned(xyz.data_ptr(), B, N, n, _ptr(st), idx.data_ptr(), _ptr(mdc), _ptr(info),
                                      ws.data_ptr(), ws.numel(), _stream()), "fp_fps_exact_pruned")
    out = [idx]
    if want_mdc:
        out.append(mdc)
    if want_info:
        out.append(info)
    return out[0] if len(out) == 1 else tuple(out)


def _pruned_workspace(xyz: torch.Tensor, B: int, N: int, ws: Optional[torch.Tensor]) -> torch.Tensor:
    need = int(load().fp_fps_pruned_workspace_bytes(B, N))
    if need == 0:
        raise ValueError("shape (B=%d, N=%d) not supported" % (B, N))
    if ws is None:
        key = ("pruned", xyz.device.type, xyz.device.index)
        ws = _workspaces.get(key)
        if ws is None or ws.numel() < need:
            ws = torch.empty(need, dtype=torch.uint8, device=xyz.device)
            _workspaces[key] = ws
    return ws


def _scattered_workspace(xyz: torch.Tensor, B: int, N: int) -> torch.Tensor:
    need = int(load().fp_mdps_scattered_workspace_bytes(B, N))
    if need == 0:
        raise ValueError("shape (B=%d, N=%d) not supported" % (B, N))
    key = ("scattered", xyz.device.type, xyz.device.index)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < need:
        ws = torch.empty(need, dtype=torch.uint8, device=xyz.device)
        _workspaces[key] = ws
    return ws


def mdps_sample_pruned(xyz: torch.Tensor, n: int, prm: MdpsParams, start_idx=None, want_info: bool = False,
                       ws: Optional[torch.Tensor] = None, bq_cache: Optional[torch.Tensor] = None,
                       bq_radius: float = 0.0):
    """Minimum distance prediction sampling with pruned distance updates: the outputs of mdps_sample."""
    B, N = _xyz(xyz)
    st = _start(start_idx, B, xyz.device)
    idx = torch.empty((B, n), dtype=torch.int32, device=xyz.device)
    info = torch.zeros((B, INFO_BYTES), dtype=torch.uint8, device=xyz.device) if want_info else None
    ws = _pruned_workspace(xyz, B, N, ws)
    c = prm.to_c()
    _check(load().fp_mdps_sample_pruned(xyz.data_ptr(), B, N, n, _ptr(st), ctypes.byref(c), idx.data_ptr(),
                                        _ptr(info), _ptr(bq_cache), 0 if bq_cache is None else bq_cache.numel(),
                                        float(bq_radius), ws.data_ptr(), ws.numel(), _stream()),
           "fp_mdps_sample_pruned")
    return (idx, info) if want_info else idx


def mdps_sample(xyz: torch.Tensor, n: int, prm: MdpsParams, start_idx=None, want_info: bool = False,
                bq_cache: Optional[torch.Tensor] = None, bq_radius: float = 0.0,
                ws: Optional[torch.Tensor] = None):
    """Minimum distance prediction sampling.  Returns idx [B][n] int32 (and info bytes)."""
    B, N = _xyz(xyz)
    st = _start(start_idx, B, xyz.device)
    idx = torch.empty((B, n), dtype=torch.int32, device=xyz.device)
    info = torch.zeros((B, INFO_BYTES), dtype=torch.uint8, device=xyz.device) if want_info else None
    if ws is None:
        ws = _scattered_workspace(xyz, B, N) if prm.scan_order == 1 else workspace(xyz.device, B, N)
    c = prm.to_c()
    _check(load().fp_mdps_sample(xyz.data_ptr(), B, N, n, _ptr(st), ctypes.byref(c), idx.data_ptr(),
                                 _ptr(info), _ptr(bq_cache), 0 if bq_cache is None else bq_cache.numel(),
                                 float(bq_radius), ws.data_ptr(), ws.numel(), _stream()), "fp_mdps_sample")
    return (idx, info) if want_info else idx


def ball_query(xyz: torch.Tensor, center_idx: torch.Tensor, radius: float, k: int,
               bq_cache: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Ball query: (idx [B][M][k] int32, cnt [B][M] int32)."""
    B, N = _xyz(xyz)
    if not (center_idx.is_cuda and center_idx.dtype == torch.int32 and center_idx.dim() == 2
            and center_idx.shape[0] == B and center_idx.is_contiguous()):
        raise ValueError("center_idx must be a contiguous CUDA int32 tensor [B][M]")
    M = int(center_idx.shape[1])
    idx = torch.empty((B, M, k), dtype=torch.int32, device=xyz.device)
    cnt = torch.empty((B, M), dtype=torch.int32, device=xyz.device)
    _check(load().fp_ball_query(xyz.data_ptr(), B, N, center_idx.data_ptr(), M, float(radius), k,
                                idx.data_ptr(), cnt.data_ptr(), _ptr(bq_cache), _stream()),
           "fp_ball_query")
    return idx, cnt


def ball_query_grid(xyz: torch.Tensor, center_idx: torch.Tensor, radius: float, k: int,
                    ws: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Ball query through a uniform grid: the outputs of ball_query without a cache."""
    B, N = _xyz(xyz)
    if not (center_idx.is_cuda and center_idx.dtype == torch.int32 and center_idx.dim() == 2
            and center_idx.shape[0] == B and center_idx.is_contiguous()):
        raise ValueError("center_idx must be a contiguous CUDA int32 tensor [B][M]")
    M = int(center_idx.shape[1])
    idx = torch.empty((B, M, k), dtype=torch.int32, device=xyz.device)
    cnt = torch.empty((B, M), dtype=torch.int32, device=xyz.device)
    need = int(load().fp_ball_query_grid_workspace_bytes(B, N))
    if need == 0:
        raise ValueError("shape (B=%d, N=%d) not supported" % (B, N))
    if ws is None:
        key = ("grid", xyz.device.type, xyz.device.index)
        ws = _workspaces.get(key)
        if ws is None or ws.numel() < need:
            ws = torch.empty(need, dtype=torch.uint8, device=xyz.device)
            _workspaces[key] = ws
    _check(load().fp_ball_query_grid(xyz.data_ptr(), B, N, _ptr(center_idx) if M else None, M, float(radius), k,
                                     _ptr(idx) if M else None, _ptr(cnt) if M else None, ws.data_ptr(), ws.numel(),
                                     _stream()), "fp_ball_query_grid")
    return idx, cnt


def knn(xyz: torch.Tensor, sample_idx: torch.Tensor, k: int, bq_cache: Optional[torch.Tensor] = None,
        want_deferred: bool = False):
    """k nearest samples of every point: (pos [B][N][k] int32 positions into sample_idx,
    d2 [B][N][k] float32); with want_deferred also the per-cloud number of points that the
    cached search handed to the brute-force pass."""
    B, N = _xyz(xyz)
    if not (sample_idx.is_cuda and sample_idx.dtype == torch.int32 and sample_idx.dim() == 2
            and sample_idx.shape[0] == B and sample_idx.is_contiguous()):
        raise ValueError("sample_idx must be a contiguous CUDA int32 tensor [B][n]")
    n = int(sample_idx.shape[1])
    pos = torch.empty((B, N, k), dtype=torch.int32, device=xyz.device)
    d2 = torch.empty((B, N, k), dtype=torch.float32, device=xyz.device)
    ws, ws_bytes, deferred = None, 0, None
    if bq_cache is not None:
        entries = int(load().fp_bq_cache_entries(bq_cache.numel(), B, N, n))
        ws_bytes = int(load().fp_knn_workspace_bytes(B, N, entries))
        if ws_bytes == 0:
            raise ValueError("shape (B=%d, N=%d) not supported" % (B, N))
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=xyz.device)
        deferred = torch.zeros(B, dtype=torch.int32, device=xyz.device)
    _check(load().fp_knn(xyz.data_ptr(), B, N, sample_idx.data_ptr(), n, k, pos.data_ptr(), d2.data_ptr(),
                         _ptr(bq_cache), _ptr(deferred), _ptr(ws), ws_bytes, _stream()), "fp_knn")
    return (pos, d2, deferred) if want_deferred else (pos, d2)


def excl_lists(xyz: torch.Tensor, thr2: torch.Tensor, ws: Optional[torch.Tensor] = None):
    """Exclusion lists for the squared radii thr2 [B][L] (float32, on the device):
    (offsets [L*B*N + 1] int64, entries int32); row (l*B + b)*N + i holds the points j of
    cloud b with dist^2(i, j) < thr2[b][l], ascending.  Reads the total back between the two
    passes (one synchronisation) to size `entries`."""
    B, N = _xyz(xyz)
    if not (thr2.is_cuda and thr2.dtype == torch.float32 and thr2.dim() == 2 and thr2.shape[0] == B
            and thr2.is_contiguous()):
        raise ValueError("thr2 must be a contiguous CUDA float32 tensor [B][L]")
    L = int(thr2.shape[1])
    need = int(load().fp_excl_workspace_bytes(B, N, L))
    if need == 0:
        raise ValueError("shape (B=%d, N=%d, L=%d) not supported" % (B, N, L))
    if ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device=xyz.device)
    offsets = torch.empty(L * B * N + 1, dtype=torch.int64, device=xyz.device)
    _check(load().fp_excl_count(xyz.data_ptr(), B, N, thr2.data_ptr(), L, offsets.data_ptr(), ws.data_ptr(),
                                ws.numel(), _stream()), "fp_excl_count")
    total = int(offsets[-1].item())
    entries = torch.empty(max(total, 1), dtype=torch.int32, device=xyz.device)
    _check(load().fp_excl_fill(xyz.data_ptr(), B, N, thr2.data_ptr(), L, offsets.data_ptr(), entries.data_ptr(),
                               total, ws.data_ptr(), ws.numel(), _stream()), "fp_excl_fill")
    return offsets, entries[:total]


def ball_query_lists(offsets: torch.Tensor, entries: torch.Tensor, B: int, N: int, L: int, level: int,
                     center_idx: torch.Tensor, k: int) -> Tuple[torch.Tensor, torch.Tensor]:
    """Ball query by lookup in exclusion lists: (idx [B][M][k] int32, cnt [B][M] int32)."""
    if not (center_idx.is_cuda and center_idx.dtype == torch.int32 and center_idx.dim() == 2
            and center_idx.shape[0] == B and center_idx.is_contiguous()):
        raise ValueError("center_idx must be a contiguous CUDA int32 tensor [B][M]")
    if offsets.numel() != L * B * N + 1 or offsets.dtype != torch.int64 or entries.dtype != torch.int32:
        raise ValueError("offsets / entries do not belong to lists of this shape")
    M = int(center_idx.shape[1])
    idx = torch.empty((B, M, k), dtype=torch.int32, device=center_idx.device)
    cnt = torch.empty((B, M), dtype=torch.int32, device=center_idx.device)
    ent = entries if entries.numel() > 0 else torch.zeros(1, dtype=torch.int32, device=center_idx.device)
    _check(load().fp_ball_query_lists(offsets.data_ptr(), ent.data_ptr(), B, N, level, L, center_idx.data_ptr(),
                                      M, k, idx.data_ptr(), cnt.data_ptr(), _stream()), "fp_ball_query_lists")
    return idx, cnt


def knn_grid(xyz: torch.Tensor, sample_idx: torch.Tensor, k: int, radius: float, want_deferred: bool = False):
    """k nearest samples through a grid over the samples (cells as wide as `radius`): the
    outputs of knn; with want_deferred also the per-cloud number of points the grid did not
    settle."""
    B, N = _xyz(xyz)
    if not (sample_idx.is_cuda and sample_idx.dtype == torch.int32 and sample_idx.dim() == 2
            and sample_idx.shape[0] == B and sample_idx.is_contiguous()):
        raise ValueError("sample_idx must be a contiguous CUDA int32 tensor [B][n]")
    n = int(sample_idx.shape[1])
    pos = torch.empty((B, N, k), dtype=torch.int32, device=xyz.device)
    d2 = torch.empty((B, N, k), dtype=torch.float32, device=xyz.device)
    need = int(load().fp_knn_grid_workspace_bytes(B, N, n))
    if need == 0:
        raise ValueError("shape (B=%d, N=%d, n=%d) not supported" % (B, N, n))
    ws = torch.empty(need, dtype=torch.uint8, device=xyz.device)
    deferred = torch.zeros(B, dtype=torch.int32, device=xyz.device)
    _check(load().fp_knn_grid(xyz.data_ptr(), B, N, sample_idx.data_ptr(), n, k, float(radius), pos.data_ptr(),
                              d2.data_ptr(), deferred.data_ptr(), ws.data_ptr(), need, _stream()), "fp_knn_grid")
    return (pos, d2, deferred) if want_deferred else (pos, d2)


def gather_xyz(xyz: torch.Tensor, idx: torch.Tensor) -> torch.Tensor:
    B, N = _xyz(xyz)
    M = int(idx.shape[1])
    out = torch.empty((B, M, 3), dtype=torch.float32, device=xyz.device)
    _check(load().fp_gather_xyz(xyz.data_ptr(), B, N, idx.data_ptr(), M, out.data_ptr(), _stream()),
           "fp_gather_xyz")
    return out


def coverage2(xyz: torch.Tensor, idx: torch.Tensor) -> torch.Tensor:
    """Squared coverage radius per cloud, [B] float32: max over points of the squared
    distance to the nearest sample."""
    B, N = _xyz(xyz)
    s = gather_xyz(xyz, idx)
    out = torch.empty(B, dtype=torch.float32, device=xyz.device)
    _check(load().fp_coverage(xyz.data_ptr(), B, N, s.data_ptr(), int(idx.shape[1]), out.data_ptr(),
                              _stream()), "fp_coverage")
    return out


def parse_info(info: torch.Tensor):
    """Host copies of the per-cloud info records as FpMdpsInfo structures."""
    raw = info.cpu().numpy().tobytes()
    return [FpMdpsInfo.from_buffer_copy(raw[i * INFO_BYTES:(i + 1) * INFO_BYTES])
            for i in range(info.shape[0])]
