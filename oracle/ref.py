"""ctypes access to the CPU oracle (oracle/fastpoint_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module.
Every function takes and returns numpy arrays on the host; batches are plain
Python loops over clouds.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
from typing import Optional, Sequence, Tuple

import numpy as np

from . import build as _build

MAX_SEG = 16


class _Params(ctypes.Structure):
    _fields_ = [("p", ctypes.c_float), ("nseg", ctypes.c_int32), ("exponent", ctypes.c_double),
                ("bias", ctypes.c_float), ("fit_window", ctypes.c_int32), ("m_min", ctypes.c_int32),
                ("use_override", ctypes.c_int32), ("thr_override", ctypes.c_float * MAX_SEG),
                ("level_scale", ctypes.c_float * MAX_SEG),
                ("mlp", ctypes.POINTER(ctypes.c_float)), ("scan_order", ctypes.c_int32)]


MLP_WEIGHTS = 32 * 128 + 128 + 128 * 128 + 128 + 128 * 64 + 64


class _Info(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int32), ("et_index", ctypes.c_int32),
                ("level_start", ctypes.c_int32 * MAX_SEG),
                ("level_exhausted", ctypes.c_int32 * MAX_SEG),
                ("thr2", ctypes.c_float * MAX_SEG)]


@dataclasses.dataclass
class MdpsParams:
    p: float = 0.1
    nseg: int = 6
    exponent: float = 1.0
    bias: float = 1.0
    fit_window: int = 32
    m_min: int = 8
    thr_override: Optional[Sequence[float]] = None
    level_scale: Optional[Sequence[float]] = None
    mlp: Optional[np.ndarray] = None      # MLP_WEIGHTS float32 weights of the MLP estimator, or None
    scan_order: int = 0                   # threshold phase: 0 lowest available index, 1 scattered walk

    def to_c(self) -> _Params:
        c = _Params()
        if self.mlp is not None:
            w = np.ascontiguousarray(self.mlp, dtype=np.float32).reshape(-1)
            assert w.shape[0] == MLP_WEIGHTS
            c._keep = w                      # the structure only holds a pointer
            c.mlp = w.ctypes.data_as(ctypes.POINTER(ctypes.c_float))
        for i in range(MAX_SEG):
            c.level_scale[i] = 1.0
        if self.level_scale is not None:
            assert len(self.level_scale) == self.nseg
            for i, v in enumerate(self.level_scale):
                c.level_scale[i] = v
        c.p, c.nseg, c.exponent, c.bias = self.p, self.nseg, self.exponent, self.bias
        c.fit_window, c.m_min = self.fit_window, self.m_min
        c.scan_order = self.scan_order
        c.use_override = 0
        if self.thr_override is not None:
            assert len(self.thr_override) == self.nseg
            c.use_override = 1
            for i, v in enumerate(self.thr_override):
                c.thr_override[i] = v
        return c


@dataclasses.dataclass
class MdpsInfo:
    m: int
    et_index: int
    level_start: np.ndarray
    level_exhausted: np.ndarray
    thr2: np.ndarray


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build.build())
        fp = ctypes.POINTER(ctypes.c_float)
        ip = ctypes.POINTER(ctypes.c_int32)
        i32 = ctypes.c_int32
        _lib.ref_fps_exact.argtypes = [fp, i32, i32, i32, ip, fp]
        _lib.ref_pow_int_base.argtypes = [ctypes.c_int64, ctypes.c_double]
        _lib.ref_pow_int_base.restype = ctypes.c_double
        _lib.ref_ln_fixed.argtypes = [ctypes.c_double]
        _lib.ref_ln_fixed.restype = ctypes.c_double
        _lib.ref_exp_fixed.argtypes = [ctypes.c_double]
        _lib.ref_exp_fixed.restype = ctypes.c_double
        _lib.ref_mlp_curve.argtypes = [fp, i32, fp, ctypes.POINTER(ctypes.c_double)]
        _lib.ref_scan_stride.argtypes = [i32]
        _lib.ref_scan_stride.restype = ctypes.c_int64
        _lib.ref_mdps_prefix_len.argtypes = [ctypes.POINTER(_Params), i32]
        _lib.ref_mdps_thresholds.argtypes = [fp, i32, i32, ctypes.POINTER(_Params), fp]
        _lib.ref_mdps_sample.argtypes = [fp, i32, i32, i32, ctypes.POINTER(_Params), ip,
                                         ctypes.POINTER(_Info)]
        _lib.ref_mdps_literal.argtypes = _lib.ref_mdps_sample.argtypes
        _lib.ref_ball_query.argtypes = [fp, i32, ip, i32, ctypes.c_float, i32, ip, ip]
        _lib.ref_gather_xyz.argtypes = [fp, i32, ip, i32, fp]
        lp = ctypes.POINTER(ctypes.c_int64)
        _lib.ref_excl_lists.argtypes = [fp, i32, fp, i32, lp, ip, ctypes.c_int64]
        _lib.ref_ball_query_lists.argtypes = [lp, ip, i32, i32, ip, i32, i32, ip, ip]
        _lib.ref_knn.argtypes = [fp, i32, ip, i32, i32, ip, i32, ip, fp]
        _lib.ref_coverage_radius.argtypes = [fp, i32, ip, i32]
        _lib.ref_coverage_radius.restype = ctypes.c_double
        _lib.ref_mean_spacing.argtypes = [fp, ip, i32]
        _lib.ref_mean_spacing.restype = ctypes.c_double
    return _lib


def _f(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _i(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _cloud(xyz) -> np.ndarray:
    a = np.ascontiguousarray(xyz, dtype=np.float32)
    assert a.ndim == 2 and a.shape[1] == 3
    return a


def fps_exact(xyz, n: int, start: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Algorithm 1 on one cloud: (idx[n] int32, mdc[n] float32 squared)."""
    a = _cloud(xyz)
    idx = np.empty(n, dtype=np.int32)
    mdc = np.empty(n, dtype=np.float32)
    rc = lib().ref_fps_exact(_f(a), a.shape[0], n, start, _i(idx), _f(mdc))
    if rc != 0:
        raise ValueError("ref_fps_exact rejected its arguments")
    return idx, mdc


def pow_int_base(x: int, e: float) -> float:
    """x^e for an integer x >= 1 by the oracle's fixed-order series."""
    return float(lib().ref_pow_int_base(int(x), float(e)))


def ln_fixed(v: float) -> float:
    return float(lib().ref_ln_fixed(float(v)))


def exp_fixed(y: float) -> float:
    return float(lib().ref_exp_fixed(float(y)))


def mlp_curve(mdc, m: int, weights) -> np.ndarray:
    """Output layer of the MLP estimator (64 log-ratios) for the prefix curve mdc[0..m]."""
    a = np.ascontiguousarray(mdc, dtype=np.float32)
    w = np.ascontiguousarray(weights, dtype=np.float32).reshape(-1)
    assert w.shape[0] == MLP_WEIGHTS and a.shape[0] >= m + 1
    out = np.empty(64, dtype=np.float64)
    rc = lib().ref_mlp_curve(_f(a), m, _f(w), out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise ValueError("ref_mlp_curve rejected its arguments")
    return out


def scan_stride(N: int) -> int:
    """Stride A of the scattered scan order j_t = (t * A) mod N of a cloud of N points."""
    return int(lib().ref_scan_stride(int(N)))


def mdps_prefix_len(prm: MdpsParams, n: int) -> int:
    c = prm.to_c()
    return int(lib().ref_mdps_prefix_len(ctypes.byref(c), n))


def mdps_thresholds(mdc, n: int, m: int, prm: MdpsParams) -> np.ndarray:
    a = np.ascontiguousarray(mdc, dtype=np.float32)
    assert a.shape[0] >= m + 1
    out = np.empty(prm.nseg, dtype=np.float32)
    c = prm.to_c()
    rc = lib().ref_mdps_thresholds(_f(a), n, m, ctypes.byref(c), _f(out))
    if rc != 0:
        raise ValueError("ref_mdps_thresholds rejected its arguments")
    return out


def _mdps(fn, xyz, n, start, prm) -> Tuple[np.ndarray, MdpsInfo]:
    a = _cloud(xyz)
    idx = np.empty(n, dtype=np.int32)
    c = prm.to_c()
    info = _Info()
    rc = fn(_f(a), a.shape[0], n, start, ctypes.byref(c), _i(idx), ctypes.byref(info))
    if rc != 0:
        raise ValueError("oracle MDPS rejected its arguments")
    return idx, MdpsInfo(int(info.m), int(info.et_index),
                         np.array(info.level_start[:prm.nseg], dtype=np.int32),
                         np.array(info.level_exhausted[:prm.nseg], dtype=np.int32),
                         np.array(info.thr2[:prm.nseg], dtype=np.float32))


def mdps_sample(xyz, n: int, prm: MdpsParams, start: int = 0) -> Tuple[np.ndarray, MdpsInfo]:
    """Algorithm 2, running-min-distance form, one cloud."""
    return _mdps(lib().ref_mdps_sample, xyz, n, start, prm)


def mdps_literal(xyz, n: int, prm: MdpsParams, start: int = 0) -> Tuple[np.ndarray, MdpsInfo]:
    """Algorithm 2 with explicit exclusion lists and bitmaps (O(N^2); tiny clouds)."""
    return _mdps(lib().ref_mdps_literal, xyz, n, start, prm)


def ball_query(xyz, centers, radius: float, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """(idx[M][k] int32, cnt[M] int32) for one cloud."""
    a = _cloud(xyz)
    c = np.ascontiguousarray(centers, dtype=np.int32)
    M = c.shape[0]
    idx = np.empty((M, k), dtype=np.int32)
    cnt = np.empty(M, dtype=np.int32)
    rc = lib().ref_ball_query(_f(a), a.shape[0], _i(c), M, np.float32(radius), k, _i(idx), _i(cnt))
    if rc != 0:
        raise ValueError("ref_ball_query rejected its arguments")
    return idx, cnt


def excl_lists(xyz, thr2) -> Tuple[np.ndarray, np.ndarray]:
    """Exclusion lists of one cloud for the squared radii thr2[L] (the list-building loops of Alg. 2):
    (offsets[L*N+1] int64, entries int32); row l*N+i holds the j with dist2(i,j) < thr2[l],
    ascending."""
    a = _cloud(xyz)
    t = np.ascontiguousarray(thr2, dtype=np.float32).reshape(-1)
    N, L = a.shape[0], t.shape[0]
    off = np.empty(L * N + 1, dtype=np.int64)
    lp = ctypes.POINTER(ctypes.c_int64)
    rc = lib().ref_excl_lists(_f(a), N, _f(t), L, off.ctypes.data_as(lp), None, 0)
    if rc != 0:
        raise ValueError("ref_excl_lists rejected its arguments")
    ent = np.empty(max(int(off[-1]), 1), dtype=np.int32)
    rc = lib().ref_excl_lists(_f(a), N, _f(t), L, off.ctypes.data_as(lp), _i(ent), ent.shape[0])
    if rc != 0:
        raise ValueError("ref_excl_lists failed (%d)" % rc)
    return off, ent[:int(off[-1])]


def ball_query_lists(offsets, entries, N: int, level: int, centers, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Ball query by lookup in the exclusion lists: (idx[M][k] int32, cnt[M] int32)."""
    off = np.ascontiguousarray(offsets, dtype=np.int64)
    ent = np.ascontiguousarray(entries, dtype=np.int32)
    if ent.shape[0] == 0:
        ent = np.zeros(1, dtype=np.int32)
    c = np.ascontiguousarray(centers, dtype=np.int32)
    M = c.shape[0]
    idx = np.empty((M, k), dtype=np.int32)
    cnt = np.empty(M, dtype=np.int32)
    rc = lib().ref_ball_query_lists(off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), _i(ent), N, level,
                                    _i(c), M, k, _i(idx), _i(cnt))
    if rc != 0:
        raise ValueError("ref_ball_query_lists rejected its arguments")
    return idx, cnt


def knn(xyz, sample_idx, k: int, points=None) -> Tuple[np.ndarray, np.ndarray]:
    """k nearest samples of every point of one cloud (or of the points listed in `points`):
    (pos[M][k] int32 positions into sample_idx, d2[M][k] float32 squared distances), nearest
    first, lower position on ties."""
    a = _cloud(xyz)
    s = np.ascontiguousarray(sample_idx, dtype=np.int32)
    N, n = a.shape[0], s.shape[0]
    pts = None if points is None else np.ascontiguousarray(points, dtype=np.int32)
    M = N if pts is None else pts.shape[0]
    pos = np.empty((M, k), dtype=np.int32)
    d2 = np.empty((M, k), dtype=np.float32)
    rc = lib().ref_knn(_f(a), N, _i(s), n, k, None if pts is None else _i(pts), M, _i(pos), _f(d2))
    if rc != 0:
        raise ValueError("ref_knn rejected its arguments")
    return pos, d2


def gather_xyz(xyz, idx) -> np.ndarray:
    a = _cloud(xyz)
    c = np.ascontiguousarray(idx, dtype=np.int32)
    out = np.empty((c.shape[0], 3), dtype=np.float32)
    rc = lib().ref_gather_xyz(_f(a), a.shape[0], _i(c), c.shape[0], _f(out))
    if rc != 0:
        raise ValueError("ref_gather_xyz rejected its arguments")
    return out


def coverage_radius(xyz, idx) -> float:
    a = _cloud(xyz)
    c = np.ascontiguousarray(idx, dtype=np.int32)
    return float(lib().ref_coverage_radius(_f(a), a.shape[0], _i(c), c.shape[0]))


def mean_spacing(xyz, idx) -> float:
    a = _cloud(xyz)
    c = np.ascontiguousarray(idx, dtype=np.int32)
    return float(lib().ref_mean_spacing(_f(a), _i(c), c.shape[0]))
