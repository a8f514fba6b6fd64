"""Seeded synthetic point clouds for the five workloads.

This module only draws random geometry.  It holds none of the sampling or
neighbour-search arithmetic, so both the CPU oracle's tests and the HIP path
can take their inputs from it without sharing any of the method.

Every cloud is float32 ``[B][N][3]`` (row-major, 12 bytes per point).  The
shapes stand in for the data sets the paper measures on (Section 5.1): they
keep the point counts, sampling ratios, value ranges and index ordering
(shuffled object scans, surface-by-surface indoor scans, ring-major LiDAR
sweeps) of those workloads; none of their records is reproduced.

Cloud ``b`` of workload ``c`` is drawn from ``numpy.random.Generator(PCG64(
BASE_SEED + 1000*c + b))``; calibration clouds (used to fit the curve
exponent, the stand-in for the paper's "training split") add 500000.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Tuple

import numpy as np

BASE_SEED = 20250723
CALIBRATION_OFFSET = 500000


@dataclasses.dataclass(frozen=True)
class Stage:
    """One sampling + ball-query stage: N points -> n samples, radius, k."""
    n: int
    radius: float
    k: int


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    B: int
    N: int
    stages: Tuple[Stage, ...]
    description: str


WORKLOADS = {
    "C1": Workload("C1", 1, 4096, (Stage(1024, 0.1, 32),),
                   "single cloud, uniform in the unit cube"),
    "C2": Workload("C2", 16, 1024, (Stage(512, 0.2, 32), Stage(128, 0.4, 64)),
                   "object-classification shape: surfaces of random primitives, unit sphere"),
    "C3": Workload("C3", 8, 24000,
                   (Stage(6000, 0.1, 32), Stage(1500, 0.2, 32), Stage(375, 0.4, 32), Stage(94, 0.8, 32)),
                   "indoor-scene shape: 5x5x3 m room with boxes, surface-ordered"),
    "C4": Workload("C4", 4, 120000, (Stage(16384, 1.0, 16),),
                   "outdoor LiDAR-like sweep: 64 rings, ring-major order"),
    "C5": Workload("C5", 1, 1000000, (Stage(65536, 0.5, 32),),
                   "large single cloud: 200 anisotropic Gaussian clusters + uniform background"),
}


def _rng(cfg: int, b: int, calibration: bool) -> np.random.Generator:
    seed = BASE_SEED + 1000 * cfg + b + (CALIBRATION_OFFSET if calibration else 0)
    return np.random.Generator(np.random.PCG64(seed))


def _random_rotation(rng: np.random.Generator) -> np.ndarray:
    """Uniform random rotation matrix (QR of a Gaussian matrix, sign-fixed)."""
    q, r = np.linalg.qr(rng.standard_normal((3, 3)))
    q = q * np.sign(np.diag(r))
    if np.linalg.det(q) < 0:
        q[:, 0] = -q[:, 0]
    return q


# --------------------------------------------------------------------------- C1
def _cloud_c1(rng: np.random.Generator, N: int) -> np.ndarray:
    return rng.random((N, 3))


# --------------------------------------------------------------------------- C2
def _sphere_surface(rng, m):
    v = rng.standard_normal((m, 3))
    return v / np.linalg.norm(v, axis=1, keepdims=True)


def _box_surface(rng, m, half):
    """Area-uniform points on the surface of a box with half extents `half`."""
    hx, hy, hz = half
    areas = np.array([hy * hz, hy * hz, hx * hz, hx * hz, hx * hy, hx * hy])
    face = rng.choice(6, size=m, p=areas / areas.sum())
    u = rng.uniform(-1.0, 1.0, (m, 2))
    pts = np.empty((m, 3))
    axis = face // 2
    sign = np.where(face % 2 == 0, -1.0, 1.0)
    for a in range(3):
        sel = axis == a
        others = [d for d in range(3) if d != a]
        pts[sel, a] = sign[sel] * half[a]
        pts[sel, others[0]] = u[sel, 0] * half[others[0]]
        pts[sel, others[1]] = u[sel, 1] * half[others[1]]
    return pts


def _cylinder_surface(rng, m, radius, half_h):
    side = 2.0 * math.pi * radius * 2.0 * half_h
    cap = math.pi * radius * radius
    part = rng.choice(3, size=m, p=np.array([side, cap, cap]) / (side + 2 * cap))
    theta = rng.uniform(0.0, 2.0 * math.pi, m)
    rad = np.where(part == 0, radius, radius * np.sqrt(rng.random(m)))
    z = np.where(part == 0, rng.uniform(-half_h, half_h, m), np.where(part == 1, -half_h, half_h))
    return np.stack([rad * np.cos(theta), rad * np.sin(theta), z], axis=1)


def _cloud_c2(rng: np.random.Generator, N: int) -> np.ndarray:
    nprim = int(rng.integers(1, 5))
    prims = []
    for _ in range(nprim):
        kind = int(rng.integers(0, 3))
        scale = rng.uniform(0.3, 1.0)
        rot = _random_rotation(rng)
        off = rng.uniform(-0.5, 0.5, 3)
        if kind == 0:
            area = 4.0 * math.pi * scale * scale
            shape = ("sphere", scale)
        elif kind == 1:
            half = scale * rng.uniform(0.3, 1.0, 3)
            area = 8.0 * (half[0] * half[1] + half[1] * half[2] + half[0] * half[2])
            shape = ("box", half)
        else:
            radius = scale * rng.uniform(0.2, 0.6)
            half_h = scale * rng.uniform(0.3, 1.0)
            area = 2.0 * math.pi * radius * (2.0 * half_h) + 2.0 * math.pi * radius * radius
            shape = ("cyl", radius, half_h)
        prims.append((shape, rot, off, area))
    areas = np.array([p[3] for p in prims])
    which = rng.choice(nprim, size=N, p=areas / areas.sum())
    pts = np.empty((N, 3))
    for i, (shape, rot, off, _) in enumerate(prims):
        sel = np.nonzero(which == i)[0]
        m = sel.size
        if m == 0:
            continue
        if shape[0] == "sphere":
            local = shape[1] * _sphere_surface(rng, m)
        elif shape[0] == "box":
            local = _box_surface(rng, m, shape[1])
        else:
            local = _cylinder_surface(rng, m, shape[1], shape[2])
        pts[sel] = local @ rot.T + off
    pts -= pts.mean(axis=0, keepdims=True)
    pts /= np.linalg.norm(pts, axis=1).max()
    return pts[rng.permutation(N)]


# --------------------------------------------------------------------------- C3
def _room_surfaces(rng) -> List[Tuple[np.ndarray, np.ndarray, np.ndarray]]:
    """Rectangles (origin, edge_u, edge_v) of a 5x5x3 m room with boxes on the floor."""
    X, Y, Z = 5.0, 5.0, 3.0
    o = np.array
    rects = [
        (o([0, 0, 0.0]), o([X, 0, 0.0]), o([0, Y, 0.0])),        # floor
        (o([0, 0, Z]), o([X, 0, 0.0]), o([0, Y, 0.0])),          # ceiling
        (o([0, 0, 0.0]), o([X, 0, 0.0]), o([0, 0, Z])),          # wall y=0
        (o([0, Y, 0.0]), o([X, 0, 0.0]), o([0, 0, Z])),          # wall y=Y
        (o([0, 0, 0.0]), o([0, Y, 0.0]), o([0, 0, Z])),          # wall x=0
        (o([X, 0, 0.0]), o([0, Y, 0.0]), o([0, 0, Z])),          # wall x=X
    ]
    for _ in range(int(rng.integers(10, 31))):
        e = rng.uniform(0.2, 1.5, 3)
        c = np.array([rng.uniform(0, X - e[0]), rng.uniform(0, Y - e[1]), 0.0])
        ex, ey, ez = o([e[0], 0, 0.0]), o([0, e[1], 0.0]), o([0, 0, e[2]])
        rects += [
            (c + ez, ex, ey),            # top
            (c, ex, ez), (c + ey, ex, ez),
            (c, ey, ez), (c + ex, ey, ez),
        ]
    return rects


def _cloud_c3(rng: np.random.Generator, N: int) -> np.ndarray:
    rects = _room_surfaces(rng)

    def accept_prob(x):          # density rises 4x along x
        return 0.25 + 0.75 * np.clip(x / 5.0, 0.0, 1.0)

    # effective area of each rectangle under the acceptance density
    eff = []
    for org, eu, ev in rects:
        x0, x1 = org[0], org[0] + eu[0] + ev[0]
        area = np.linalg.norm(np.cross(eu, ev))
        eff.append(area * 0.5 * (accept_prob(np.array(x0)) + accept_prob(np.array(x1))))
    eff = np.array(eff)
    counts = rng.multinomial(N, eff / eff.sum())
    chunks = []
    for (org, eu, ev), m in zip(rects, counts):
        got = np.empty((0, 3))
        while got.shape[0] < m:
            uv = rng.random((2 * (m - got.shape[0]) + 16, 2))
            cand = org + uv[:, :1] * eu + uv[:, 1:] * ev
            keep = rng.random(cand.shape[0]) < accept_prob(cand[:, 0])
            got = np.concatenate([got, cand[keep]], axis=0)
        got = got[:m]
        # raster order inside a surface: 5 cm bands along v, then along u
        lu = (got - org) @ eu / max(eu @ eu, 1e-12)
        lv = (got - org) @ ev / max(ev @ ev, 1e-12)
        band = np.floor(lv * np.linalg.norm(ev) / 0.05)
        order = np.lexsort((lu, band))
        chunks.append(got[order])
    pts = np.concatenate(chunks, axis=0)
    pts += rng.normal(0.0, 0.005, pts.shape)
    return pts


# --------------------------------------------------------------------------- C4
def _cloud_c4(rng: np.random.Generator, N: int) -> np.ndarray:
    nbox = int(rng.integers(20, 61))
    foot = rng.uniform(1.0, 6.0, (nbox, 2))
    height = rng.uniform(1.0, 4.0, nbox)
    ang = rng.uniform(0.0, 2.0 * math.pi, nbox)
    rad = rng.uniform(4.0, 48.0, nbox)
    cxy = np.stack([rad * np.cos(ang), rad * np.sin(ang)], axis=1)
    lo = np.concatenate([cxy - 0.5 * foot, np.zeros((nbox, 1))], axis=1)
    hi = np.concatenate([cxy + 0.5 * foot, height[:, None]], axis=1)

    rings = 64
    az_steps = 4000
    elev = np.deg2rad(np.linspace(-24.0, 2.0, rings))
    az = np.linspace(0.0, 2.0 * math.pi, az_steps, endpoint=False)
    origin = np.array([0.0, 0.0, 1.7])
    ce, se = np.cos(elev)[:, None], np.sin(elev)[:, None]
    d = np.stack([ce * np.cos(az)[None, :], ce * np.sin(az)[None, :],
                  np.broadcast_to(se, (rings, az_steps))], axis=2).reshape(-1, 3)   # ring-major
    t = np.full(d.shape[0], np.inf)
    down = d[:, 2] < -1e-9
    t[down] = -origin[2] / d[down, 2]
    with np.errstate(divide="ignore", invalid="ignore"):
        inv = 1.0 / d
        for b in range(nbox):
            t0 = (lo[b] - origin) * inv
            t1 = (hi[b] - origin) * inv
            tn = np.nanmax(np.minimum(t0, t1), axis=1)
            tf = np.nanmin(np.maximum(t0, t1), axis=1)
            hit = (tn <= tf) & (tn > 0.0)
            t = np.where(hit & (tn < t), tn, t)
    t = t + rng.normal(0.0, 0.02, t.shape)
    ok = np.isfinite(t) & (t > 0.5) & (t <= 50.0)
    pts = origin + t[ok, None] * d[ok]
    if pts.shape[0] < N:
        raise RuntimeError("LiDAR generator produced too few returns: %d" % pts.shape[0])
    keep = np.sort(rng.choice(pts.shape[0], size=N, replace=False))   # order-preserving decimation
    return pts[keep]


# --------------------------------------------------------------------------- C5
def _cloud_c5(rng: np.random.Generator, N: int) -> np.ndarray:
    K = 200
    L = 100.0
    centers = rng.uniform(0.0, L, (K, 3))
    weights = rng.uniform(0.2, 1.0, K)
    sig = np.exp(rng.uniform(math.log(0.3), math.log(5.0), (K, 3)))
    rots = np.stack([_random_rotation(rng) for _ in range(K)])
    n_bg = N // 10
    n_cl = N - n_bg
    comp = rng.choice(K, size=n_cl, p=weights / weights.sum())
    pts = np.empty((n_cl, 3))
    todo = np.arange(n_cl)
    while todo.size:
        c = comp[todo]
        z = rng.standard_normal((todo.size, 3)) * sig[c]
        p = np.einsum("nij,nj->ni", rots[c], z) + centers[c]
        inside = np.all((p >= 0.0) & (p < L), axis=1)
        pts[todo[inside]] = p[inside]
        todo = todo[~inside]
    bg = rng.uniform(0.0, L, (n_bg, 3))
    allp = np.concatenate([pts, bg], axis=0)
    return allp[rng.permutation(N)]


_GENERATORS = {"C1": (1, _cloud_c1), "C2": (2, _cloud_c2), "C3": (3, _cloud_c3),
               "C4": (4, _cloud_c4), "C5": (5, _cloud_c5)}


def make_cloud(name: str, b: int = 0, N: int | None = None, calibration: bool = False) -> np.ndarray:
    """One float32 ``[N][3]`` cloud of workload `name` (N defaults to the workload's)."""
    cfg, fn = _GENERATORS[name]
    n_pts = WORKLOADS[name].N if N is None else int(N)
    pts = fn(_rng(cfg, b, calibration), n_pts)
    out = np.ascontiguousarray(pts, dtype=np.float32)
    assert out.shape == (n_pts, 3) and np.isfinite(out).all()
    return out


def make_batch(name: str, B: int | None = None, N: int | None = None,
               calibration: bool = False) -> np.ndarray:
    """float32 ``[B][N][3]`` batch of workload `name`."""
    nb = WORKLOADS[name].B if B is None else int(B)
    return np.stack([make_cloud(name, b, N, calibration) for b in range(nb)], axis=0)


def uniform_cube(seed: int, N: int) -> np.ndarray:
    """Small i.i.d. uniform cloud for unit tests (float32 ``[N][3]``)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return np.ascontiguousarray(rng.random((N, 3)), dtype=np.float32)


def lattice_with_ties(seed: int, N: int, cells: int = 6) -> np.ndarray:
    """Points on a coarse integer lattice (many exactly equal distances and
    duplicate points) -- exercises the lowest-index tie-breaking rules."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return np.ascontiguousarray(rng.integers(0, cells, (N, 3)), dtype=np.float32)
