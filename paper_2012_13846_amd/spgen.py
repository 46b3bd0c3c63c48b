"""Seeded synthetic inputs: voxelised surface point clouds, features, weights.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests/benchmarks.  It holds none of the method's arithmetic: it only
draws random points on surfaces, quantises them to integer voxel coordinates
(batch index first, Sec. III-B sparse-tensor definition) and draws Gaussian
features / weights.  Deduplication, strided coordinates, kernel maps and the
convolution itself are NOT done here.

The clouds stand in for the paper's voxelised ModelNet40 shapes (Sec. IV-A):
thin-surface occupancy at grid resolutions 32^3 .. 256^3.

numpy only; every function is a pure function of its seed.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20121384


def seed_for(config: int, cloud: int = 0, stream: int = 0) -> int:
    """Seed of cloud `cloud` of workload `config`; `stream` separates coords/features/weights."""
    return BASE_SEED + 1000 * config + cloud + 100000 * stream


# ----------------------------------------------------------------------------
# dtype helpers (storage conversion only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to the float32 holding the same value."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array whose every value is exactly representable in bfloat16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


# ----------------------------------------------------------------------------
# point samplers
# ----------------------------------------------------------------------------
def _unit_vectors(rng: np.random.Generator, n: int) -> np.ndarray:
    v = rng.standard_normal((n, 3))
    nrm = np.linalg.norm(v, axis=1, keepdims=True)
    nrm[nrm == 0] = 1.0
    return v / nrm


def _random_rotation(rng: np.random.Generator) -> np.ndarray:
    """Uniform rotation from a normalised Gaussian quaternion."""
    q = rng.standard_normal(4)
    q /= np.linalg.norm(q)
    w, x, y, z = q
    return np.array([
        [1 - 2 * (y * y + z * z), 2 * (x * y - z * w), 2 * (x * z + y * w)],
        [2 * (x * y + z * w), 1 - 2 * (x * x + z * z), 2 * (y * z - x * w)],
        [2 * (x * z - y * w), 2 * (y * z + x * w), 1 - 2 * (x * x + y * y)],
    ])


def _box_surface(rng, n, half):
    """n points uniform on the surface of the box [-half, half] (half = 3 half-extents)."""
    hx, hy, hz = half
    areas = np.array([hy * hz, hy * hz, hx * hz, hx * hz, hx * hy, hx * hy])
    face = rng.choice(6, size=n, p=areas / areas.sum())
    uvw = rng.uniform(-1.0, 1.0, size=(n, 3)) * np.asarray(half)
    axis = face // 2
    sign = np.where(face % 2 == 0, -1.0, 1.0)
    uvw[np.arange(n), axis] = sign * np.asarray(half)[axis]
    return uvw


def _cylinder_surface(rng, n, radius, half_h):
    """n points uniform on a closed cylinder (axis z)."""
    a_side = 2 * np.pi * radius * 2 * half_h
    a_cap = np.pi * radius * radius
    part = rng.choice(3, size=n, p=np.array([a_side, a_cap, a_cap]) / (a_side + 2 * a_cap))
    phi = rng.uniform(0, 2 * np.pi, n)
    r = np.where(part == 0, radius, radius * np.sqrt(rng.uniform(0, 1, n)))
    z = np.where(part == 0, rng.uniform(-half_h, half_h, n), np.where(part == 1, -half_h, half_h))
    return np.stack([r * np.cos(phi), r * np.sin(phi), z], axis=1)


def quantize(points: np.ndarray, origin: float, voxel: float, grid: int | None, batch: int,
             drop_outside: bool = False) -> np.ndarray:
    """Points -> int32 rows (b, x, y, z) with v = floor((p - origin) / voxel).

    With `grid` given, coordinates are clamped to [0, grid-1], or (drop_outside)
    rows with any coordinate outside are removed.
    """
    v = np.floor((points - origin) / voxel).astype(np.int64)
    if grid is not None:
        if drop_outside:
            keep = np.all((v >= 0) & (v < grid), axis=1)
            v = v[keep]
        else:
            v = np.clip(v, 0, grid - 1)
    out = np.empty((v.shape[0], 4), dtype=np.int32)
    out[:, 0] = batch
    out[:, 1:] = v
    return out


def sphere_cloud(seed: int, n_pts: int, grid: int, batch: int = 0, radius: float = 0.9) -> np.ndarray:
    """n_pts points uniform on a sphere surface in the box [-1,1]^3, quantised to grid^3."""
    rng = np.random.default_rng(seed)
    p = radius * _unit_vectors(rng, n_pts)
    return quantize(p, -1.0, 2.0 / grid, grid, batch)


def primitives_cloud(seed: int, n_pts: int, grid: int, batch: int = 0, scale_lo: float = 0.2,
                     scale_hi: float = 0.8) -> np.ndarray:
    """n_pts points on the surfaces of 1-4 random primitives in the unit cube, quantised to grid^3.

    Each primitive is a box, sphere or cylinder of scale U[scale_lo, scale_hi] (full extent; default U[0.2,0.8]),
    uniformly rotated, centred so that its bounding sphere mostly fits; points are
    allotted area-weighted; points that fall outside [0,1)^3 are dropped.
    """
    rng = np.random.default_rng(seed)
    n_prim = int(rng.integers(1, 5))
    prims = []
    for _ in range(n_prim):
        kind = int(rng.integers(0, 3))
        scale = rng.uniform(scale_lo, scale_hi)
        rot = _random_rotation(rng)
        if kind == 0:
            half = 0.5 * scale * rng.uniform(0.5, 1.0, 3)
            area = 8 * (half[0] * half[1] + half[1] * half[2] + half[0] * half[2])
            reach = float(np.linalg.norm(half))
            par = half
        elif kind == 1:
            rad = 0.5 * scale
            area = 4 * np.pi * rad * rad
            reach = rad
            par = rad
        else:
            rad = 0.5 * scale * rng.uniform(0.3, 1.0)
            hh = 0.5 * scale * rng.uniform(0.5, 1.0)
            area = 2 * np.pi * rad * 2 * hh + 2 * np.pi * rad * rad
            reach = float(np.hypot(rad, hh))
            par = (rad, hh)
        margin = min(reach * 0.8, 0.5)
        centre = rng.uniform(margin, 1.0 - margin, 3) if margin < 0.5 else np.full(3, 0.5)
        prims.append((kind, par, rot, centre, area))
    areas = np.array([p[4] for p in prims])
    which = rng.choice(n_prim, size=n_pts, p=areas / areas.sum())
    pts = np.empty((n_pts, 3))
    for j, (kind, par, rot, centre, _) in enumerate(prims):
        m = int(np.count_nonzero(which == j))
        if m == 0:
            continue
        if kind == 0:
            loc = _box_surface(rng, m, par)
        elif kind == 1:
            loc = par * _unit_vectors(rng, m)
        else:
            loc = _cylinder_surface(rng, m, par[0], par[1])
        pts[which == j] = loc @ rot.T + centre
    return quantize(pts, 0.0, 1.0 / grid, grid, batch, drop_outside=True)


def room_cloud(seed: int, voxel: float = 0.05, pts_per_cell: float = 5.0, n_boxes: int = 30,
               batch: int = 0) -> np.ndarray:
    """Indoor-scene-like cloud: 10 x 10 x 3 m room (6 planes) + axis-aligned boxes on the floor.

    Points are area-weighted with about `pts_per_cell` points per voxel-face of area,
    jittered by U[-1,1] cm per axis, quantised with voxel size `voxel` (metres), origin 0.
    """
    rng = np.random.default_rng(seed)
    room = np.array([10.0, 10.0, 3.0])
    rects = []  # (origin, edge_u, edge_v)
    X, Y, Z = room
    rects += [(np.array([0, 0, 0.0]), np.array([X, 0, 0]), np.array([0, Y, 0])),
              (np.array([0, 0, Z]), np.array([X, 0, 0]), np.array([0, Y, 0])),
              (np.array([0, 0, 0.0]), np.array([X, 0, 0]), np.array([0, 0, Z])),
              (np.array([0, Y, 0.0]), np.array([X, 0, 0]), np.array([0, 0, Z])),
              (np.array([0, 0, 0.0]), np.array([0, Y, 0]), np.array([0, 0, Z])),
              (np.array([X, 0, 0.0]), np.array([0, Y, 0]), np.array([0, 0, Z]))]
    for _ in range(n_boxes):
        e = rng.uniform(0.3, 2.0, 3)
        e[2] = min(e[2], Z - 0.1)
        o = np.array([rng.uniform(0.05, X - e[0] - 0.05), rng.uniform(0.05, Y - e[1] - 0.05), 0.0])
        ex, ey, ez = np.diag(e)
        rects += [(o + ez, ex, ey),                      # top
                  (o, ex, ez), (o + ey, ex, ez),          # two y-faces
                  (o, ey, ez), (o + ex, ey, ez)]          # two x-faces
    areas = np.array([np.linalg.norm(np.cross(u, v)) for _, u, v in rects])
    n_pts = int(pts_per_cell * areas.sum() / (voxel * voxel))
    which = rng.choice(len(rects), size=n_pts, p=areas / areas.sum())
    s = rng.uniform(0, 1, n_pts)[:, None]
    t = rng.uniform(0, 1, n_pts)[:, None]
    O = np.stack([r[0] for r in rects])[which]
    U = np.stack([r[1] for r in rects])[which]
    V = np.stack([r[2] for r in rects])[which]
    pts = O + s * U + t * V + rng.uniform(-0.01, 0.01, (n_pts, 3))
    pts = np.clip(pts, 0.0, room - 1e-6)
    return quantize(pts, 0.0, voxel, None, batch)


def batch_of(fn, config: int, n_clouds: int, **kw) -> np.ndarray:
    """Concatenate n_clouds clouds from `fn`, cloud c drawn with seed_for(config, c)."""
    parts = [fn(seed_for(config, c), batch=c, **kw) for c in range(n_clouds)]
    return np.ascontiguousarray(np.concatenate(parts, axis=0))


# ----------------------------------------------------------------------------
# the five workloads' raw coordinates (duplicates NOT merged)
# ----------------------------------------------------------------------------
def coords_config(cfg: int, scale: float = 1.0) -> np.ndarray:
    """Raw int32 [n_raw][4] (b,x,y,z) coordinates of workload cfg (0..4).

    `scale` < 1 shrinks the point count (and for cfg 4 coarsens nothing): used
    only to make small variants for CPU-side tests.
    """
    if cfg == 0:
        return batch_of(sphere_cloud, 0, 1, n_pts=max(1, int(2048 * scale)), grid=32)
    if cfg == 1:
        return batch_of(primitives_cloud, 1, 8, n_pts=max(1, int(20000 * scale)), grid=128)
    if cfg == 2:
        return batch_of(sphere_cloud, 2, 8, n_pts=max(1, int(131072 * scale)), grid=256)
    if cfg == 3:
        return batch_of(sphere_cloud, 3, 4, n_pts=max(1, int(131072 * scale)), grid=256)
    if cfg == 4:
        return room_cloud(seed_for(4, 0), voxel=0.025, pts_per_cell=5.0 * scale)
    raise ValueError(f"unknown config {cfg}")


def coords_literal(which: str) -> np.ndarray:
    """The literal readings of two BASELINE configs whose text contradicts its own voxel count:
    "cfg2_2048pt": the config-0 generator with its 2048 points per cloud at a 256^3 grid, 8 clouds (latency datapoint);
    "cfg4_5cm": the room at 5 cm voxels (about a quarter of the ~1 M voxels the config names)."""
    if which == "cfg2_2048pt":
        return batch_of(sphere_cloud, 2, 8, n_pts=2048, grid=256)
    if which == "cfg4_5cm":
        return room_cloud(seed_for(4, 0), voxel=0.05, pts_per_cell=5.0)
    raise ValueError(which)


# ----------------------------------------------------------------------------
# the paper's sparsity sweep (Sec. IV-C, Table II): many small clouds per batch, with point dropout
# ----------------------------------------------------------------------------
SWEEP_POINTS = 4096            # points kept per shape before dropout (Sec. IV-A)
SWEEP_GRIDS = (32, 50)
SWEEP_P = (1.0, 0.5, 0.25)


def sweep_cloud(seed: int, grid: int, p: float, batch: int = 0) -> np.ndarray:
    """One shape of the sparsity sweep: 4096 surface points of 1-4 primitives that fill most of the unit cube
    (scale U[0.6,1]: 7.6 % occupied voxels at 32^3, 2.6 % at 50^3, the paper's figures for its shapes), of which
    a fraction theta ~ U[0, 1-p] is dropped, quantised to grid^3."""
    raw = primitives_cloud(seed, SWEEP_POINTS, grid, batch, 0.6, 1.0)
    theta = np.random.default_rng(seed + 77_000_000).uniform(0.0, 1.0 - p) if p < 1.0 else 0.0
    keep = int(round((1.0 - theta) * len(raw)))     # the points are i.i.d.: dropping a random subset = keeping a prefix
    return np.ascontiguousarray(raw[:keep])


def coords_sweep(grid: int, p: float, n_clouds: int) -> np.ndarray:
    """Raw coordinates of one batch of the sparsity sweep (workload index 5)."""
    stream = 10 + SWEEP_GRIDS.index(grid) * len(SWEEP_P) + SWEEP_P.index(p)
    parts = [sweep_cloud(seed_for(5, c, stream), grid, p, batch=c) for c in range(n_clouds)]
    return np.ascontiguousarray(np.concatenate(parts, axis=0))


# ----------------------------------------------------------------------------
# features and weights
# ----------------------------------------------------------------------------
def features(seed: int, n: int, c: int, bf16: bool = False) -> np.ndarray:
    """[n][c] float32 ~ N(0,1); with bf16=True every value is bf16-representable."""
    x = np.random.default_rng(seed).standard_normal((n, c)).astype(np.float32)
    return round_to_bf16(x) if bf16 else x


def weights(seed: int, kvol: int, cin: int, cout: int, bf16: bool = False) -> np.ndarray:
    """[kvol][cout][cin] float32 ~ N(0, 1/(kvol*cin)) (layout of Sec. III-B: K^D x N_out x N_in)."""
    w = np.random.default_rng(seed).standard_normal((kvol, cout, cin)) / np.sqrt(kvol * cin)
    w = w.astype(np.float32)
    return round_to_bf16(w) if bf16 else w
