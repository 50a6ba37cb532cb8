"""Seeded synthetic point clouds for the FPS tests and benchmark.

This module only *draws inputs*.  It contains none of the sampling method's
arithmetic (no distances between points, no min/argmax, no pruning rules), so
that the CPU oracle and the HIP path can both be fed from it without sharing
any of the method itself.  It imports nothing from the rest of the package.

Each generator stands in for a workload class that the FlashFPS paper names
(Sec. 1 and Sec. 4.1): ~1K-point object clouds, 13K-297K-point indoor rooms,
and ~300K-point LiDAR frames.  No dataset item is used; only sizes, surface
structure and density fall-off are imitated.  All draws are made in float64
with NumPy's PCG64 stream and rounded once to float32.  Point order is kept
structured (surface by surface, scan order): clouds are never shuffled.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "seed_for", "uniform_cube", "shape_cloud", "planes_and_clusters", "room",
    "lidar_frame", "make_config", "lattice_line", "lattice_grid", "CONFIGS",
]


def seed_for(config: int, cloud: int = 0) -> int:
    """Seed convention: 1000*config + cloud index."""
    return 1000 * int(config) + int(cloud)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


def _f32(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


# ----------------------------------------------------------------------------
# config 1: uniform cube
# ----------------------------------------------------------------------------
def uniform_cube(n: int, seed: int, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    """n points uniform in [lo, hi)^3."""
    r = _rng(seed)
    return _f32(r.uniform(lo, hi, size=(n, 3)))


# ----------------------------------------------------------------------------
# config 2: one closed surface per cloud (sphere / cube / cylinder)
# ----------------------------------------------------------------------------
def _random_rotation(r: np.random.Generator) -> np.ndarray:
    q, rr = np.linalg.qr(r.standard_normal((3, 3)))
    q = q * np.sign(np.diag(rr))
    if np.linalg.det(q) < 0:
        q[:, 0] = -q[:, 0]
    return q


def _sphere_surface(r, n):
    v = r.standard_normal((n, 3))
    return v / np.linalg.norm(v, axis=1, keepdims=True)


def _cube_surface(r, n):
    # faces of [-1,1]^3, all of equal area
    face = r.integers(0, 6, size=n)
    uv = r.uniform(-1.0, 1.0, size=(n, 2))
    p = np.empty((n, 3))
    axis = face // 2
    sign = np.where(face % 2 == 0, -1.0, 1.0)
    for a in range(3):
        m = axis == a
        o = [i for i in range(3) if i != a]
        p[m, a] = sign[m]
        p[m, o[0]] = uv[m, 0]
        p[m, o[1]] = uv[m, 1]
    return p


def _cylinder_surface(r, n):
    # radius 1, height 2, caps included; area weights: side 4*pi, caps pi each
    part = r.uniform(0.0, 6.0, size=n)
    th = r.uniform(0.0, 2.0 * np.pi, size=n)
    p = np.empty((n, 3))
    side = part < 4.0
    ns = int(side.sum())
    p[side, 0] = np.cos(th[side])
    p[side, 1] = np.sin(th[side])
    p[side, 2] = r.uniform(-1.0, 1.0, size=ns)
    cap = ~side
    nc = int(cap.sum())
    rad = np.sqrt(r.uniform(0.0, 1.0, size=nc))
    p[cap, 0] = rad * np.cos(th[cap])
    p[cap, 1] = rad * np.sin(th[cap])
    p[cap, 2] = np.where(part[cap] < 5.0, -1.0, 1.0)
    return p


def shape_cloud(n: int, seed: int, sigma: float = 0.005) -> np.ndarray:
    """Surface-uniform samples of a randomly rotated sphere, cube or cylinder
    (chosen by the seed's stream) plus isotropic Gaussian noise."""
    r = _rng(seed)
    kind = int(r.integers(0, 3))
    p = (_sphere_surface, _cube_surface, _cylinder_surface)[kind](r, n)
    p = p @ _random_rotation(r).T
    p = p + r.normal(0.0, sigma, size=p.shape)
    return _f32(p)


# ----------------------------------------------------------------------------
# config 3: planes + Gaussian clusters in a box
# ----------------------------------------------------------------------------
def planes_and_clusters(n: int, seed: int, box: float = 4.0, n_planes: int = 4,
                        n_clusters: int = 20, sigma: float = 0.05,
                        plane_frac: float = 0.6) -> np.ndarray:
    """60 % of the points on random planes clipped to [0,box]^3, 40 % in
    isotropic Gaussian clusters; listed plane by plane, then cluster by cluster."""
    r = _rng(seed)
    n_pl = int(round(n * plane_frac))
    per_plane = [n_pl // n_planes + (1 if i < n_pl % n_planes else 0) for i in range(n_planes)]
    n_cl = n - n_pl
    per_cl = [n_cl // n_clusters + (1 if i < n_cl % n_clusters else 0) for i in range(n_clusters)]
    out = []
    for cnt in per_plane:
        nrm = r.standard_normal(3)
        nrm /= np.linalg.norm(nrm)
        p0 = r.uniform(0.25 * box, 0.75 * box, size=3)
        # orthonormal basis of the plane
        a = np.cross(nrm, [1.0, 0.0, 0.0] if abs(nrm[0]) < 0.9 else [0.0, 1.0, 0.0])
        a /= np.linalg.norm(a)
        b = np.cross(nrm, a)
        got = np.empty((0, 3))
        while got.shape[0] < cnt:
            uv = r.uniform(-box, box, size=(4 * cnt + 16, 2))
            q = p0 + uv[:, :1] * a + uv[:, 1:] * b
            ok = np.all((q >= 0.0) & (q <= box), axis=1)
            got = np.concatenate([got, q[ok]], axis=0)
        out.append(got[:cnt])
    for cnt in per_cl:
        c = r.uniform(0.05 * box, 0.95 * box, size=3)
        out.append(c + r.normal(0.0, sigma, size=(cnt, 3)))
    return _f32(np.concatenate(out, axis=0))


# ----------------------------------------------------------------------------
# config 4: indoor room
# ----------------------------------------------------------------------------
def _rect(origin, eu, ev):
    return (np.asarray(origin, float), np.asarray(eu, float), np.asarray(ev, float))


def _box_faces(lo, hi):
    lx, ly, lz = lo
    hx, hy, hz = hi
    dx, dy, dz = hx - lx, hy - ly, hz - lz
    return [
        _rect((lx, ly, lz), (dx, 0, 0), (0, dy, 0)),
        _rect((lx, ly, hz), (dx, 0, 0), (0, dy, 0)),
        _rect((lx, ly, lz), (dx, 0, 0), (0, 0, dz)),
        _rect((lx, hy, lz), (dx, 0, 0), (0, 0, dz)),
        _rect((lx, ly, lz), (0, dy, 0), (0, 0, dz)),
        _rect((hx, ly, lz), (0, dy, 0), (0, 0, dz)),
    ]


def room(n: int, seed: int, size=(10.0, 10.0, 3.0), n_boxes: int = 30,
         sigma: float = 0.01) -> np.ndarray:
    """Surface samples of a room shell plus axis-aligned boxes, density
    proportional to area, listed surface by surface, with Gaussian noise."""
    r = _rng(seed)
    sx, sy, sz = size
    rects = _box_faces((0.0, 0.0, 0.0), (sx, sy, sz))  # floor, ceiling, 4 walls
    for i in range(n_boxes):
        ext = r.uniform(0.3, 1.5, size=3)
        ext[2] = min(ext[2], sz - 0.1)
        x0 = r.uniform(0.05, sx - 0.05 - ext[0])
        y0 = r.uniform(0.05, sy - 0.05 - ext[1])
        z0 = 0.0 if i % 2 == 0 else r.uniform(0.0, sz - ext[2])
        rects += _box_faces((x0, y0, z0), (x0 + ext[0], y0 + ext[1], z0 + ext[2]))
    area = np.array([np.linalg.norm(np.cross(u, v)) for (_, u, v) in rects])
    share = n * area / area.sum()
    cnt = np.floor(share).astype(np.int64)
    rest = n - int(cnt.sum())
    order = np.argsort(-(share - cnt), kind="stable")
    cnt[order[:rest]] += 1
    out = []
    for (o, u, v), c in zip(rects, cnt):
        ab = r.uniform(0.0, 1.0, size=(int(c), 2))
        out.append(o + ab[:, :1] * u + ab[:, 1:] * v)
    p = np.concatenate(out, axis=0)
    p = p + r.normal(0.0, sigma, size=p.shape)
    return _f32(p)


# ----------------------------------------------------------------------------
# config 5: spinning multi-beam LiDAR frame
# ----------------------------------------------------------------------------
def lidar_frame(n: int, seed: int, beams: int = 64, az_steps: int = 4688,
                el_lo: float = -25.0, el_hi: float = 15.0, height: float = 1.8,
                max_range: float = 80.0, n_boxes: int = 200, sigma: float = 0.02,
                max_revs: int = 16) -> np.ndarray:
    """Ray-cast a ground plane and random boxes from a spinning sensor.

    Returns beyond max_range and rays that hit nothing are dropped.  Because
    one revolution then yields fewer than beams*az_steps returns, further
    revolutions at a sub-step azimuth phase offset follow, and the first n
    valid returns in scan order (revolution, azimuth step, beam) are kept.
    """
    r = _rng(seed)
    # boxes resting on the ground, centres in an annulus around the sensor
    rad = np.sqrt(r.uniform(4.0 ** 2, (max_range - 4.0) ** 2, size=n_boxes))
    ang = r.uniform(0.0, 2.0 * np.pi, size=n_boxes)
    ext = np.stack([r.uniform(1.0, 6.0, n_boxes), r.uniform(1.0, 6.0, n_boxes),
                    r.uniform(1.0, 4.0, n_boxes)], axis=1)
    ctr = np.stack([rad * np.cos(ang), rad * np.sin(ang), 0.5 * ext[:, 2]], axis=1)
    blo = ctr - 0.5 * ext
    bhi = ctr + 0.5 * ext
    origin = np.array([0.0, 0.0, height])
    el = np.deg2rad(np.linspace(el_lo, el_hi, beams))
    kept = []
    total = 0
    step = 2.0 * np.pi / az_steps
    chunk = 586  # azimuth steps per chunk
    for rev in range(max_revs):
        phase = step * (rev / float(max_revs))
        for a0 in range(0, az_steps, chunk):
            az = phase + step * np.arange(a0, min(a0 + chunk, az_steps))
            d = np.stack([np.outer(np.cos(az), np.cos(el)),
                          np.outer(np.sin(az), np.cos(el)),
                          np.outer(np.ones_like(az), np.sin(el))], axis=2).reshape(-1, 3)
            t = np.full(d.shape[0], np.inf)
            down = d[:, 2] < 0.0
            t[down] = height / (-d[down, 2])
            # slab test against every box
            with np.errstate(divide="ignore", invalid="ignore"):
                inv = 1.0 / d
                t1 = (blo[None, :, :] - origin) * inv[:, None, :]
                t2 = (bhi[None, :, :] - origin) * inv[:, None, :]
            tn = np.nanmax(np.minimum(t1, t2), axis=2)
            tf = np.nanmin(np.maximum(t1, t2), axis=2)
            hit = (tn <= tf) & (tf > 0.0)
            tb = np.where(hit, np.where(tn > 0.0, tn, tf), np.inf).min(axis=1)
            t = np.minimum(t, tb)
            rng = t + r.normal(0.0, sigma, size=t.shape)
            ok = np.isfinite(t) & (rng <= max_range) & (rng > 0.0)
            pts = origin + d[ok] * rng[ok, None]
            kept.append(pts)
            total += pts.shape[0]
            if total >= n:
                return _f32(np.concatenate(kept, axis=0)[:n])
    raise RuntimeError(f"lidar_frame: only {total} valid returns for n={n}")


# ----------------------------------------------------------------------------
# exact-in-fp32 lattice inputs (tie-heavy; used by pins and edge-case parity)
# ----------------------------------------------------------------------------
def lattice_line(n: int) -> np.ndarray:
    """Points (i, 0, 0), i = 0..n-1."""
    p = np.zeros((n, 3))
    p[:, 0] = np.arange(n)
    return _f32(p)


def lattice_grid(a: int, b: int, c: int = 1) -> np.ndarray:
    """Integer lattice a x b x c; point (i*b + j)*c + k sits at (i, j, k)."""
    i, j, k = np.meshgrid(np.arange(a), np.arange(b), np.arange(c), indexing="ij")
    return _f32(np.stack([i.ravel(), j.ravel(), k.ravel()], axis=1))


# ----------------------------------------------------------------------------
# the five benchmark configurations
# ----------------------------------------------------------------------------
CONFIGS = {
    1: dict(B=1, N=1024, stages=(512,)),
    2: dict(B=32, N=1024, stages=(512, 128)),
    3: dict(B=8, N=16384, stages=(4096, 1024, 256, 64)),
    4: dict(B=1, N=200000, stages=(50000, 12500, 3125, 781)),
    5: dict(B=1, N=300000, stages=(16384, 4096, 1024, 256)),
}


def make_config(config: int, B: int | None = None, N: int | None = None) -> np.ndarray:
    """float32 array [B, N, 3] for benchmark configuration `config` (1..5).
    B and N default to the configuration's sizes; smaller values give the same
    kind of cloud at test size."""
    spec = CONFIGS[config]
    B = spec["B"] if B is None else B
    N = spec["N"] if N is None else N
    gen = {1: uniform_cube, 2: shape_cloud, 3: planes_and_clusters,
           4: room, 5: lidar_frame}[config]
    return np.stack([gen(N, seed_for(config, b)) for b in range(B)], axis=0)
