"""Synthetic point clouds: unit cube, jittered box surfaces, furnished rooms.

All generators take a numpy Generator and return float32 [N,3] arrays.
"""
import numpy as np


def uniform_cube(rng, n):
    return rng.random((n, 3), dtype=np.float32)


def _largest_remainder(weights, total):
    """Integer allotment of `total` items proportional to `weights`."""
    w = np.asarray(weights, dtype=np.float64)
    q = w / w.sum() * total
    base = np.floor(q).astype(np.int64)
    rem = total - int(base.sum())
    if rem > 0:
        order = np.argsort(-(q - base), kind="stable")
        base[order[:rem]] += 1
    return base


def _box_rects(lo, hi):
    """The 6 axis-aligned rectangles of the box [lo,hi] as (origin, u, v)."""
    lo = np.asarray(lo, np.float64)
    hi = np.asarray(hi, np.float64)
    ext = hi - lo
    rects = []
    for ax in range(3):
        a, b = [i for i in range(3) if i != ax]
        for side in (lo[ax], hi[ax]):
            o = lo.copy()
            o[ax] = side
            u = np.zeros(3)
            u[a] = ext[a]
            v = np.zeros(3)
            v[b] = ext[b]
            rects.append((o, u, v))
    return rects


def _sample_rects(rng, rects, n, sigma):
    areas = [np.linalg.norm(u) * np.linalg.norm(v) for (_, u, v) in rects]
    counts = _largest_remainder(areas, n)
    out = np.empty((n, 3), dtype=np.float32)
    at = 0
    for (o, u, v), m in zip(rects, counts):
        m = int(m)
        if m == 0:
            continue
        s = rng.random((m, 1))
        t = rng.random((m, 1))
        out[at:at + m] = (o + s * u + t * v).astype(np.float32)
        at += m
    out += rng.normal(0.0, sigma, size=(n, 3)).astype(np.float32)
    return out


def box_surface_cloud(rng, n, sigma=0.005, clutter=0.2):
    """Points on the 6 faces of a random box (sides U[0.5,1.5]) with Gaussian
    jitter, plus a `clutter` fraction drawn uniformly inside the box."""
    side = rng.uniform(0.5, 1.5, size=3)
    n_in = int(round(n * clutter))
    n_surf = n - n_in
    surf = _sample_rects(rng, _box_rects(np.zeros(3), side), n_surf, sigma)
    inside = (rng.random((n_in, 3)) * side).astype(np.float32)
    pts = np.concatenate([surf, inside], axis=0)
    return pts[rng.permutation(n)]


def room_cloud(rng, n, size=(10.0, 10.0, 3.0), n_boxes=30, sigma=0.005):
    """A room of planar walls/floor/ceiling plus `n_boxes` axis-aligned box
    'furniture' pieces (all 6 faces each); points allotted in proportion to
    area, uniform on each rectangle, Gaussian jitter on all axes."""
    size = np.asarray(size, np.float64)
    rects = _box_rects(np.zeros(3), size)
    for _ in range(n_boxes):
        ext = rng.uniform(0.3, 2.0, size=3)
        ext[2] = min(ext[2], size[2])
        lo = rng.random(3) * (size - ext)
        lo[2] = 0.0 if rng.random() < 0.7 else lo[2]   # most furniture stands on the floor
        rects += _box_rects(lo, lo + ext)
    return _sample_rects(rng, rects, n, sigma)


def morton_order(pts, bits=10):
    """Permutation that sorts points along a 3*bits-bit Z-order curve."""
    p = np.asarray(pts, np.float64)
    lo = p.min(axis=0)
    span = np.maximum(p.max(axis=0) - lo, 1e-30)
    q = np.minimum(((p - lo) / span * (1 << bits)).astype(np.uint64), (1 << bits) - 1)

    def spread(x):
        x = x & np.uint64(0x3FF)
        x = (x | (x << np.uint64(16))) & np.uint64(0x030000FF)
        x = (x | (x << np.uint64(8))) & np.uint64(0x0300F00F)
        x = (x | (x << np.uint64(4))) & np.uint64(0x030C30C3)
        x = (x | (x << np.uint64(2))) & np.uint64(0x09249249)
        return x

    assert bits <= 10
    code = spread(q[:, 0]) | (spread(q[:, 1]) << np.uint64(1)) | (spread(q[:, 2]) << np.uint64(2))
    return np.argsort(code, kind="stable")
