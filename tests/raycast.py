"""Brute-force float64 ray caster: an independent definition of 'nearest triangle per pixel'.

Used only to pin the oracle.  For each pixel centre a ray is un-projected with the
inverse of the view-projection matrix and intersected with every triangle
(Moller-Trumbore, two-sided); the hit with the smallest eye depth (row 3 of M applied
to the hit point) inside the near/far slab wins.
"""
import numpy as np


def raycast(vertices, indices, M, H, W, offsets=((0.0, 0.0),)):
    """Returns (ids [n_off,H,W] int64 (-1 = miss), depth [n_off,H,W], gap [n_off,H,W]).

    gap = relative distance between nearest and second-nearest hit (inf if < 2 hits)."""
    V = np.asarray(vertices, np.float64)
    I = np.asarray(indices, np.int64)
    M = np.asarray(M, np.float64).reshape(4, 4)
    Minv = np.linalg.inv(M)
    p0, p1, p2 = V[I[:, 0]], V[I[:, 1]], V[I[:, 2]]
    e1, e2 = p1 - p0, p2 - p0
    ids_all, dep_all, gap_all = [], [], []
    jj, ii = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    for (ox, oy) in offsets:
        xn = (ii + 0.5 + ox) * 2.0 / W - 1.0
        yn = (jj + 0.5 + oy) * 2.0 / H - 1.0
        a = np.stack([xn, yn, np.zeros_like(xn), np.ones_like(xn)], -1) @ Minv.T    # on the near plane
        b = np.stack([xn, yn, np.ones_like(xn), np.ones_like(xn)], -1) @ Minv.T     # on the far plane
        a = a[..., :3] / a[..., 3:4]
        b = b[..., :3] / b[..., 3:4]
        o = a.reshape(-1, 1, 3)
        d = (b - a).reshape(-1, 1, 3)                      # ray parameter s in [0,1] spans near..far
        pvec = np.cross(d, e2[None])
        det = np.einsum("ptk,ptk->pt", np.broadcast_to(e1[None], pvec.shape), pvec)
        with np.errstate(divide="ignore", invalid="ignore"):
            inv = 1.0 / det
            tvec = o - p0[None]
            u = np.einsum("ptk,ptk->pt", tvec, pvec) * inv
            qvec = np.cross(tvec, e1[None])
            v = np.einsum("ptk,ptk->pt", np.broadcast_to(d, qvec.shape), qvec) * inv
            s = np.einsum("ptk,ptk->pt", np.broadcast_to(e2[None], qvec.shape), qvec) * inv
        hit = (np.abs(det) > 0) & (u >= 0) & (v >= 0) & (u + v <= 1) & (s >= 0) & (s <= 1)
        P = o + s[..., None] * d
        depth = P @ M[3, :3] + M[3, 3]
        depth = np.where(hit, depth, np.inf)
        order = np.argsort(depth, axis=1)
        first = order[:, 0]
        dmin = depth[np.arange(depth.shape[0]), first]
        if depth.shape[1] > 1:
            second = depth[np.arange(depth.shape[0]), order[:, 1]]
        else:
            second = np.full_like(dmin, np.inf)
        ids = np.where(np.isfinite(dmin), first, -1)
        with np.errstate(invalid="ignore"):
            gap = np.where(np.isfinite(second), (second - dmin) / np.maximum(dmin, 1e-30), np.inf)
        ids_all.append(ids.reshape(H, W))
        dep_all.append(dmin.reshape(H, W))
        gap_all.append(gap.reshape(H, W))
    return np.stack(ids_all), np.stack(dep_all), np.stack(gap_all)
