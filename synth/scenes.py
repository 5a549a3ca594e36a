"""Procedural indoor scenes: box rooms with box / cylinder furniture.

World frame: Y up, metres, floor at y = 0.  Every planar face is an
(nu x nv) grid of quads, two triangles per quad, vertices shared inside one
face only, so V is roughly T/2 as in a scanned mesh.  One global cell size
controls the tessellation; it is searched so the triangle count lands within
2 % of the requested one.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

ROOM_X, ROOM_Z, ROOM_Y = 10.0, 8.0, 3.0     # one room: 10 (x) by 8 (z) by 3 (y) metres
DOOR_W, DOOR_H = 1.0, 2.1


@dataclass
class Scene:
    vertices: np.ndarray            # float32 [V,3]
    indices: np.ndarray             # uint32  [T,3]
    colors: np.ndarray              # uint8   [V,3]
    uvs: np.ndarray                 # float32 [V,2] texture coordinates (one repeat per metre of surface)
    texture: np.ndarray             # uint8   [256,256,3] procedural texture of the scene
    extent: tuple                   # (x_size, z_size) of the floor rectangle, origin at (0,0)
    boxes: np.ndarray = field(default_factory=lambda: np.zeros((0, 4)))      # footprints x0,z0,x1,z1
    cylinders: np.ndarray = field(default_factory=lambda: np.zeros((0, 3)))  # cx,cz,r
    wall_x: tuple = ()              # interior wall planes x = const
    wall_z: tuple = ()              # interior wall planes z = const
    cell: float = 0.0
    seed: int = 0

    @property
    def T(self) -> int:
        return int(self.indices.shape[0])

    @property
    def V(self) -> int:
        return int(self.vertices.shape[0])


class _MeshBuilder:
    """Accumulates faces; with count_only=True it only tallies triangles."""

    def __init__(self, count_only: bool):
        self.count_only = count_only
        self.verts, self.tris, self.obj, self.uv = [], [], [], []
        self.nv = 0
        self.nt = 0
        self.cur_obj = 0

    def next_object(self):
        self.cur_obj += 1

    def grid(self, origin, du, dv, nu, nv, keep=None):
        """Quad grid spanning origin + s*du + t*dv, s,t in [0,1]; keep[nv,nu] masks cells."""
        ncell = nu * nv if keep is None else int(keep.sum())
        self.nt += 2 * ncell
        if self.count_only:
            return
        s = np.linspace(0.0, 1.0, nu + 1)
        t = np.linspace(0.0, 1.0, nv + 1)
        S, Tt = np.meshgrid(s, t)                                   # [nv+1, nu+1]
        P = (np.asarray(origin, np.float64)[None, None, :]
             + S[..., None] * np.asarray(du, np.float64)[None, None, :]
             + Tt[..., None] * np.asarray(dv, np.float64)[None, None, :])
        base = self.nv
        jj, ii = np.meshgrid(np.arange(nv), np.arange(nu), indexing="ij")
        if keep is not None:
            jj, ii = jj[keep], ii[keep]
        jj, ii = jj.ravel(), ii.ravel()
        a = base + jj * (nu + 1) + ii
        b = a + 1
        c = a + (nu + 1)
        d = c + 1
        tri = np.empty((jj.size, 2, 3), np.int64)
        tri[:, 0, 0], tri[:, 0, 1], tri[:, 0, 2] = a, b, d
        tri[:, 1, 0], tri[:, 1, 1], tri[:, 1, 2] = a, d, c
        self.verts.append(P.reshape(-1, 3))
        self.tris.append(tri.reshape(-1, 3))
        self.obj.append(np.full(P.shape[0] * P.shape[1], self.cur_obj, np.int64))
        lu, lv = float(np.linalg.norm(du)), float(np.linalg.norm(dv))
        self.uv.append(np.stack([S * lu, Tt * lv], -1).reshape(-1, 2))
        self.nv += P.shape[0] * P.shape[1]

    def disc(self, centre, r, nseg, nring):
        """Horizontal disc (cylinder cap): centre fan plus nring-1 quad rings."""
        self.nt += nseg + 2 * nseg * (nring - 1)
        if self.count_only:
            return
        cx, cy, cz = centre
        ang = np.arange(nseg) * (2.0 * math.pi / nseg)
        pts = [np.array([[cx, cy, cz]])]
        for k in range(1, nring + 1):
            rr = r * k / nring
            pts.append(np.stack([cx + rr * np.cos(ang), np.full(nseg, cy), cz + rr * np.sin(ang)], 1))
        P = np.concatenate(pts, 0)
        base = self.nv
        i = np.arange(nseg)
        i1 = (i + 1) % nseg
        tris = [np.stack([np.full(nseg, base), base + 1 + i, base + 1 + i1], 1)]
        for k in range(1, nring):
            r0 = base + 1 + (k - 1) * nseg
            r1 = base + 1 + k * nseg
            tris.append(np.stack([r0 + i, r1 + i, r1 + i1], 1))
            tris.append(np.stack([r0 + i, r1 + i1, r0 + i1], 1))
        self.verts.append(P)
        self.tris.append(np.concatenate(tris, 0))
        self.obj.append(np.full(P.shape[0], self.cur_obj, np.int64))
        self.uv.append(P[:, [0, 2]].copy())
        self.nv += P.shape[0]

    def finish(self):
        return (np.concatenate(self.verts, 0), np.concatenate(self.tris, 0), np.concatenate(self.obj, 0),
                np.concatenate(self.uv, 0))


def _n(length, cell):
    return max(1, int(math.ceil(length / cell - 1e-9)))


def _add_room_shell(mb, x0, z0, sx, sz, sy, cell, walls=("x0", "x1", "z0", "z1")):
    """Floor, ceiling and the requested outer walls of one rectangular room."""
    nx, nz, ny = _n(sx, cell), _n(sz, cell), _n(sy, cell)
    mb.next_object()
    mb.grid((x0, 0, z0), (sx, 0, 0), (0, 0, sz), nx, nz)           # floor
    mb.next_object()
    mb.grid((x0, sy, z0), (sx, 0, 0), (0, 0, sz), nx, nz)          # ceiling
    for w in walls:
        mb.next_object()
        if w == "x0":
            mb.grid((x0, 0, z0), (0, 0, sz), (0, sy, 0), nz, ny)
        elif w == "x1":
            mb.grid((x0 + sx, 0, z0), (0, 0, sz), (0, sy, 0), nz, ny)
        elif w == "z0":
            mb.grid((x0, 0, z0), (sx, 0, 0), (0, sy, 0), nx, ny)
        elif w == "z1":
            mb.grid((x0, 0, z0 + sz), (sx, 0, 0), (0, sy, 0), nx, ny)


def _add_box(mb, x0, z0, sx, sz, sy, cell):
    nx, nz, ny = _n(sx, cell), _n(sz, cell), _n(sy, cell)
    mb.next_object()
    mb.grid((x0, sy, z0), (sx, 0, 0), (0, 0, sz), nx, nz)              # top
    mb.grid((x0, 0, z0), (sx, 0, 0), (0, sy, 0), nx, ny)               # z = z0 side
    mb.grid((x0, 0, z0 + sz), (sx, 0, 0), (0, sy, 0), nx, ny)          # z = z1 side
    mb.grid((x0, 0, z0), (0, 0, sz), (0, sy, 0), nz, ny)               # x = x0 side
    mb.grid((x0 + sx, 0, z0), (0, 0, sz), (0, sy, 0), nz, ny)          # x = x1 side


def _add_cylinder(mb, cx, cz, r, h, segs, cell):
    nseg = max(segs, _n(2.0 * math.pi * r, cell))
    ny = _n(h, cell)
    nring = _n(r, cell)
    mb.next_object()
    mb.nt += 2 * nseg * ny
    if not mb.count_only:
        ang = np.arange(nseg + 1) * (2.0 * math.pi / nseg)            # seam duplicated
        yy = np.linspace(0.0, h, ny + 1)
        A, Y = np.meshgrid(ang, yy)
        P = np.stack([cx + r * np.cos(A), Y, cz + r * np.sin(A)], -1).reshape(-1, 3)
        base = mb.nv
        jj, ii = np.meshgrid(np.arange(ny), np.arange(nseg), indexing="ij")
        jj, ii = jj.ravel(), ii.ravel()
        a = base + jj * (nseg + 1) + ii
        b, c = a + 1, a + (nseg + 1)
        d = c + 1
        tri = np.stack([np.stack([a, b, d], 1), np.stack([a, d, c], 1)], 1).reshape(-1, 3)
        mb.verts.append(P)
        mb.tris.append(tri)
        mb.obj.append(np.full(P.shape[0], mb.cur_obj, np.int64))
        mb.uv.append(np.stack([A * r, Y], -1).reshape(-1, 2))
        mb.nv += P.shape[0]
    mb.disc((cx, h, cz), r, nseg, nring)


def _search_cell(build, target_T):
    """Largest-to-smallest bisection on the cell size until |T - target| <= 2 %."""
    def count(cell):
        mb = _MeshBuilder(count_only=True)
        build(mb, cell)
        return mb.nt
    lo, hi = 1e-3, 16.0                     # count(lo) huge, count(hi) minimal
    best = (abs(count(hi) - target_T), hi)
    for _ in range(80):
        mid = math.sqrt(lo * hi)
        c = count(mid)
        err = abs(c - target_T)
        if err < best[0]:
            best = (err, mid)
        if err <= 0.02 * target_T * 0.25:   # well inside the 2 % band: stop early
            break
        if c > target_T:
            lo = mid
        else:
            hi = mid
    return best[1]


def _colorize(rng, obj_ids, nobj):
    base = rng.integers(0, 256, size=(nobj + 1, 3))
    noise = rng.integers(-16, 17, size=(obj_ids.shape[0], 3))
    return np.clip(base[obj_ids] + noise, 0, 255).astype(np.uint8)


def _texture(rng, size=256):
    """Coloured checker (8 x 8 cells) with per-texel noise: structure at every mip level."""
    cells = rng.integers(40, 216, size=(8, 8, 3))
    tex = np.repeat(np.repeat(cells, size // 8, 0), size // 8, 1)
    tex = tex + rng.integers(-24, 25, size=(size, size, 3))
    return np.clip(tex, 0, 255).astype(np.uint8)


def make_room_scene(target_T=10_000, seed=1000, n_boxes=20):
    """Single 10 x 8 x 3 m room with axis-aligned box furniture standing on the floor."""
    rng = np.random.default_rng(seed)
    sizes = rng.uniform(0.3, 2.0, size=(n_boxes, 3))                 # sx, sz, height
    ux = rng.uniform(0.0, 1.0, size=(n_boxes, 2))
    boxes = []
    for k in range(n_boxes):
        sx, sz, sy = sizes[k]
        x0 = 0.1 + ux[k, 0] * (ROOM_X - 0.2 - sx)
        z0 = 0.1 + ux[k, 1] * (ROOM_Z - 0.2 - sz)
        boxes.append((x0, z0, sx, sz, sy))

    def build(mb, cell):
        _add_room_shell(mb, 0.0, 0.0, ROOM_X, ROOM_Z, ROOM_Y, cell)
        for (x0, z0, sx, sz, sy) in boxes:
            _add_box(mb, x0, z0, sx, sz, sy, cell)

    cell = _search_cell(build, target_T)
    mb = _MeshBuilder(count_only=False)
    build(mb, cell)
    P, Tt, obj, uv = mb.finish()
    colors = _colorize(rng, obj, mb.cur_obj)
    fp = np.array([[b[0], b[1], b[0] + b[2], b[1] + b[3]] for b in boxes])
    return Scene(P.astype(np.float32), Tt.astype(np.uint32), colors, uv.astype(np.float32), _texture(rng), (ROOM_X, ROOM_Z),
                 boxes=fp, cell=cell, seed=seed)


def _make_irregular(P, obj, first_furniture, objs, cell, jitter, seed):
    """Irregular variant of a scene: every piece of furniture is turned about its vertical axis by a
    seeded angle (its faces stop being axis-aligned) and every vertex is displaced by up to
    `jitter` x cell in each axis (grids stop being regular, faces stop being planar).
    Returns the new positions and the axis-aligned footprints of the turned boxes."""
    rng = np.random.default_rng(seed + 7919)
    P = P.copy()
    footprints = []
    for k, o in enumerate(objs):
        m = obj == first_furniture + k
        c = 0.5 * (P[m][:, [0, 2]].min(0) + P[m][:, [0, 2]].max(0))
        a = rng.uniform(0.0, 2.0 * math.pi)
        ca, sa = math.cos(a), math.sin(a)
        dx, dz = P[m, 0] - c[0], P[m, 2] - c[1]
        P[m, 0] = c[0] + ca * dx - sa * dz
        P[m, 2] = c[1] + sa * dx + ca * dz
        if o[0] == "box":
            footprints.append([P[m, 0].min(), P[m, 2].min(), P[m, 0].max(), P[m, 2].max()])
    P += rng.uniform(-jitter, jitter, size=P.shape) * cell
    return P, np.array(footprints).reshape(-1, 4)


def make_multiroom_scene(target_T=200_000, seed=1000, n_objects=150, rooms=(3, 2), jitter=0.0):
    """rooms[0] x rooms[1] grid of rooms joined by doorways, with boxes and cylinders.
    jitter > 0 gives the irregular variant (see _make_irregular)."""
    rng = np.random.default_rng(seed)
    RX, RZ = rooms
    SX, SZ = RX * ROOM_X, RZ * ROOM_Z
    objs = []
    kinds = rng.integers(0, 2, size=n_objects)
    for k in range(n_objects):
        rx, rz = int(rng.integers(0, RX)), int(rng.integers(0, RZ))
        ox, oz = rx * ROOM_X, rz * ROOM_Z
        if kinds[k] == 0:
            sx, sz, sy = rng.uniform(0.3, 2.0, size=3)
            x0 = ox + 0.1 + rng.uniform() * (ROOM_X - 0.2 - sx)
            z0 = oz + 0.1 + rng.uniform() * (ROOM_Z - 0.2 - sz)
            objs.append(("box", x0, z0, sx, sz, sy))
        else:
            r = rng.uniform(0.15, 0.6)
            h = rng.uniform(0.3, 2.0)
            segs = int(rng.integers(16, 33))
            cx = ox + 0.1 + r + rng.uniform() * (ROOM_X - 0.2 - 2 * r)
            cz = oz + 0.1 + r + rng.uniform() * (ROOM_Z - 0.2 - 2 * r)
            objs.append(("cyl", cx, cz, r, h, segs))
    # one doorway per interior wall segment, centred at a seeded position along it
    doors_x = {(i, j): 1.5 + rng.uniform() * (ROOM_Z - 3.0) for i in range(1, RX) for j in range(RZ)}
    doors_z = {(i, j): 1.5 + rng.uniform() * (ROOM_X - 3.0) for j in range(1, RZ) for i in range(RX)}

    def wall_with_door(mb, origin, along, length, door_c, cell):
        nu, nv = _n(length, cell), _n(ROOM_Y, cell)
        u0 = (np.arange(nu)) * (length / nu)
        u1 = u0 + length / nu
        v0 = (np.arange(nv)) * (ROOM_Y / nv)
        hit_u = (u1 > door_c - DOOR_W / 2) & (u0 < door_c + DOOR_W / 2)
        hit_v = v0 < DOOR_H
        keep = ~(hit_v[:, None] & hit_u[None, :])
        mb.next_object()
        mb.grid(origin, along, (0, ROOM_Y, 0), nu, nv, keep=keep)

    def build(mb, cell):
        # outer shell: floor, ceiling and the four outer walls of the whole block
        _add_room_shell(mb, 0.0, 0.0, SX, SZ, ROOM_Y, cell)
        for (i, j), c in doors_x.items():      # interior walls at x = i*ROOM_X
            wall_with_door(mb, (i * ROOM_X, 0, j * ROOM_Z), (0, 0, ROOM_Z), ROOM_Z, c, cell)
        for (i, j), c in doors_z.items():      # interior walls at z = j*ROOM_Z
            wall_with_door(mb, (i * ROOM_X, 0, j * ROOM_Z), (ROOM_X, 0, 0), ROOM_X, c, cell)
        for o in objs:
            if o[0] == "box":
                _add_box(mb, *o[1:], cell)
            else:
                _add_cylinder(mb, *o[1:], cell)

    cell = _search_cell(build, target_T)
    mb = _MeshBuilder(count_only=False)
    build(mb, cell)
    P, Tt, obj, uv = mb.finish()
    colors = _colorize(rng, obj, mb.cur_obj)
    fp = np.array([[o[1], o[2], o[1] + o[3], o[2] + o[4]] for o in objs if o[0] == "box"]).reshape(-1, 4)
    cy = np.array([[o[1], o[2], o[3]] for o in objs if o[0] == "cyl"]).reshape(-1, 3)
    if jitter > 0.0:
        # objects are numbered in build order: floor, ceiling, four outer walls, the interior walls, then the furniture
        first_furniture = 6 + len(doors_x) + len(doors_z) + 1
        P, fp = _make_irregular(P, obj, first_furniture, objs, cell, jitter, seed)
    return Scene(P.astype(np.float32), Tt.astype(np.uint32), colors, uv.astype(np.float32), _texture(rng), (SX, SZ),
                 boxes=fp, cylinders=cy,
                 wall_x=tuple(i * ROOM_X for i in range(1, RX)),
                 wall_z=tuple(j * ROOM_Z for j in range(1, RZ)), cell=cell, seed=seed)
