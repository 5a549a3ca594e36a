"""Pins for the CPU oracle: closed forms, brute force, invariants (no GPU needed).

The paper prints no renderer output to compare with (Sec. 3.2 delegates rasterisation to
the graphics API), so the oracle is tied to things that do not depend on it: analytic
depths of planes, a float64 ray caster, exact-integer point-in-polygon tests and a
hand-enumerated fill-rule fixture.
"""
import math
import os

import numpy as np
import pytest

import oracle
import synth
from raycast import raycast

HERE = os.path.dirname(os.path.abspath(__file__))
NOHIT = 0xFFFFFFFF


def cam(pos=(0, 0, 0), yaw=0.0, pitch=0.0, near=0.01, far=20.0, hfov=90.0, aspect=1.0):
    return synth.view_proj_from_pose(pos, yaw, pitch, hfov, aspect, near, far)


def ulp_diff(a, b):
    ai = np.asarray(a, np.float32).view(np.int32).astype(np.int64)
    bi = np.asarray(b, np.float32).view(np.int32).astype(np.int64)
    return np.abs(ai - bi)


# ---------------------------------------------------------------- 1. camera-facing quad

def facing_quad(d, i0, i1, j0, j1, W, H):
    """Quad at eye distance d whose corners project onto pixel-centre lines i0,i1 / j0,j1."""
    xn = lambda i: (i + 0.5) * 2.0 / W - 1.0
    yn = lambda j: (j + 0.5) * 2.0 / H - 1.0
    # camera at origin, looking down -z, y up; image y is down so world y = -yn * d
    tl = (xn(i0) * d, -yn(j0) * d, -d)
    tr = (xn(i1) * d, -yn(j0) * d, -d)
    br = (xn(i1) * d, -yn(j1) * d, -d)
    bl = (xn(i0) * d, -yn(j1) * d, -d)
    return np.array([tl, tr, br, bl], np.float32)


@pytest.mark.parametrize("split", ["tl-br", "tr-bl"])
@pytest.mark.parametrize("flip", [False, True])
@pytest.mark.parametrize("d", [2.0, 0.5, 16.0])
def test_facing_quad_exact_rectangle_and_depth(split, flip, d):
    H = W = 64
    v = facing_quad(d, 8, 40, 16, 48, W, H)
    idx = np.array([[0, 1, 2], [0, 2, 3]] if split == "tl-br" else [[0, 1, 3], [1, 2, 3]], np.uint32)
    if flip:
        idx = idx[:, ::-1].copy()
    r = oracle.render_scene(v, idx, cam()[None], H, W, want_cover=True)
    covered = r["tri_id"][0] != NOHIT
    expect = np.zeros((H, W), bool)
    expect[16:48, 8:40] = True          # left/top boundary pixels in, right/bottom out
    assert np.array_equal(covered, expect)
    assert covered.sum() == 32 * 32
    assert np.array_equal(r["cover"][0], expect.astype(np.uint32))   # diagonal pixels exactly once
    assert ulp_diff(r["depth"][0][expect], np.float32(d)).max() <= 4
    assert np.all(r["depth"][0][~expect] == 0.0)


@pytest.mark.parametrize("side", ["left", "right", "top", "bottom"])
def test_facing_quad_clipped_by_each_side_plane(side):
    H = W = 64
    d = 2.0
    v = facing_quad(d, 8, 40, 16, 48, W, H)
    expect = np.zeros((H, W), bool)
    if side == "left":
        v[[0, 3], 0] = -3.0 * d
        expect[16:48, 0:40] = True
    elif side == "right":
        v[[1, 2], 0] = 3.0 * d
        expect[16:48, 8:64] = True
    elif side == "top":
        v[[0, 1], 1] = 3.0 * d
        expect[0:48, 8:40] = True
    else:
        v[[2, 3], 1] = -3.0 * d
        expect[16:64, 8:40] = True
    idx = np.array([[0, 1, 2], [0, 2, 3]], np.uint32)
    r = oracle.render_scene(v, idx, cam()[None], H, W, want_cover=True)
    assert np.array_equal(r["tri_id"][0] != NOHIT, expect)
    assert r["cover"][0].max() == 1
    assert ulp_diff(r["depth"][0][expect], np.float32(d)).max() <= 4


@pytest.mark.parametrize("d,visible", [(0.0101, True), (0.0099, False), (19.99, True), (20.01, False)])
def test_facing_quad_near_and_far_limits(d, visible):
    H = W = 32
    v = facing_quad(d, 4, 20, 4, 20, W, H)
    idx = np.array([[0, 1, 2], [0, 2, 3]], np.uint32)
    r = oracle.render_scene(v, idx, cam()[None], H, W)
    n = int((r["tri_id"][0] != NOHIT).sum())
    if visible:
        assert n == 16 * 16
        assert np.allclose(r["depth"][0][4:20, 4:20], d, rtol=1e-5)
    else:
        assert n == 0


def test_background_value_and_miss_id():
    v = facing_quad(2.0, 2, 6, 2, 6, 16, 16)
    idx = np.array([[0, 1, 2], [0, 2, 3]], np.uint32)
    r = oracle.render_scene(v, idx, cam()[None], 16, 16, background=7.5)
    miss = r["tri_id"][0] == NOHIT
    assert miss.sum() == 256 - 16
    assert np.all(r["depth"][0][miss] == np.float32(7.5))


# ---------------------------------------------------------------- 2. floor / sloped planes

@pytest.mark.parametrize("H,W", [(64, 64), (32, 64)])
def test_level_camera_over_floor_is_perspective_correct(H, W):
    h = 1.25
    far = 200.0
    S = 150.0
    v = np.array([[-S, 0, -S], [S, 0, -S], [S, 0, S], [-S, 0, S]], np.float32)   # two huge triangles
    idx = np.array([[0, 1, 2], [0, 2, 3]], np.uint32)
    aspect = W / H
    M = cam(pos=(0.3, h, -0.2), yaw=0.7, far=far, aspect=aspect)
    r = oracle.render_scene(v, idx, M[None], H, W)
    tan_v = 1.0                                     # hFoV 90 and P[1][1] = -f*aspect: y_n = -y_e * aspect / d
    for j in range(H):
        yn = (j + 0.5) * 2.0 / H - 1.0
        row = r["depth"][0, j]
        if yn <= 0:
            assert np.all(r["tri_id"][0, j] == NOHIT)
            continue
        expect = h * aspect / (yn * tan_v)
        if expect < far * 0.7:                       # rows whose floor point is inside the patch and far plane
            # vertices are snapped to 1/256 px: a row k pixels below the horizon shifts by about 1/(256 k)
            rtol = 2.0 * (1.0 / 256.0) / (j + 0.5 - H / 2) + 1e-5
            assert np.allclose(row, expect, rtol=rtol), (j, row.min(), row.max(), expect)


def test_sloped_plane_against_raycast_depth_with_large_triangles():
    # One large tilted triangle pair: affine interpolation of w would be off by far more than 1e-3.
    v = np.array([[-4, -1, -1.0], [4, -1.5, -2.0], [5, 3, -9.0], [-5, 2.5, -8.0]], np.float32)
    idx = np.array([[0, 1, 2], [0, 2, 3]], np.uint32)
    M = cam()
    r = oracle.render_scene(v, idx, M[None], 64, 64)
    ids, dep, _ = raycast(v, idx, M, 64, 64)
    hit = ids[0] >= 0
    both = hit & (r["tri_id"][0] != NOHIT)
    assert both.sum() > 1500
    assert np.allclose(r["depth"][0][both], dep[0][both], rtol=1e-3)


# ---------------------------------------------------------------- 3. brute-force ray casting

def random_soup(rng, n, spread=3.0, zmin=-8.0, zmax=1.0, size=2.0):
    c = np.stack([rng.uniform(-spread, spread, n), rng.uniform(-spread, spread, n), rng.uniform(zmin, zmax, n)], 1)
    v = c[:, None, :] + rng.uniform(-size, size, (n, 3, 3))
    return v.reshape(-1, 3).astype(np.float32), np.arange(3 * n, dtype=np.uint32).reshape(n, 3)


@pytest.mark.parametrize("seed,n,res", [(0, 40, 16), (1, 120, 32), (2, 200, 64), (3, 60, 64), (4, 200, 16)])
def test_random_soup_matches_raycast(seed, n, res):
    """Triangles cross the near plane and every side plane; ids must agree wherever the
    ray-cast answer is stable under a 2/256-pixel nudge, depths to 1e-3."""
    rng = np.random.default_rng(seed)
    v, idx = random_soup(rng, n)
    M = cam(pos=(0.1, -0.2, 0.5), yaw=0.2 * seed, pitch=0.1 * (seed - 2), near=0.05, far=12.0)
    r = oracle.render_scene(v, idx, M[None], res, res)
    e = 2.0 / 256.0
    ids, dep, gap = raycast(v, idx, M, res, res, offsets=((0, 0), (e, 0), (-e, 0), (0, e), (0, -e)))
    stable = np.all(ids == ids[0:1], axis=0) & np.all(gap > 1e-4, axis=0)
    assert stable.mean() > 0.85
    oid = r["tri_id"][0].astype(np.int64)
    oid[oid == NOHIT] = -1
    assert np.array_equal(oid[stable], ids[0][stable])
    hit = stable & (ids[0] >= 0)
    assert hit.sum() > 0.2 * res * res
    # vertex snapping moves a steep triangle's plane by about what a 2/256-px nudge of the ray does
    with np.errstate(invalid="ignore"):
        slack = 2.0 * np.abs(dep[1:] - dep[0:1]).max(axis=0) + 1e-4 * dep[0]
    assert np.all(np.abs(r["depth"][0] - dep[0])[hit] <= slack[hit])
    assert np.allclose(r["depth"][0][hit], dep[0][hit], rtol=1e-2)


def test_room_scene_matches_raycast_subset():
    """A slice of the smallest benchmark scene through the same check (one camera, 32x32)."""
    w = synth.build_config(1, B=2, scale=0.06)
    s = w.scenes[0]
    M = w.view_proj[1]
    r = oracle.render_scene(s.vertices, s.indices, M[None], 32, 32)
    e = 2.0 / 256.0
    ids, dep, gap = raycast(s.vertices, s.indices, M, 32, 32, offsets=((0, 0), (e, 0), (-e, 0), (0, e), (0, -e)))
    # adjacent coplanar triangles are legitimately ambiguous at shared edges only; the nudge test removes them
    stable = np.all(ids == ids[0:1], axis=0) & np.all(gap > 1e-4, axis=0)
    oid = r["tri_id"][0].astype(np.int64)
    oid[oid == NOHIT] = -1
    assert stable.mean() > 0.5
    assert np.array_equal(oid[stable], ids[0][stable])
    assert np.allclose(r["depth"][0][stable], dep[0][stable], rtol=1e-3)


# ---------------------------------------------------------------- 4. fill rule and watertightness

def load_golden(name):
    tris, rows = [], []
    with open(os.path.join(HERE, "golden", name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("tri"):
                tris.append([int(t) for t in line.split()[1:]])
            else:
                rows.append([int(ch) for ch in line])
    return np.array(tris, np.int32).reshape(-1, 3, 2), np.array(rows, np.uint32)


@pytest.mark.parametrize("name", ["fill_rule_upper_left.txt", "fill_rule_lower_right.txt",
                                  "fill_rule_centre_corners.txt"])
def test_hand_enumerated_fill_rule(name):
    tris, expect = load_golden(name)
    got = oracle.cover_fixed(tris, expect.shape[0], expect.shape[1])
    assert np.array_equal(got, expect)
    # vertex order and winding must not matter
    for perm in ([1, 2, 0], [2, 0, 1], [0, 2, 1], [2, 1, 0], [1, 0, 2]):
        assert np.array_equal(oracle.cover_fixed(tris[:, perm, :], *expect.shape), expect)


def strictly_inside_convex(poly, px, py):
    """Exact integer test: strictly inside / strictly outside a convex polygon (any winding)."""
    poly = [(int(x), int(y)) for x, y in poly]
    n = len(poly)
    signs = []
    for k in range(n):
        (x0, y0), (x1, y1) = poly[k], poly[(k + 1) % n]
        signs.append((x1 - x0) * (py - y0) - (y1 - y0) * (px - x0))
    signs = np.array(signs)
    inside = np.all(signs > 0, axis=0) | np.all(signs < 0, axis=0)
    outside = (np.any(signs > 0, axis=0) & np.any(signs < 0, axis=0))
    return inside, outside


def test_shared_edge_pairs_cover_each_pixel_once():
    rng = np.random.default_rng(11)
    H = W = 16
    jj, ii = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    px, py = 256 * ii + 128, 256 * jj + 128
    checked = 0
    for trial in range(1500):
        # convex quad = two triangles sharing the diagonal a-c; snap some vertices onto pixel centres
        while True:
            q = rng.integers(-300, 256 * W + 300, size=(4, 2))
            if trial % 3 == 0:
                q = (q // 256) * 256 + 128
            elif trial % 3 == 1:
                q[:, 0] = (q[:, 0] // 128) * 128
            c = [int((q[(k + 1) % 4, 0] - q[k, 0]) * (q[(k + 2) % 4, 1] - q[(k + 1) % 4, 1])
                     - (q[(k + 1) % 4, 1] - q[k, 1]) * (q[(k + 2) % 4, 0] - q[(k + 1) % 4, 0])) for k in range(4)]
            if all(x > 0 for x in c) or all(x < 0 for x in c):
                break
        tris = np.array([[q[0], q[1], q[2]], [q[0], q[2], q[3]]])
        cover = oracle.cover_fixed(tris, H, W)
        inside, outside = strictly_inside_convex(q, px, py)
        assert cover.max() <= 1, trial
        assert np.all(cover[inside] == 1), trial
        assert np.all(cover[outside] == 0), trial
        checked += int(inside.sum())
    assert checked > 20000


def test_fans_and_jittered_grids_are_watertight():
    rng = np.random.default_rng(5)
    H = W = 24
    jj, ii = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    px, py = 256 * ii + 128, 256 * jj + 128
    n_fans = n_grids = 0
    # (a) fan around an interior vertex of a convex polygon
    for trial in range(300):
        n = int(rng.integers(3, 12))
        ang = np.sort(rng.uniform(0, 2 * np.pi, n))
        rad = rng.uniform(500, 2800)
        c = rng.integers(2000, 4000, 2)
        poly = np.stack([c[0] + rad * np.cos(ang), c[1] + rad * np.sin(ang)], 1).round().astype(np.int64)
        if trial % 2:
            poly = (poly // 128) * 128
            c = (c // 128) * 128
        cr = [(poly[(k + 1) % n] - poly[k]) for k in range(n)]
        z = [int(cr[k][0] * cr[(k + 1) % n][1] - cr[k][1] * cr[(k + 1) % n][0]) for k in range(n)]
        ins_c, _ = strictly_inside_convex(poly, np.array([c[0]]), np.array([c[1]]))
        if not (all(v > 0 for v in z) and ins_c[0]):
            continue
        tris = np.array([[c, poly[k], poly[(k + 1) % n]] for k in range(n)])
        cover = oracle.cover_fixed(tris, H, W)
        inside, outside = strictly_inside_convex(poly, px, py)
        assert cover.max() <= 1
        assert np.all(cover[inside] == 1) and np.all(cover[outside] == 0)
        n_fans += 1
    # (b) jittered grid with random diagonals; boundary is an axis-aligned rectangle
    for trial in range(40):
        n = 9
        base = np.arange(n + 1) * 600 + 200
        gx, gy = np.meshgrid(base, base)
        jit = rng.integers(-250, 251, size=(n + 1, n + 1, 2))
        jit[0, :], jit[-1, :], jit[:, 0], jit[:, -1] = 0, 0, 0, 0
        P = np.stack([gx + jit[..., 0], gy + jit[..., 1]], -1)
        if trial % 2:
            P = (P // 64) * 64
        tris = []
        for r in range(n):
            for q in range(n):
                a, b, c2, d = P[r, q], P[r, q + 1], P[r + 1, q + 1], P[r + 1, q]
                tris += [[a, b, c2], [a, c2, d]] if rng.integers(0, 2) else [[a, b, d], [b, c2, d]]
        tris = np.array(tris)
        a2 = ((tris[:, 1, 0] - tris[:, 0, 0]) * (tris[:, 2, 1] - tris[:, 0, 1])
              - (tris[:, 2, 0] - tris[:, 0, 0]) * (tris[:, 1, 1] - tris[:, 0, 1]))
        if np.any(a2 <= 0):          # a jitter folded a cell over: not a valid planar mesh
            continue
        cover = oracle.cover_fixed(tris, H, W)
        rect = np.array([P[0, 0], P[0, -1], P[-1, -1], P[-1, 0]])
        inside, outside = strictly_inside_convex(rect, px, py)
        assert cover.max() <= 1
        assert np.all(cover[inside] == 1) and np.all(cover[outside] == 0)
        n_grids += 1
    assert n_fans > 100 and n_grids > 20


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_jittered_wall_through_clipper_is_watertight(seed):
    """A tessellated plane filling the whole view, straddling every side plane and (for
    oblique close cameras) the near plane: every pixel is covered exactly once, which
    pins the canonical inside->outside interpolation of the clipper."""
    rng = np.random.default_rng(100 + seed)
    n = 26
    u = np.linspace(-30, 30, n + 1)
    U, Vv = np.meshgrid(u, u)
    jit = rng.uniform(-0.3, 0.3, size=(n + 1, n + 1, 2))
    jit[0, :], jit[-1, :], jit[:, 0], jit[:, -1] = 0, 0, 0, 0
    P = np.stack([U + jit[..., 0], Vv + jit[..., 1], np.full_like(U, -3.0)], -1).reshape(-1, 3).astype(np.float32)
    a = (np.arange(n)[:, None] * (n + 1) + np.arange(n)[None, :]).ravel()
    flip = rng.integers(0, 2, a.size).astype(bool)
    t1 = np.where(flip[:, None], np.stack([a, a + 1, a + n + 1], 1), np.stack([a, a + 1, a + n + 2], 1))
    t2 = np.where(flip[:, None], np.stack([a + 1, a + n + 2, a + n + 1], 1), np.stack([a, a + n + 2, a + n + 1], 1))
    idx = np.concatenate([t1, t2], 0).astype(np.uint32)
    e = 2.0 / 256.0
    offs = ((0, 0), (e, 0), (-e, 0), (0, e), (0, -e))
    n_hit = 0
    for k in range(4):
        pos = (rng.uniform(-5, 5), rng.uniform(-5, 5), rng.uniform(-2.93, 0.0))
        yaw, pitch = rng.uniform(-1.0, 1.0), rng.uniform(-0.8, 0.8)
        M = cam(pos=pos, yaw=yaw, pitch=pitch, near=0.05, far=500.0)
        r = oracle.render_scene(P, idx, M[None], 32, 32, want_cover=True)
        ids, _, _ = raycast(P, idx, M, 32, 32, offsets=offs)
        hit_all = np.all(ids >= 0, axis=0)
        miss_all = np.all(ids < 0, axis=0)
        assert r["cover"][0].max() <= 1                       # never twice, anywhere
        assert np.all(r["cover"][0][hit_all] == 1)            # no cracks
        assert np.all(r["cover"][0][miss_all] == 0)
        n_hit += int(hit_all.sum())
    assert n_hit > 2500


# ---------------------------------------------------------------- 5. invariants

def small_workload():
    w = synth.build_config(1, B=4)
    return w, w.scenes[0]


def test_closed_room_has_no_background_and_depth_in_range():
    w, s = small_workload()
    r = oracle.render_scene(s.vertices, s.indices, w.view_proj, 64, 64)
    assert (r["tri_id"] == NOHIT).sum() == 0
    assert r["depth"].min() >= 0.01
    assert r["depth"].max() <= 20.0 * (1 + 1e-6)
    assert r["depth"].max() <= math.sqrt(10 ** 2 + 8 ** 2 + 3 ** 2)


def test_index_permutation_permutes_ids_only():
    w, s = small_workload()
    r0 = oracle.render_scene(s.vertices, s.indices, w.view_proj, 64, 64)
    perm = np.random.default_rng(3).permutation(s.T)
    r1 = oracle.render_scene(s.vertices, s.indices[perm], w.view_proj, 64, 64)
    same_depth = r0["depth"] == r1["depth"]
    assert same_depth.all()                       # depth is the minimum either way
    mapped = perm[r1["tri_id"]]
    differ = mapped != r0["tri_id"]
    # ids may differ only where two triangles tie exactly in depth
    assert differ.mean() < 0.02


def test_vertex_rotation_within_triangles_keeps_coverage():
    w, s = small_workload()
    r0 = oracle.render_scene(s.vertices, s.indices, w.view_proj, 64, 64, want_cover=True)
    rolled = np.roll(s.indices, 1, axis=1)
    r1 = oracle.render_scene(s.vertices, rolled, w.view_proj, 64, 64, want_cover=True)
    assert np.array_equal(r0["cover"], r1["cover"])
    assert np.array_equal(r0["tri_id"], r1["tri_id"])
    # a clipped triangle fans from a different vertex after rotation; the snapped pieces then
    # span slightly different planes (most visibly on slivers seen edge-on), so depth agrees
    # closely but not to the last bits; unclipped triangles must agree to rounding
    assert np.allclose(r0["depth"], r1["depth"], rtol=1e-3)
    assert np.mean(np.abs(r0["depth"] - r1["depth"]) > 1e-5 * r0["depth"]) < 0.05


def test_exact_depth_tie_goes_to_lower_triangle_id():
    v = facing_quad(2.0, 2, 10, 2, 10, 16, 16)
    idx = np.array([[0, 1, 2], [0, 2, 3], [0, 1, 2], [0, 2, 3]], np.uint32)   # every triangle twice
    r = oracle.render_scene(v, idx, cam()[None], 16, 16, want_cover=True)
    hit = r["tri_id"][0] != NOHIT
    assert hit.sum() == 64
    assert r["tri_id"][0][hit].max() <= 1
    assert np.all(r["cover"][0][hit] == 2)


def test_degenerate_hidden_and_subpixel_triangles_contribute_nothing():
    M = cam()
    v = np.array([
        [0, 0, -2], [1, 1, -2], [2, 2, -2],                 # zero area
        [0, 0, 3], [1, 0, 3], [0, 1, 3],                    # behind the camera
        [0.001, 0.001, -2], [0.004, 0.001, -2], [0.001, 0.004, -2],   # between pixel centres
        [50, 0, -2], [51, 0, -2], [50, 1, -2],              # outside the right plane
        [np.nan, 0, -2], [1, 0, -2], [0, 1, -2],            # non-finite vertex
    ], np.float32)
    idx = np.arange(15, dtype=np.uint32).reshape(5, 3)
    r = oracle.render_scene(v, idx, M[None], 64, 64)
    assert (r["tri_id"] != NOHIT).sum() == 0


def test_nearer_triangle_wins_and_orthographic_depth_is_affine():
    # orthographic matrix (w == 1): depth must be exactly 1 everywhere, ids decided by the tie rule
    M = np.array([[0.25, 0, 0, 0], [0, 0.25, 0, 0], [0, 0, -0.1, 0], [0, 0, 0, 1]], np.float32)
    v = np.array([[-2, -2, -1], [2, -2, -1], [0, 3, -1], [-3, -1, -5], [3, -1, -5], [0, 2, -5]], np.float32)
    idx = np.array([[3, 4, 5], [0, 1, 2]], np.uint32)
    r = oracle.render_scene(v, idx, M[None], 32, 32)
    hit = r["tri_id"][0] != NOHIT
    assert hit.sum() > 100
    assert np.all(r["depth"][0][hit] == 1.0)
    # perspective: put triangle 1 nearer than triangle 0 -> it must win wherever both cover
    Mp = cam()
    r2 = oracle.render_scene(v, idx, Mp[None], 32, 32, want_cover=True)
    both = r2["cover"][0] == 2
    assert both.sum() > 5
    assert np.all(r2["tri_id"][0][both] == 1)
    assert np.allclose(r2["depth"][0][both], 1.0, rtol=1e-5)


def test_clipper_output_lies_in_the_frustum_and_keeps_plane_area():
    """The clipped polygon of a camera-facing triangle has the area of (triangle ∩ view square)."""
    rng = np.random.default_rng(8)
    M = cam()
    d = 2.0
    for _ in range(200):
        tri = np.concatenate([rng.uniform(-3 * d, 3 * d, (3, 2)), np.full((3, 1), -d)], 1).astype(np.float32)
        poly = oracle.clip(M, tri)
        # reference area: float64 half-plane cuts of the triangle against the view square, written separately
        ref_area = _clip_area_reference(tri[:, :2].astype(np.float64), d)
        if poly.shape[0] == 0:
            assert ref_area < 1e-6
            continue
        assert np.all(np.abs(poly[:, 0]) <= poly[:, 3] * (1 + 1e-5))
        assert np.all(np.abs(poly[:, 1]) <= poly[:, 3] * (1 + 1e-5))
        xy = poly[:, :2].astype(np.float64)
        area = 0.5 * abs(np.sum(xy[:, 0] * np.roll(xy[:, 1], -1) - np.roll(xy[:, 0], -1) * xy[:, 1]))
        assert abs(area - ref_area) <= 1e-4 * max(1.0, ref_area)


def _clip_area_reference(tri, d):
    """Area of triangle ∩ [-d,d]^2 in float64 by successive half-plane cuts."""
    poly = [tuple(p) for p in tri]
    for axis, sign in ((0, 1), (0, -1), (1, 1), (1, -1)):
        out = []
        for i in range(len(poly)):
            a, b = poly[i], poly[(i + 1) % len(poly)]
            da, db = d - sign * a[axis], d - sign * b[axis]
            if da >= 0:
                out.append(a)
            if (da >= 0) != (db >= 0):
                t = da / (da - db)
                out.append((a[0] + t * (b[0] - a[0]), a[1] + t * (b[1] - a[1])))
        poly = out
        if len(poly) < 3:
            return 0.0
    xy = np.array(poly)
    return 0.5 * abs(np.sum(xy[:, 0] * np.roll(xy[:, 1], -1) - np.roll(xy[:, 0], -1) * xy[:, 1]))


def test_colour_interpolation_constant_and_linear():
    """Constant vertex colour stays constant; on a camera-facing quad colour is affine in the pixel index."""
    H = W = 32
    v = facing_quad(2.0, 0, 31, 0, 31, W, H)
    idx = np.array([[0, 1, 2], [0, 2, 3]], np.uint32)
    col = np.array([[10, 200, 30]] * 4, np.uint8)
    r = oracle.render_scene(v, idx, cam()[None], H, W, colors=col)
    hit = r["tri_id"][0] != NOHIT
    assert np.all(r["rgb"][0][hit] == np.array([10, 200, 30], np.uint8))
    col = np.array([[0, 0, 0], [248, 0, 0], [248, 248, 0], [0, 248, 0]], np.uint8)   # r = 8 i, g = 8 j
    r = oracle.render_scene(v, idx, cam()[None], H, W, colors=col)
    jj, ii = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    assert np.all(np.abs(r["rgb"][0][..., 0].astype(int) - 8 * ii)[hit] <= 1)
    assert np.all(np.abs(r["rgb"][0][..., 1].astype(int) - 8 * jj)[hit] <= 1)
    assert np.all(r["rgb"][0][..., 2][hit] == 0)


def test_colour_is_perspective_correct_on_a_receding_plane():
    # floor quad receding from the camera; colour r encodes world z; compare with the ray-cast hit point
    v = np.array([[-50, -1, 0], [50, -1, 0], [50, -1, -25.5], [-50, -1, -25.5]], np.float32)
    idx = np.array([[0, 1, 2], [0, 2, 3]], np.uint32)
    col = np.array([[0, 0, 0], [0, 0, 0], [255, 0, 0], [255, 0, 0]], np.uint8)       # r = -10 z
    M = cam(far=100.0)
    r = oracle.render_scene(v, idx, M[None], 64, 64, colors=col)
    hit = r["tri_id"][0] != NOHIT
    # hit point on the plane y = -1 along the view axis: z = -depth
    expect = np.clip(np.rint(10.0 * r["depth"][0]), 0, 255)
    assert hit.sum() > 1000
    assert np.all(np.abs(r["rgb"][0][..., 0].astype(int) - expect.astype(int))[hit] <= 1)


# ---------------------------------------------------------------- 6. snapping and canonical clipping

@pytest.mark.parametrize("frac,left_in", [(0.25, True), (0.75, False), (-0.25, True), (-0.75, True)])
def test_snapping_rounds_to_nearest_subpixel(frac, left_in):
    """A quad edge `frac`/256 px right of a pixel-centre line snaps to the nearest 1/256 px:
    +0.25 -> onto the line (pixel kept by the left-edge rule), +0.75 -> one unit right (pixel lost);
    truncation or floor instead of rounding would flip one of these cases."""
    H = W = 64
    d = 2.0
    v = facing_quad(d, 8, 40, 16, 48, W, H)
    fx = 256.0 * 8 + 128.0 + frac                      # wanted un-rounded coordinate, exact in binary32
    x = (fx / (128.0 * W) - 1.0) * d
    v[[0, 3], 0] = x
    idx = np.array([[0, 1, 2], [0, 2, 3]], np.uint32)
    r = oracle.render_scene(v, idx, cam()[None], H, W)
    col8 = r["tri_id"][0][16:48, 8] != NOHIT
    assert np.all(col8 == left_in)
    assert np.all(r["tri_id"][0][16:48, 9] != NOHIT)
    assert np.all(r["tri_id"][0][16:48, 7] == NOHIT) or frac < -0.5   # -0.75 snaps one unit left: still right of centre 7


def test_clipper_generates_bit_identical_points_on_shared_edges():
    """Two triangles sharing edge PQ, walked in opposite directions, must produce the very same
    crossing point where PQ leaves the frustum (interpolation always runs inside -> outside)."""
    rng = np.random.default_rng(21)
    M = cam(pos=(0.2, 0.1, 0.3), yaw=0.3, pitch=-0.2, near=0.5, far=9.0)
    found = 0
    for _ in range(400):
        P = np.array([rng.uniform(-1, 1), rng.uniform(-1, 1), rng.uniform(-6, -2)], np.float32)     # inside
        Q = P + rng.uniform(-12, 12, 3).astype(np.float32)                                          # mostly outside
        R1 = P + rng.uniform(-1, 1, 3).astype(np.float32)
        R2 = P + rng.uniform(-1, 1, 3).astype(np.float32)
        a = oracle.clip(M, np.stack([P, Q, R1]))
        b = oracle.clip(M, np.stack([Q, P, R2]))
        c = oracle.clip(M, np.stack([R2, Q, P]))
        if a.shape[0] <= 3 or b.shape[0] <= 3:
            continue
        # every generated point on PQ seen by one triangle must be seen, bit for bit, by the others
        pq = [{row.tobytes() for row in poly if _on_segment(row, M, P, Q)} for poly in (a, b, c)]
        assert pq[0] == pq[1] == pq[2]
        found += bool(pq[0])
    assert found > 100


def _on_segment(g, M, P, Q):
    """Is clip-space point g (approximately) on the image of segment PQ and not an endpoint?"""
    M = M.astype(np.float64)
    p = M @ np.append(P.astype(np.float64), 1.0)
    q = M @ np.append(Q.astype(np.float64), 1.0)
    d = q - p
    t = np.dot(g.astype(np.float64) - p, d) / np.dot(d, d)
    if not (1e-4 < t < 1 - 1e-4):
        return False
    return np.linalg.norm(p + t * d - g) <= 1e-4 * (1 + np.linalg.norm(g))


# ---------------------------------------------------------------- 7. textures (rule N10)

def _pyramid_reference(tex):
    """Independent numpy construction of the mip pyramid: (a+b+c+d+2)>>2 over 2x2 parents."""
    levels = [tex.astype(np.int32)]
    while levels[-1].shape[0] > 1 or levels[-1].shape[1] > 1:
        t = levels[-1]
        h, w = t.shape[:2]
        ys = np.minimum(np.arange(max(h // 2, 1))[:, None] * 2 + np.array([0, 1])[None, :], h - 1)
        xs = np.minimum(np.arange(max(w // 2, 1))[:, None] * 2 + np.array([0, 1])[None, :], w - 1)
        s = (t[ys[:, 0]][:, xs[:, 0]] + t[ys[:, 0]][:, xs[:, 1]] + t[ys[:, 1]][:, xs[:, 0]] + t[ys[:, 1]][:, xs[:, 1]])
        levels.append((s + 2) >> 2)
    return [l.astype(np.uint8) for l in levels]


def _corner_quad(d, W, H):
    """Camera-facing quad at distance d exactly filling the frame (corners on the frame corners)."""
    return np.array([[-d, d, -d], [d, d, -d], [d, -d, -d], [-d, -d, -d]], np.float32)


def test_texture_sampling_rule_on_single_lookups():
    rng = np.random.default_rng(4)
    tex = rng.integers(0, 256, (8, 16, 3)).astype(np.uint8)          # h = 8, w = 16
    pyr = _pyramid_reference(tex)
    assert [p.shape[:2] for p in pyr] == [(8, 16), (4, 8), (2, 4), (1, 2), (1, 1)]
    for L, lv in enumerate(pyr):
        lh, lw = lv.shape[:2]
        for (u, v) in [(0.0, 0.0), (0.5, 0.5), (0.999999, 0.999999), (1.0, 1.0), (-0.25, 2.75), (3.0625, -1.9375)]:
            fu, fv = u - math.floor(u), v - math.floor(v)
            x, y = min(int(np.float32(fu) * lw), lw - 1), min(int(np.float32(fv) * lh), lh - 1)
            assert np.array_equal(oracle.sample(tex, L, u, v), lv[y, x]), (L, u, v)
    assert np.array_equal(oracle.sample(tex, 0, float("nan"), float("inf")), tex[0, 0])
    assert np.array_equal(oracle.sample(tex, 99, 0.7, 0.2), pyr[-1][0, 0])    # level clamps to the last one
    assert np.array_equal(oracle.sample(tex, 0, -1e-9, 0.0), tex[0, 0])       # frac rounds to 1.0: guarded


@pytest.mark.parametrize("scale,level", [(1, 0), (2, 1), (4, 2), (8, 3)])
def test_textured_quad_picks_the_expected_mip_level_and_texel(scale, level):
    """Frame-filling quad, uv 0..1, texture `scale` times the frame size: every pixel covers
    scale x scale texels, so the level is log2(scale) and pixel (i, j) shows that level's texel (i, j)."""
    H = W = 32
    rng = np.random.default_rng(9)
    tex = rng.integers(0, 256, (H * scale, W * scale, 3)).astype(np.uint8)
    v = _corner_quad(2.0, W, H)
    uv = np.array([[0, 0], [1, 0], [1, 1], [0, 1]], np.float32)
    idx = np.array([[0, 1, 2], [0, 2, 3]], np.uint32)
    r = oracle.render_scene(v, idx, cam()[None], H, W, uvs=uv, texture=tex)
    assert (r["tri_id"][0] != NOHIT).all()
    assert np.array_equal(r["rgb"][0], _pyramid_reference(tex)[level])


def test_texture_wraps_and_constant_texture_gives_constant_colour():
    H = W = 16
    v = _corner_quad(2.0, W, H)
    idx = np.array([[0, 1, 2], [0, 2, 3]], np.uint32)
    tex = np.random.default_rng(1).integers(0, 256, (8, 8, 3)).astype(np.uint8)
    uv = np.array([[0, 0], [2, 0], [2, 2], [0, 2]], np.float32)          # two repeats across the frame
    r = oracle.render_scene(v, idx, cam()[None], H, W, uvs=uv, texture=tex)
    assert np.array_equal(r["rgb"][0], np.tile(tex, (2, 2, 1)))
    uv3 = uv - 5.0                                                        # negative coordinates wrap the same way
    r3 = oracle.render_scene(v, idx, cam()[None], H, W, uvs=uv3, texture=tex)
    assert np.array_equal(r3["rgb"][0], np.tile(tex, (2, 2, 1)))
    flat = np.full((4, 4, 3), (9, 99, 199), np.uint8)
    r2 = oracle.render_scene(v, idx, cam()[None], H, W, uvs=uv * 7.3, texture=flat)
    assert np.all(r2["rgb"][0] == np.array([9, 99, 199], np.uint8))


def test_texture_coordinates_are_perspective_correct():
    """Receding floor: the texel column must follow the ray-cast hit point, not an affine guess."""
    v = np.array([[-40, -1, 0], [40, -1, 0], [40, -1, -32], [-40, -1, -32]], np.float32)
    uv = np.array([[0, 0], [1, 0], [1, 1], [0, 1]], np.float32)          # v runs with distance, 32 m per repeat
    idx = np.array([[0, 1, 2], [0, 2, 3]], np.uint32)
    tex = np.zeros((32, 4, 3), np.uint8)
    tex[:, :, 0] = np.arange(32)[:, None] * 8                             # red encodes the row = metres from the camera
    M = cam(far=100.0)
    r = oracle.render_scene(v, idx, M[None], 64, 64, uvs=uv, texture=tex)
    hit = r["tri_id"][0] != NOHIT
    assert hit.sum() > 1000
    # depth along the view axis == distance in -z here; level 0 as long as a pixel sees < 2 texel rows
    near = hit & (r["depth"][0] < 6.0)
    expect_row = np.floor(r["depth"][0]).astype(int)
    got_row = r["rgb"][0][..., 0].astype(int) // 8
    frac = r["depth"][0] - np.floor(r["depth"][0])
    safe = near & (frac > 0.02) & (frac < 0.98)
    assert safe.sum() > 300
    assert np.array_equal(got_row[safe], expect_row[safe])


def test_mip_level_uses_the_uv_area_of_a_sheared_mapping():
    """uv = A p with det(A) = 3 texel areas per pixel area at level 0 (level 0 expected); a wrong
    cross product (e.g. du1 dv1 - du2 dv2, which gives 6) would pick level 1 and other texels."""
    H = W = 32
    rng = np.random.default_rng(12)
    tex = rng.integers(0, 256, (W, W, 3)).astype(np.uint8)
    k = math.sqrt(3.0 / 5.0)
    A = np.array([[2.0, 1.0], [1.0, 3.0]]) * k
    corners = np.array([[0, 0], [1, 0], [1, 1], [0, 1]], np.float64)          # frame coordinates of the quad's corners
    uv = (corners @ A.T).astype(np.float32)
    v = _corner_quad(2.0, W, H)
    idx = np.array([[0, 1, 2], [0, 2, 3]], np.uint32)
    r = oracle.render_scene(v, idx, cam()[None], H, W, uvs=uv, texture=tex)
    jj, ii = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    p = np.stack([(ii + 0.5) / W, (jj + 0.5) / H], -1)
    uvp = p @ A.T
    fr = uvp - np.floor(uvp)
    tx, ty = fr[..., 0] * W, fr[..., 1] * W
    safe = (np.abs(tx - np.round(tx)) > 1e-2) & (np.abs(ty - np.round(ty)) > 1e-2)
    expect = tex[np.minimum(ty.astype(int), W - 1), np.minimum(tx.astype(int), W - 1)]
    assert safe.mean() > 0.9
    assert np.array_equal(r["rgb"][0][safe], expect[safe])


# ---------------------------------------------------------------- supersampled output and the clipper's capacity

def test_box_filter_hand_computed_block_and_constant_plane():
    """2x2 box filter of supersampled frames: one block worked out by hand (a background sample
    counts with the frame's background value; the sum is taken pairwise, rows first), a constant
    frame stays what it is, colours round half up."""
    d = np.zeros((1, 4, 4), np.float32)
    d[0, 0:2, 0:2] = [[1.5, 2.5], [0.0, 4.0]]                 # 0.0 = a background sample
    d[0, 0:2, 2:4] = [[np.float32(1e8), 1.0], [-np.float32(1e8), 1.0]]   # order matters: (1e8 + 1) + (-1e8 + 1) = 0 in float32
    d[0, 2:4, :] = 7.25
    c = np.zeros((1, 4, 4, 3), np.uint8)
    c[0, 0:2, 0:2, 0] = [[1, 2], [3, 4]]                      # 10 + 2 >> 2 = 3
    c[0, 0:2, 0:2, 1] = [[255, 255], [255, 254]]              # 1019 + 2 >> 2 = 255
    c[0, 0:2, 0:2, 2] = [[0, 0], [0, 1]]                      # 1 + 2 >> 2 = 0
    od, oc = oracle.downsample2(d, c)
    assert od.shape == (1, 2, 2) and oc.shape == (1, 2, 2, 3)
    assert od[0, 0, 0] == np.float32(2.0)                     # (1.5 + 2.5) + (0 + 4) = 8, / 4
    assert od[0, 0, 1] == np.float32(0.0)                     # both row sums round to +-1e8
    assert od[0, 1, 0] == np.float32(7.25) and od[0, 1, 1] == np.float32(7.25)
    assert tuple(oc[0, 0, 0]) == (3, 255, 0)
    assert np.all(oc[0, 1] == 0)
    plane = np.full((3, 16, 24), 3.375, np.float32)
    assert np.all(oracle.downsample2(plane)[0] == np.float32(3.375))


def test_clipper_capacity_is_never_reached_and_is_reported_if_it_were():
    """Clip-heavy random soups, cameras inside the geometry: the largest polygon the clipper ever
    builds stays well below its 16 corners (nine in exact arithmetic), and no polygon is dropped
    for lack of room.  Every render call would fail loudly otherwise."""
    oracle.clip_stats(reset=True)
    for seed in range(6):
        rng = np.random.default_rng(100 + seed)
        v, idx = random_soup(rng, 400, spread=2.0, zmin=-3.0, zmax=2.0, size=4.0)
        M = cam(pos=(0.1 * seed, -0.2, 0.5), yaw=0.7 * seed, pitch=0.3 * (seed - 3), near=0.05, far=6.0)
        oracle.render_scene(v, idx, M[None], 32, 32)
    w = synth.build_config(2, B=6, scale=0.02)
    oracle.render_batch(w.scenes, w.scene_ids, w.view_proj, 64, 64)
    overflows, largest = oracle.clip_stats()
    assert overflows == 0
    assert 7 <= largest <= 10, largest          # six planes cut: up to nine corners, one more through rounding at most


# ---------------------------------------------------------------- bilinear texture filtering (rule N11)

def test_bilinear_constant_texture_texel_centres_and_midpoints():
    """N11 against what bilinear filtering must give: a constant texture stays constant; at a texel
    centre the result is that texel; halfway between two texels it is their mean (a tie rounds to
    even, as the rule's lrint says); a linear ramp is reproduced exactly between texel centres."""
    rng = np.random.default_rng(5)
    const = np.full((8, 8, 3), (17, 200, 93), np.uint8)
    for u, v in rng.uniform(-3, 3, (50, 2)):
        assert tuple(oracle.sample(const, 0, u, v, bilinear=True)) == (17, 200, 93)
    tex = rng.integers(0, 256, (8, 16, 3), dtype=np.uint8)           # 16 wide, 8 high
    for _ in range(60):
        i, j = int(rng.integers(0, 16)), int(rng.integers(0, 8))
        got = oracle.sample(tex, 0, (i + 0.5) / 16 + int(rng.integers(-2, 3)), (j + 0.5) / 8, bilinear=True)
        assert np.array_equal(got, tex[j, i])
    ramp = np.zeros((4, 8, 3), np.uint8)
    ramp[:, :, 0] = np.arange(8) * 10                                 # value 10 x at texel x
    ramp[:, :, 1] = (np.arange(4) * 20)[:, None]
    for x in (1.0, 1.25, 2.5, 3.75, 6.0):                             # in texel-centre units, away from the wrap
        got = oracle.sample(ramp, 0, (x + 0.5) / 8, (1.5 + 0.5) / 4, bilinear=True)
        assert got[0] == int(np.rint(10 * x)) and got[1] == 30        # halfway between rows 1 and 2: (20 + 40) / 2
    two = np.zeros((1, 2, 3), np.uint8)
    two[0, 0], two[0, 1] = (10, 0, 0), (11, 0, 0)
    assert oracle.sample(two, 0, 0.5, 0.5, bilinear=True)[0] == 10    # 10.5 rounds to even


def test_bilinear_wraps_at_the_border_and_uses_the_chosen_level():
    """The texture repeats: left of the first texel centre the last texel of the row is blended in
    (and above the first row the last one); at a coarser level the same rule applies to that level's
    texels (the pyramid is N10's)."""
    ramp = np.zeros((4, 8, 3), np.uint8)
    ramp[:, :, 0] = np.arange(8) * 10
    ramp[:, :, 1] = (np.arange(4) * 20)[:, None]
    assert oracle.sample(ramp, 0, 0.0, 0.125, bilinear=True)[0] == 35         # halfway between texel 7 (70) and texel 0 (0)
    assert oracle.sample(ramp, 0, 1.0 / 64, 0.125, bilinear=True)[0] == 26    # x = -0.375: 0.375 * 70 = 26.25
    assert oracle.sample(ramp, 0, 1.0 / 16, 0.0, bilinear=True)[1] == 30      # halfway between row 3 (60) and row 0 (0)
    # level 1 of the ramp: texels (0+10)/2 ... -> 5, 25, 45, 65 (rounded pyramid), two rows 10 and 50
    assert [int(oracle.sample(ramp, 1, (i + 0.5) / 4, 0.25, bilinear=True)[0]) for i in range(4)] == [5, 25, 45, 65]
    assert oracle.sample(ramp, 1, 0.5, 0.25, bilinear=True)[0] == 35          # between 25 and 45
    assert oracle.sample(ramp, 1, 0.375, 0.5, bilinear=True)[1] == 30         # between rows 10 and 50 of level 1
    one = np.full((1, 1, 3), 77, np.uint8)
    assert tuple(oracle.sample(one, 0, 0.3, 0.9, bilinear=True)) == (77, 77, 77)


def test_bilinear_render_of_a_camera_facing_textured_quad():
    """Through the renderer: a camera-facing quad whose texture coordinates put exactly one texel on
    every pixel, shifted by half a texel, shows the mean of horizontally adjacent texels; with the
    nearest rule the same picture shows single texels."""
    H = W = 16
    z = -2.0
    v = np.array([[-2, -2, z], [2, -2, z], [2, 2, z], [-2, 2, z]], np.float32)     # fills the 90-degree view exactly
    idx = np.array([[0, 1, 2], [0, 2, 3]], np.uint32)
    tex = np.random.default_rng(9).integers(0, 256, (16, 16, 3), dtype=np.uint8)
    shift = 0.5 / 16
    uv0 = np.array([[0, 1], [1, 1], [1, 0], [0, 0]], np.float32)      # pixel (i, j) looks at the centre of one texel
    uv = uv0 + np.array([shift, 0], np.float32)                       # ... and now at the border of texels i and i + 1
    M = cam()
    near = oracle.render_scene(v, idx, M[None], H, W, uvs=uv0, texture=tex)
    lin0 = oracle.render_scene(v, idx, M[None], H, W, uvs=uv0, texture=tex, bilinear=True)
    lin = oracle.render_scene(v, idx, M[None], H, W, uvs=uv, texture=tex, bilinear=True)
    assert np.all(near["tri_id"][0] != NOHIT)
    # which texel row each image row shows (unambiguous: texel centres)
    rows = [int(np.flatnonzero(np.all(near["rgb"][0, j, 4] == tex[:, 4], axis=1))[0]) for j in range(H)]
    assert sorted(rows) == list(range(16))
    for j in range(H):
        assert np.array_equal(near["rgb"][0, j], tex[rows[j]])
    # at texel centres filtering changes nothing (up to the rounding of the interpolated coordinates: the
    # weight of the neighbour is at most a few 1e-6)
    assert np.array_equal(lin0["rgb"][0], near["rgb"][0])
    t = tex.astype(np.int32)
    for j in range(H):
        for i in range(W - 1):
            pair = t[rows[j], i] + t[rows[j], i + 1]
            got = lin["rgb"][0, j, i].astype(np.int32)
            even = pair % 2 == 0
            assert np.all(got[even] == pair[even] // 2)                       # the mean of the two texels
            assert np.all(np.abs(2 * got[~even] - pair[~even]) == 1)          # a tie: either neighbour of the half
