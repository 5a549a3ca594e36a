"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, element by element."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu
NOHIT = 0xFFFFFFFF


def _render_gpu(scenes, scene_ids, view_proj, H, W, splits=0, threads=0, background=0.0, device_matrices=False,
                flags=0):
    import torch
    import paper_2103_07013_amd as bps
    B = len(scene_ids)
    with bps.Renderer(max_batch=B, height=H, width=W, splits=splits, threads=threads,
                      background_depth=background, flags=flags) as r:
        handles = [r.load_scene(s.vertices, s.indices, s.colors) for s in scenes]
        ids = np.array([handles[k] for k in scene_ids], np.int32)
        vp = torch.from_numpy(np.ascontiguousarray(view_proj)).cuda() if device_matrices else view_proj
        depth, _, tid = r.render(ids, vp, want_tri_id=True)
        torch.cuda.synchronize()
        info = dict(splits=bps.bps_query(r.handle, 0, 4), groups=bps.bps_query(r.handle, 0, 5),
                    threads=bps.bps_query(r.handle, 0, 6), lds=bps.bps_query(r.handle, 0, 7))
        return depth.cpu().numpy(), tid.cpu().numpy().view(np.uint32), info


def _compare(gd, gi, ref, tag=""):
    od, oi = ref["depth"], ref["tri_id"]
    bad_id = gi != oi
    assert not bad_id.any(), f"{tag}: {int(bad_id.sum())} pixels differ in coverage / triangle id, first at {np.argwhere(bad_id)[:5]}"
    # bar: 1e-5 relative; the arithmetic is the same IEEE sequence so exact equality is expected
    rel = np.abs(gd - od) <= 1e-5 * np.abs(od)
    assert rel.all(), f"{tag}: depth off at {np.argwhere(~rel)[:5]}"
    return int((gd != od).sum())


def _oracle(w):
    import oracle
    return oracle.render_batch(w.scenes, w.scene_ids, w.view_proj, w.H, w.W)


@pytest.mark.parametrize("splits,threads", [(1, 512), (0, 0), (3, 256), (2, 1024)])
def test_config1_room_matches_oracle(splits, threads):
    w = synth.build_config(1)
    ref = _oracle(w)
    gd, gi, info = _render_gpu(w.scenes, w.scene_ids, w.view_proj, w.H, w.W, splits=splits, threads=threads)
    print(info)
    nd = _compare(gd, gi, ref, f"config1 splits={splits} threads={threads}")
    assert nd == 0, f"{nd} depths differ in the last bits"
    assert (gi == NOHIT).sum() == 0          # closed room: no background


def test_config2_slice_matches_oracle():
    w = synth.build_config(2, B=24)
    ref = _oracle(w)
    for splits in (1, 5):
        gd, gi, info = _render_gpu(w.scenes, w.scene_ids, w.view_proj, w.H, w.W, splits=splits)
        _compare(gd, gi, ref, f"config2 splits={splits}")


def test_mixed_scenes_interleaved_ids():
    w = synth.build_config(3, B=16, scale=0.1)       # 4 scenes x ~50k triangles, ids b mod 4
    ref = _oracle(w)
    gd, gi, _ = _render_gpu(w.scenes, w.scene_ids, w.view_proj, w.H, w.W, device_matrices=True)
    _compare(gd, gi, ref, "mixed")


def test_cluster_culling_never_changes_a_frame():
    import paper_2103_07013_amd as bps
    w = synth.build_config(2, B=32)
    ref = _oracle(w)
    a = _render_gpu(w.scenes, w.scene_ids, w.view_proj, w.H, w.W)
    b = _render_gpu(w.scenes, w.scene_ids, w.view_proj, w.H, w.W, flags=bps.FLAG_NO_CLUSTER_CULL)
    c = _render_gpu(w.scenes, w.scene_ids, w.view_proj, w.H, w.W, flags=bps.FLAG_NO_OCCLUSION_CULL)
    d = _render_gpu(w.scenes, w.scene_ids, w.view_proj, w.H, w.W, splits=3)
    _compare(a[0], a[1], ref, "frustum + occlusion culling")
    _compare(b[0], b[1], ref, "culling off")
    _compare(c[0], c[1], ref, "frustum culling only")
    _compare(d[0], d[1], ref, "culling with split frames")
    # cameras with pitch and roll-free tilt, close to walls: bounds straddle every plane
    Ms = np.stack([synth.view_proj_from_pose((1.0 + 1.1 * k, 0.3 + 0.1 * k, 0.7 * k + 0.4), 0.8 * k, 0.3 * (k % 5 - 2))
                   for k in range(16)])
    import oracle
    s = w.scenes[0]
    ref2 = oracle.render_scene(s.vertices, s.indices, Ms, 64, 64)
    c = _render_gpu(w.scenes, [0] * 16, Ms, 64, 64)
    _compare(c[0], c[1], ref2, "tilted cameras")


@pytest.mark.parametrize("threads", [0, 256, 1024])
def test_random_soup_with_heavy_clipping(threads):
    """Most triangles straddle a frustum plane: the work-group's clip ring runs full at every group size
    (its capacity goes with the number of wavefronts)."""
    import oracle
    rng = np.random.default_rng(7)
    n = 3000
    c = np.stack([rng.uniform(-4, 4, n), rng.uniform(-4, 4, n), rng.uniform(-9, 2, n)], 1)
    v = (c[:, None, :] + rng.uniform(-1.5, 1.5, (n, 3, 3))).reshape(-1, 3).astype(np.float32)
    idx = np.arange(3 * n, dtype=np.uint32).reshape(n, 3)
    scene = synth.Scene(v, idx, np.zeros((3 * n, 3), np.uint8), np.zeros((3 * n, 2), np.float32),
                        np.zeros((4, 4, 3), np.uint8), (1, 1))
    Ms = np.stack([synth.view_proj_from_pose((0.1 * k, -0.2, 0.5), 0.4 * k, 0.15 * (k - 3), near=0.05, far=12.0)
                   for k in range(8)])
    for (H, W) in ((64, 64), (32, 96), (128, 128)):
        Ma = np.stack([synth.view_proj_from_pose((0.1 * k, -0.2, 0.5), 0.4 * k, 0.15 * (k - 3), near=0.05, far=12.0,
                                                 aspect=W / H) for k in range(8)])
        ref = oracle.render_scene(v, idx, Ma, H, W)
        gd, gi, info = _render_gpu([scene], [0] * 8, Ma, H, W, background=3.5, threads=threads, splits=1 if threads else 0)
        assert not threads or info["threads"] == threads
        ref["depth"][ref["tri_id"] == NOHIT] = 3.5
        _compare(gd, gi, ref, f"soup {H}x{W} threads {threads}")


def test_rgbd_small_scene_matches_oracle_colours():
    import torch
    import oracle
    import paper_2103_07013_amd as bps
    w = synth.build_config(4, B=16, scale=0.02)       # 8 scenes x ~20k triangles with colours
    ref = oracle.render_batch(w.scenes, w.scene_ids, w.view_proj, w.H, w.W, rgbd=True)
    with bps.Renderer(max_batch=w.B, height=w.H, width=w.W, mode=bps.MODE_RGBD) as r:
        hs = [r.load_scene(s.vertices, s.indices, s.colors) for s in w.scenes]
        ids = np.array([hs[k] for k in w.scene_ids], np.int32)
        depth, rgb, _ = r.render(ids, w.view_proj)       # no id buffer from the caller
        torch.cuda.synchronize()
        gd, grgb = depth.cpu().numpy(), rgb.cpu().numpy()
    assert np.all(np.abs(gd - ref["depth"]) <= 1e-5 * np.abs(ref["depth"]))
    assert np.array_equal(grgb, ref["rgb"])             # same IEEE sequence: exact


def test_rgbd_room_with_clipped_large_triangles():
    import torch
    import oracle
    import paper_2103_07013_amd as bps
    w = synth.build_config(1)                           # big triangles, many cross the frustum planes
    s = w.scenes[0]
    ref = oracle.render_scene(s.vertices, s.indices, w.view_proj, 64, 64, colors=s.colors)
    with bps.Renderer(max_batch=w.B, mode=bps.MODE_RGBD, splits=3) as r:
        h = r.load_scene(s.vertices, s.indices, s.colors)
        depth, rgb, tid = r.render(np.full(w.B, h, np.int32), w.view_proj, want_tri_id=True)
        torch.cuda.synchronize()
    assert np.array_equal(tid.cpu().numpy().view(np.uint32), ref["tri_id"])
    assert np.array_equal(rgb.cpu().numpy(), ref["rgb"])


@pytest.mark.parametrize("H,W", [(128, 128), (72, 96), (128, 64), (8, 8), (24, 120)])
def test_frames_cut_into_tiles_match_oracle(H, W):
    """Frames wider or taller than 64 pixels are rendered as several windows by separate
    work-groups; triangles crossing window borders and uneven windows must still be exact."""
    import oracle
    w = synth.build_config(1)                      # large triangles: most cross window borders
    s = w.scenes[0]
    Ms = np.stack([synth.view_proj_from_pose((1.0 + 0.5 * k, 1.25, 0.8 + 0.4 * k), 0.7 * k, 0.1 * (k % 3 - 1),
                                             aspect=W / H) for k in range(12)])
    ref = oracle.render_scene(s.vertices, s.indices, Ms, H, W)
    for splits in (1, 2):
        gd, gi, info = _render_gpu([s], [0] * 12, Ms, H, W, splits=splits)
        _compare(gd, gi, ref, f"{H}x{W} splits={splits}")
    w2 = synth.build_config(2, B=6)                # sub-pixel triangles
    ref2 = oracle.render_scene(w2.scenes[0].vertices, w2.scenes[0].indices, w2.view_proj, H, W)
    gd, gi, _ = _render_gpu(w2.scenes, [0] * 6, w2.view_proj, H, W)
    _compare(gd, gi, ref2, f"{H}x{W} dense")


@pytest.mark.parametrize("rgbd", [False, True])
def test_supersampled_output_is_the_box_filter_of_the_double_resolution_render(rgbd):
    """Render at 2H x 2W and average 2x2 blocks (the paper's 256 -> 128 downsampling, at the sizes
    this library supports).  Expected values: the oracle's double-resolution frames through the
    oracle's own box filter."""
    import torch
    import oracle
    import paper_2103_07013_amd as bps
    w = synth.build_config(4 if rgbd else 2, B=8, scale=0.05 if rgbd else 0.2)
    H = W = 48
    ref = oracle.render_batch(w.scenes, w.scene_ids, w.view_proj, 2 * H, 2 * W, rgbd=rgbd)
    expect, expect_rgb = oracle.downsample2(ref["depth"], ref["rgb"] if rgbd else None)
    with bps.Renderer(max_batch=w.B, height=H, width=W, supersample=2,
                      mode=bps.MODE_RGBD if rgbd else bps.MODE_DEPTH) as r:
        hs = [r.load_scene(s.vertices, s.indices, s.colors if rgbd else None) for s in w.scenes]
        ids = np.array([hs[k] for k in w.scene_ids], np.int32)
        depth, rgb, _ = r.render(ids, w.view_proj)
        torch.cuda.synchronize()
        assert tuple(depth.shape) == (w.B, H, W)
        assert np.array_equal(depth.cpu().numpy(), expect)
        if rgbd:
            assert np.array_equal(rgb.cpu().numpy(), expect_rgb)
        with pytest.raises(bps.BpsError):
            r.render(ids, w.view_proj, want_tri_id=True)


@pytest.mark.parametrize("bilinear", [False, True])
@pytest.mark.parametrize("cfg,B,scale,H,W", [(4, 16, 0.02, 64, 64), (1, 32, 1.0, 64, 64), (4, 6, 0.05, 96, 128)])
def test_textured_scenes_match_oracle_texels(cfg, B, scale, H, W, bilinear):
    """Texture coordinates interpolated (and clipped) like colours, one mip level per rasterised
    triangle, nearest texel or the bilinear blend of four: the same float sequence as the oracle,
    so every byte is equal."""
    import torch
    import oracle
    import paper_2103_07013_amd as bps
    w = synth.build_config(cfg, B=B, scale=scale)
    ref = oracle.render_batch(w.scenes, w.scene_ids, w.view_proj, H, W, rgbd=True, textured=True, bilinear=bilinear)
    with bps.Renderer(max_batch=w.B, height=H, width=W, mode=bps.MODE_RGBD,
                      flags=bps.FLAG_BILINEAR if bilinear else 0) as r:
        hs = [r.load_scene_textured(s.vertices, s.indices, s.uvs, s.texture) for s in w.scenes]
        ids = np.array([hs[k] for k in w.scene_ids], np.int32)
        depth, rgb, tid = r.render(ids, w.view_proj, want_tri_id=True)
        torch.cuda.synchronize()
    assert np.array_equal(tid.cpu().numpy().view(np.uint32), ref["tri_id"])
    grgb = rgb.cpu().numpy()
    assert np.array_equal(grgb, ref["rgb"])
    hit = ref["tri_id"] != NOHIT
    assert len(np.unique(grgb[hit].reshape(-1, 3), axis=0)) > 50      # really texels, not flat colours


def test_textured_and_coloured_scenes_mix_in_one_batch_and_odd_textures_work():
    """One batch may reference textured and vertex-coloured scenes; a 1x1 and a 4x64 texture are
    legal (all levels clamp at 1 texel per side); uv far outside [0,1) wraps."""
    import torch
    import oracle
    import paper_2103_07013_amd as bps
    w = synth.build_config(1, B=12)
    s = w.scenes[0]
    rng = np.random.default_rng(5)
    texA = rng.integers(0, 256, size=(64, 4, 3)).astype(np.uint8)
    texB = np.array([[[9, 200, 31]]], np.uint8)
    uvA = (s.uvs * 7.5 - 40.0).astype(np.float32)
    refA = oracle.render_scene(s.vertices, s.indices, w.view_proj[:4], 64, 64, uvs=uvA, texture=texA)
    refB = oracle.render_scene(s.vertices, s.indices, w.view_proj[4:8], 64, 64, uvs=s.uvs, texture=texB)
    refC = oracle.render_scene(s.vertices, s.indices, w.view_proj[8:], 64, 64, colors=s.colors)
    with bps.Renderer(max_batch=12, mode=bps.MODE_RGBD) as r:
        a = r.load_scene_textured(s.vertices, s.indices, uvA, texA)
        b = r.load_scene_textured(s.vertices, s.indices, s.uvs, texB)
        c = r.load_scene(s.vertices, s.indices, s.colors)
        ids = np.array([a] * 4 + [b] * 4 + [c] * 4, np.int32)
        depth, rgb, _ = r.render(ids, w.view_proj)
        torch.cuda.synchronize()
        with pytest.raises(bps.BpsError):
            r.load_scene_textured(s.vertices, s.indices, s.uvs, np.zeros((48, 64, 3), np.uint8))   # 48: not 2^k
    g = rgb.cpu().numpy()
    assert np.array_equal(g[:4], refA["rgb"])
    assert np.array_equal(g[4:8], refB["rgb"])
    assert np.array_equal(g[8:], refC["rgb"])


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_scenes_cameras_and_frame_sizes(seed):
    """Randomised sweep: triangle soups with sizes from sub-pixel to frame-filling, cameras with
    roll, pitch, narrow to very wide fields of view and near planes that cut the geometry, odd
    frame sizes; every frame must equal the oracle's."""
    import oracle
    rng = np.random.default_rng(seed)
    n = 2500
    centre = np.stack([rng.uniform(-5, 5, n), rng.uniform(-3, 3, n), rng.uniform(-5, 5, n)], 1)
    size = np.exp(rng.uniform(np.log(0.01), np.log(3.0), n))[:, None, None]          # 1 cm .. 3 m
    v = (centre[:, None, :] + rng.uniform(-1, 1, (n, 3, 3)) * size).reshape(-1, 3).astype(np.float32)
    # share some vertices between triangles, and repeat a few triangles exactly (depth ties -> lowest id)
    idx = np.arange(3 * n, dtype=np.uint32).reshape(n, 3)
    idx[100:200] = idx[0:100]
    idx[300:400, 0] = idx[299:399, 1]
    scene = synth.Scene(v, idx, np.zeros((3 * n, 3), np.uint8), np.zeros((3 * n, 2), np.float32),
                        np.zeros((4, 4, 3), np.uint8), (1, 1))
    H, W = [(64, 64), (40, 72), (128, 96), (16, 128)][seed % 4]
    Ms = []
    for k in range(12):
        pos = rng.uniform(-4, 4, 3)
        yaw, pitch, roll = rng.uniform(0, 2 * np.pi), rng.uniform(-1.2, 1.2), rng.uniform(-np.pi, np.pi)
        hfov = rng.choice([25.0, 60.0, 90.0, 140.0, 170.0])
        near = float(rng.choice([0.01, 0.3, 2.0]))
        P = synth.perspective(hfov, W / H, near, near + float(rng.choice([5.0, 30.0])))
        V = synth.look_yaw(pos, yaw, pitch)
        c, s = np.cos(roll), np.sin(roll)
        R = np.eye(4)
        R[0, 0], R[0, 1], R[1, 0], R[1, 1] = c, -s, s, c
        Ms.append((P @ R @ V).astype(np.float32))
    Ms = np.stack(Ms)
    ref = oracle.render_scene(v, idx, Ms, H, W)
    for splits in (0, 1):
        gd, gi, _ = _render_gpu([scene], [0] * 12, Ms, H, W, splits=splits)
        _compare(gd, gi, ref, f"seed {seed} {H}x{W} splits={splits}")
    assert (ref["tri_id"] != NOHIT).mean() > 0.2


@pytest.mark.parametrize("bilinear", [False, True])
def test_random_soup_rgbd_and_texture_through_the_clipper(bilinear):
    """Colour and texture coordinates of triangles cut by every frustum plane (wide field of view,
    near plane inside the geometry, rolled cameras; texture coordinates far outside [0, 1), so
    the bilinear blend wraps around the texture's sides all the time): bytes equal the oracle's."""
    import torch
    import oracle
    import paper_2103_07013_amd as bps
    rng = np.random.default_rng(21)
    n = 1500
    centre = np.stack([rng.uniform(-4, 4, n), rng.uniform(-2, 2, n), rng.uniform(-4, 4, n)], 1)
    size = np.exp(rng.uniform(np.log(0.05), np.log(4.0), n))[:, None, None]
    v = (centre[:, None, :] + rng.uniform(-1, 1, (n, 3, 3)) * size).reshape(-1, 3).astype(np.float32)
    idx = np.arange(3 * n, dtype=np.uint32).reshape(n, 3)
    colors = rng.integers(0, 256, size=(3 * n, 3)).astype(np.uint8)
    uvs = rng.uniform(-3, 3, size=(3 * n, 2)).astype(np.float32)
    tex = rng.integers(0, 256, size=(32, 64, 3)).astype(np.uint8)
    Ms = []
    for k in range(10):
        P = synth.perspective(float(rng.choice([60.0, 120.0, 165.0])), 1.0, float(rng.choice([0.05, 1.0])), 25.0)
        V = synth.look_yaw(rng.uniform(-3, 3, 3), rng.uniform(0, 6.28), rng.uniform(-1, 1))
        c, s = np.cos(0.6 * k), np.sin(0.6 * k)
        R = np.eye(4)
        R[0, 0], R[0, 1], R[1, 0], R[1, 1] = c, -s, s, c
        Ms.append((P @ R @ V).astype(np.float32))
    Ms = np.stack(Ms)
    ref_c = oracle.render_scene(v, idx, Ms, 64, 64, colors=colors)
    ref_t = oracle.render_scene(v, idx, Ms, 64, 64, uvs=uvs, texture=tex, bilinear=bilinear)
    with bps.Renderer(max_batch=20, mode=bps.MODE_RGBD, flags=bps.FLAG_BILINEAR if bilinear else 0) as r:
        a = r.load_scene(v, idx, colors)
        b = r.load_scene_textured(v, idx, uvs, tex)
        ids = np.array([a] * 10 + [b] * 10, np.int32)
        depth, rgb, tid = r.render(ids, np.concatenate([Ms, Ms]), want_tri_id=True)
        torch.cuda.synchronize()
    g, gi = rgb.cpu().numpy(), tid.cpu().numpy().view(np.uint32)
    assert np.array_equal(gi[:10], ref_c["tri_id"]) and np.array_equal(gi[10:], ref_t["tri_id"])
    assert np.array_equal(g[:10], ref_c["rgb"])
    assert np.array_equal(g[10:], ref_t["rgb"])


@pytest.mark.parametrize("seed,H,W", [(31, 64, 64), (32, 128, 128), (33, 48, 104)])
def test_connected_scene_under_arbitrary_cameras(seed, H, W):
    """A connected mesh (clusters grown over shared vertices, occlusion between rooms) seen by cameras
    anywhere in it, also inside objects and walls, with pitch, roll, narrow to very wide fields of view
    and near planes that cut the geometry; culling on and off must both equal the oracle."""
    import oracle
    import paper_2103_07013_amd as bps
    rng = np.random.default_rng(seed)
    scene = synth.make_multiroom_scene(40_000, seed=1400 + seed)
    lo, hi = scene.vertices.min(0), scene.vertices.max(0)
    Ms = []
    for k in range(16):
        pos = rng.uniform(lo, hi)
        yaw, pitch, roll = rng.uniform(0, 2 * np.pi), rng.uniform(-1.4, 1.4), rng.uniform(-np.pi, np.pi)
        hfov = float(rng.choice([20.0, 60.0, 90.0, 150.0, 175.0]))
        near = float(rng.choice([0.01, 0.5, 3.0]))
        P = synth.perspective(hfov, W / H, near, near + float(rng.choice([4.0, 20.0, 100.0])))
        V = synth.look_yaw(pos, yaw, pitch)
        c, s = np.cos(roll), np.sin(roll)
        R = np.eye(4)
        R[0, 0], R[0, 1], R[1, 0], R[1, 1] = c, -s, s, c
        Ms.append((P @ R @ V).astype(np.float32))
    Ms = np.stack(Ms)
    ref = oracle.render_scene(scene.vertices, scene.indices, Ms, H, W)
    for flags in (0, bps.FLAG_NO_OCCLUSION_CULL, bps.FLAG_NO_CLUSTER_CULL):
        gd, gi, _ = _render_gpu([scene], [0] * 16, Ms, H, W, flags=flags)
        _compare(gd, gi, ref, f"seed {seed} {H}x{W} flags={flags}")
    assert (ref["tri_id"] != NOHIT).mean() > 0.3


def test_scene_with_more_blocks_than_the_visiting_order_holds():
    """A 6.3 M-triangle scene has 1032 blocks of 64 clusters, more than a work-group can rank near to
    far (1024): with one work-group per environment the blocks are then visited in storage order and
    none may be skipped; split over several work-groups each share is small enough to be ranked."""
    import oracle
    scene = synth.make_multiroom_scene(6_300_000, seed=1700)
    cams = synth.make_cameras(scene, 4, seed=9)[0]
    ref = oracle.render_scene(scene.vertices, scene.indices, cams, 64, 64)
    for splits in (1, 0):
        gd, gi, info = _render_gpu([scene], [0] * 4, cams, 64, 64, splits=splits)
        if splits == 1:
            assert info["groups"] == 4
        _compare(gd, gi, ref, f"splits={splits}")
