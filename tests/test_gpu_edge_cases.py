"""GPU edge cases and invariants of the C-ABI renderer (all inputs small and seeded)."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu
NOHIT = 0xFFFFFFFF


@pytest.fixture(scope="module")
def room():
    return synth.build_config(1)


def _frames(r, ids, vp, **kw):
    import torch
    d, rgb, t = r.render(np.asarray(ids, np.int32), vp, want_tri_id=True, **kw)
    torch.cuda.synchronize()
    return d.cpu().numpy(), t.cpu().numpy().view(np.uint32)


def test_error_paths_return_statuses(room):
    import torch
    import paper_2103_07013_amd as bps
    s = room.scenes[0]
    with bps.Renderer(max_batch=4) as r:
        h = r.load_scene(s.vertices, s.indices)
        out = torch.empty((8, 64, 64), dtype=torch.float32, device="cuda")
        with pytest.raises(bps.BpsError) as e:           # B > max_batch
            bps.bps_render(r.handle, np.zeros(8, np.int32), room.view_proj[:8], out)
        assert e.value.status == -1
        with pytest.raises(bps.BpsError) as e:           # unknown scene
            bps.bps_render(r.handle, np.array([h + 5], np.int32), room.view_proj[:1], out[:1])
        assert e.value.status == -2
        with pytest.raises(bps.BpsError) as e:           # index out of range at load
            r.load_scene(s.vertices[:10], s.indices)
        assert e.value.status == -1
        bad = s.vertices.copy()
        bad[3, 1] = np.inf
        with pytest.raises(bps.BpsError):                # non-finite vertex at load
            r.load_scene(bad, s.indices)
        r.unload_scene(h)
        with pytest.raises(bps.BpsError) as e:           # stale handle
            bps.bps_render(r.handle, np.array([h], np.int32), room.view_proj[:1], out[:1])
        assert e.value.status == -2
        with pytest.raises(bps.BpsError):
            r.unload_scene(h)
        # empty batch is a no-op
        bps.bps_render(r.handle, np.zeros(0, np.int32), room.view_proj[:0], out[:0])
        h2 = r.load_scene(s.vertices, s.indices)         # loading after an unload works (slot may be reused)
        assert h2 >= 0
    with bps.Renderer(max_batch=2, mode=bps.MODE_RGBD) as r:
        h = r.load_scene(s.vertices, s.indices)          # no colours
        rgb = torch.empty((1, 64, 64, 3), dtype=torch.uint8, device="cuda")
        with pytest.raises(bps.BpsError) as e:
            bps.bps_render(r.handle, np.array([h], np.int32), room.view_proj[:1], out[:1], out_rgb=rgb)
        assert e.value.status == -1


def test_batch_independence_two_handles_and_determinism(room):
    import paper_2103_07013_amd as bps
    s = room.scenes[0]
    with bps.Renderer(max_batch=16) as r:
        h1 = r.load_scene(s.vertices, s.indices)
        h2 = r.load_scene(s.vertices, s.indices)
        d_all, t_all = _frames(r, [h1] * 16, room.view_proj)
        for b in (0, 7, 15):                             # an environment alone == its slot in the batch
            d1, t1 = _frames(r, [h1], room.view_proj[b:b + 1])
            assert np.array_equal(d1[0], d_all[b]) and np.array_equal(t1[0], t_all[b])
        d2, t2 = _frames(r, [h2] * 16, room.view_proj)   # same mesh under another handle
        assert np.array_equal(d2, d_all) and np.array_equal(t2, t_all)
        dm, tm = _frames(r, [h1, h2] * 8, room.view_proj)
        assert np.array_equal(dm, d_all) and np.array_equal(tm, t_all)
        for _ in range(5):                               # run-to-run determinism
            d3, t3 = _frames(r, [h1] * 16, room.view_proj)
            assert np.array_equal(d3, d_all) and np.array_equal(t3, t_all)


def test_split_and_unsplit_frames_agree_and_buffer_is_left_clean(room):
    import paper_2103_07013_amd as bps
    s = room.scenes[0]
    with bps.Renderer(max_batch=16, splits=1) as r1, bps.Renderer(max_batch=16, splits=4) as r4:
        a = r1.load_scene(s.vertices, s.indices)
        b = r4.load_scene(s.vertices, s.indices)
        d1, t1 = _frames(r1, [a] * 16, room.view_proj)
        for rep in range(3):                             # the merge buffer must come back empty every time
            d4, t4 = _frames(r4, [b] * 16, room.view_proj)
            assert np.array_equal(d1, d4) and np.array_equal(t1, t4), rep
        # a smaller, different request after a larger one
        d4, t4 = _frames(r4, [b] * 3, room.view_proj[5:8])
        assert np.array_equal(d1[5:8], d4) and np.array_equal(t1[5:8], t4)


def test_non_finite_and_degenerate_matrices_give_background(room):
    import paper_2103_07013_amd as bps
    s = room.scenes[0]
    vp = room.view_proj[:4].copy()
    vp[0, 1, 2] = np.nan
    vp[1] = 0.0
    vp[2, 3, :] = np.inf
    with bps.Renderer(max_batch=4, background_depth=-1.0) as r:
        h = r.load_scene(s.vertices, s.indices)
        d, t = _frames(r, [h] * 4, vp)
    for b in (0, 1, 2):
        assert np.all(t[b] == NOHIT) and np.all(d[b] == -1.0)
    assert (t[3] != NOHIT).all()


def test_tiny_meshes_and_hand_enumerated_fill_rule():
    """One triangle, fewer triangles than lanes, and the 8x8 hand-enumerated fixtures through the GPU."""
    import os
    import paper_2103_07013_amd as bps
    here = os.path.dirname(os.path.abspath(__file__))
    M = np.array([[0.25, 0, 0, -1], [0, 0.25, 0, -1], [0, 0, 0, 0.5], [0, 0, 0, 1]], np.float32)  # pixel k at x in [k, k+1)
    for name in ("fill_rule_upper_left.txt", "fill_rule_lower_right.txt", "fill_rule_centre_corners.txt"):
        tris, rows = [], []
        for line in open(os.path.join(here, "golden", name)):
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("tri"):
                tris.append([int(x) for x in line.split()[1:]])
            else:
                rows.append([int(ch) for ch in line])
        xy = np.array(tris, np.float64).reshape(-1, 3, 2) / 256.0
        v = np.concatenate([xy, np.zeros((xy.shape[0], 3, 1))], 2).reshape(-1, 3).astype(np.float32)
        idx = np.arange(v.shape[0], dtype=np.uint32).reshape(-1, 3)
        with bps.Renderer(max_batch=1, height=8, width=8) as r:
            h = r.load_scene(v, idx)
            d, t = _frames(r, [h], M[None])
        assert np.array_equal((t[0] != NOHIT).astype(np.uint32), np.array(rows, np.uint32)), name
        assert np.all(d[0][t[0] != NOHIT] == 1.0)


def test_device_and_host_matrices_and_explicit_stream(room):
    import torch
    import paper_2103_07013_amd as bps
    s = room.scenes[0]
    with bps.Renderer(max_batch=16) as r:
        h = r.load_scene(s.vertices, s.indices)
        d0, t0 = _frames(r, [h] * 16, room.view_proj)
        side = torch.cuda.Stream()
        vp = torch.from_numpy(room.view_proj).cuda()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            d1, t1 = _frames(r, [h] * 16, vp, stream=side)
        assert np.array_equal(d0, d1) and np.array_equal(t0, t1)


def test_asynchronous_scene_rotation_while_rendering():
    """Scenes are loaded on a side stream and retired while requests that use them are queued;
    every frame must still match the oracle and device blocks must be recycled."""
    import torch
    import oracle
    import paper_2103_07013_amd as bps
    scenes = [synth.make_multiroom_scene(30_000, seed=1100 + k) for k in range(6)]
    cams = [synth.make_cameras(sc, 8, seed=77 + k)[0] for k, sc in enumerate(scenes)]
    refs = [oracle.render_scene(sc.vertices, sc.indices, cams[k], 64, 64) for k, sc in enumerate(scenes)]
    copy_stream = torch.cuda.Stream()
    with bps.Renderer(max_batch=16) as r:
        live = {0: r.load_scene(scenes[0].vertices, scenes[0].indices),
                1: r.load_scene(scenes[1].vertices, scenes[1].indices)}
        outs = []
        for step in range(12):
            a, b = sorted(live)[-2:]
            ids = np.array([live[a]] * 8 + [live[b]] * 8, np.int32)
            vp = np.concatenate([cams[a], cams[b]])
            depth, _, tid = r.render(ids, vp, want_tri_id=True)          # not synchronised
            outs.append((a, b, depth, tid))
            if step % 2 == 1 and step // 2 + 2 < len(scenes) + 3:
                nxt = (max(live) + 1) % len(scenes)
                if nxt not in live:
                    old = min(live)
                    r.unload_scene(live.pop(old))                          # still referenced by queued work
                    live[nxt] = r.load_scene_async(scenes[nxt].vertices, scenes[nxt].indices, copy_stream=copy_stream)
        torch.cuda.synchronize()
        for (a, b, depth, tid) in outs:
            d, t = depth.cpu().numpy(), tid.cpu().numpy().view(np.uint32)
            assert np.array_equal(t[:8], refs[a]["tri_id"]) and np.array_equal(t[8:], refs[b]["tri_id"])
            assert np.array_equal(d[:8], refs[a]["depth"]) and np.array_equal(d[8:], refs[b]["depth"])
        assert all(bps.bps_scene_ready(r.handle, h) for h in live.values())
        assert bps.bps_query(r.handle, 0, 8) <= 4          # blocks were reused, not allocated per load


def test_loader_thread_rotates_scenes_beside_the_render_thread():
    """The paper's asynchronous asset loading with real threads: a loader thread keeps replacing the
    resident scenes (asynchronous upload on its own stream, retirement of the scene it replaces) while
    the main thread issues render requests without ever synchronising.  Every frame of every request
    is checked against the oracle for the scenes that request named."""
    import threading
    import torch
    import oracle
    import paper_2103_07013_amd as bps
    meshes = [synth.make_multiroom_scene(20_000, seed=1200 + k) for k in range(7)]
    cams = [synth.make_cameras(m, 8, seed=91 + k)[0] for k, m in enumerate(meshes)]
    refs = [oracle.render_scene(m.vertices, m.indices, cams[k], 64, 64) for k, m in enumerate(meshes)]
    K, want_sets, max_requests = 3, 5, 6000
    ref_d = torch.from_numpy(np.stack([x["depth"] for x in refs])).cuda()                      # [mesh, 8, H, W]
    ref_t = torch.from_numpy(np.stack([x["tri_id"] for x in refs]).view(np.int32)).cuda()
    copy_stream = torch.cuda.Stream()
    with bps.Renderer(max_batch=8 * K) as r:
        lock = threading.Lock()
        state = {"mesh": [0, 1, 2], "stop": False, "swaps": 0, "error": None}
        state["handle"] = [r.load_scene(meshes[k].vertices, meshes[k].indices) for k in state["mesh"]]

        def loader():
            try:
                n = 0
                while not state["stop"]:
                    slot, mesh = n % K, (n + K) % len(meshes)
                    n += 1
                    if mesh in state["mesh"]:
                        continue
                    new = bps.bps_load_scene_async(r.handle, meshes[mesh].vertices, meshes[mesh].indices, None, copy_stream)
                    with lock:      # the render thread names scenes and submits under the same lock
                        old = state["handle"][slot]
                        state["handle"][slot], state["mesh"][slot] = new, mesh
                        bps.bps_unload_scene(r.handle, old)      # requests that use it may still be queued
                    state["swaps"] += 1
            except Exception as e:      # surfaces in the main thread's assert
                state["error"] = e

        th = threading.Thread(target=loader)
        th.start()
        # expected frames per set of resident meshes, put together on the device (no host round trip per
        # request: the render thread never waits for the GPU while the loader runs)
        expected = {}
        wrong = torch.zeros((), dtype=torch.int64, device="cuda")
        depth = [torch.empty((8 * K, 64, 64), dtype=torch.float32, device="cuda") for _ in range(2)]
        tid = [torch.empty((8 * K, 64, 64), dtype=torch.int32, device="cuda") for _ in range(2)]
        issued, sets_seen = 0, set()
        try:
            while len(sets_seen) < want_sets and issued < max_requests and state["error"] is None:
                with lock:
                    used = tuple(state["mesh"])
                    ids = np.repeat(np.array(state["handle"], np.int32), 8)
                    vp = np.concatenate([cams[m] for m in used])
                    bps.bps_render(r.handle, ids, vp, depth[issued & 1], out_tri_id=tid[issued & 1])   # not synchronised
                if used not in expected:
                    expected[used] = (torch.cat([ref_d[m] for m in used]), torch.cat([ref_t[m] for m in used]))
                wrong += (depth[issued & 1] != expected[used][0]).sum() + (tid[issued & 1] != expected[used][1]).sum()
                sets_seen.add(used)
                issued += 1
        finally:
            state["stop"] = True
            th.join()
        torch.cuda.synchronize()
        assert state["error"] is None, state["error"]
        assert len(sets_seen) >= want_sets, "the requests did not get to see scenes being replaced"
        assert state["swaps"] >= want_sets - 1 and issued >= want_sets
        assert int(wrong.item()) == 0, f"{int(wrong.item())} pixels of {issued} requests differ from the oracle"


@pytest.mark.parametrize("rgbd", [False, True])
def test_requests_in_flight_on_two_streams(rgbd):
    """Consecutive requests on two alternating streams may overlap on the device.  Every frame must
    still match the oracle, also where requests share the renderer's own buffers (RGB-D) and where a
    scene is retired while requests on both streams still read it."""
    import torch
    import oracle
    import paper_2103_07013_amd as bps
    scenes = [synth.make_multiroom_scene(40_000, seed=1300 + k) for k in range(3)]
    cams = [synth.make_cameras(sc, 24, seed=5 + k)[0] for k, sc in enumerate(scenes)]
    refs = [oracle.render_scene(sc.vertices, sc.indices, cams[k], 64, 64, colors=sc.colors if rgbd else None)
            for k, sc in enumerate(scenes)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    mode = bps.MODE_RGBD if rgbd else bps.MODE_DEPTH
    with bps.Renderer(max_batch=24, mode=mode) as r:
        handles = [r.load_scene(sc.vertices, sc.indices, sc.colors if rgbd else None) for sc in scenes[:2]]
        live = [0, 1]
        outs = []
        for step in range(10):
            k = live[step % 2]
            n = 24 - (step % 3) * 5                       # batch sizes 24, 19, 14
            depth = torch.empty((n, 64, 64), dtype=torch.float32, device="cuda")
            rgb = torch.empty((n, 64, 64, 3), dtype=torch.uint8, device="cuda") if rgbd else None
            ids = np.full(n, handles[live.index(k)], np.int32)
            bps.bps_render(r.handle, ids, cams[k][:n], depth, out_rgb=rgb, stream=streams[step % 2])
            outs.append((k, n, depth, rgb))
            if step == 5:                                 # scene 0 leaves while both streams are busy
                r.unload_scene(handles[0])
                handles[0] = r.load_scene(scenes[2].vertices, scenes[2].indices, scenes[2].colors if rgbd else None)
                live[0] = 2
        torch.cuda.synchronize()
        for step, (k, n, depth, rgb) in enumerate(outs):
            assert np.array_equal(depth.cpu().numpy(), refs[k]["depth"][:n]), f"request {step}"
            if rgbd:
                assert np.array_equal(rgb.cpu().numpy(), refs[k]["rgb"][:n]), f"request {step}"


@pytest.mark.parametrize("device_matrices", [False, True])
def test_requests_planned_on_the_renderers_own_stream(device_matrices):
    """Requests whose inputs are complete at the call (host matrices always; device matrices with
    FLAG_INPUTS_READY) are staged and planned on a stream of the renderer while earlier requests are
    still being drawn.  Batches large enough for launch planning, different cameras and batch sizes
    back to back, a scene uploaded asynchronously in between: every frame must match the oracle."""
    import torch
    import oracle
    import paper_2103_07013_amd as bps
    scenes = [synth.make_multiroom_scene(30_000, seed=1800 + k) for k in range(2)]
    B = 640                                                  # more work-groups than the device holds at once
    cams = [synth.make_cameras(sc, B, seed=31 + k)[0] for k, sc in enumerate(scenes)]
    refs = [oracle.render_scene(sc.vertices, sc.indices, cams[k], 64, 64) for k, sc in enumerate(scenes)]
    copy_stream = torch.cuda.Stream()
    with bps.Renderer(max_batch=B, flags=bps.FLAG_INPUTS_READY if device_matrices else 0) as r:
        h0 = r.load_scene(scenes[0].vertices, scenes[0].indices)
        h1 = None
        outs = []
        mats = [torch.from_numpy(c).cuda() if device_matrices else c for c in cams]
        torch.cuda.synchronize()                             # the device matrices are complete from here on
        for step in range(8):
            if step == 3:
                h1 = r.load_scene_async(scenes[1].vertices, scenes[1].indices, copy_stream=copy_stream)
            k = 1 if (h1 is not None and step % 2 == 1) else 0
            n = B - 37 * (step % 3)
            depth = torch.empty((n, 64, 64), dtype=torch.float32, device="cuda")
            bps.bps_render(r.handle, np.full(n, h1 if k else h0, np.int32), mats[k][:n], depth)
            outs.append((k, n, depth))
        torch.cuda.synchronize()
        for step, (k, n, depth) in enumerate(outs):
            assert np.array_equal(depth.cpu().numpy(), refs[k]["depth"][:n]), f"request {step}"


def test_stale_scene_handles_are_refused_after_their_slot_is_reused(room):
    """A handle names one load.  After bps_unload_scene it is refused, also once a later scene has taken
    its table slot (the new scene gets a different handle), and retiring a scene whose asynchronous
    upload has only just been enqueued does not wait and does not break later loads."""
    import torch
    import paper_2103_07013_amd as bps
    w = room
    s = w.scenes[0]
    small = synth.make_room_scene(2_000, seed=5)
    copy_stream = torch.cuda.Stream()
    with bps.Renderer(max_batch=4) as r:
        first = r.load_scene(s.vertices, s.indices)
        r.unload_scene(first)
        torch.cuda.synchronize()
        second = r.load_scene(small.vertices, small.indices)          # takes the free slot
        assert second != first
        for stale_call in (lambda: r.render(np.full(4, first, np.int32), w.view_proj[:4]),
                           lambda: bps.bps_unload_scene(r.handle, first),
                           lambda: bps.bps_scene_ready(r.handle, first),
                           lambda: bps.bps_query(r.handle, first, 1)):
            with pytest.raises(bps.BpsError) as e:
                stale_call()
            assert e.value.status == -2
        assert bps.bps_query(r.handle, second, 1) == small.T
        # retire a scene right after enqueuing its upload, then keep loading and rendering
        for k in range(4):
            h = bps.bps_load_scene_async(r.handle, s.vertices, s.indices, None, copy_stream)
            bps.bps_unload_scene(r.handle, h)
        h = bps.bps_load_scene_async(r.handle, s.vertices, s.indices, None, copy_stream)
        depth, _, tid = r.render(np.full(4, h, np.int32), w.view_proj[:4], want_tri_id=True)
        torch.cuda.synchronize()
        import oracle
        ref = oracle.render_scene(s.vertices, s.indices, w.view_proj[:4], 64, 64)
        assert np.array_equal(tid.cpu().numpy().view(np.uint32), ref["tri_id"])
        assert np.array_equal(depth.cpu().numpy(), ref["depth"])
