#!/usr/bin/env python3
"""Benchmark of the batch renderer hot path on one MI355X.

A step is one complete render request (request staging, dispatch planning, the fused raster
kernel, plus the resolve kernel when frames are split) for the headline workload: 4 procedural
multi-room scenes of ~500k triangles, 1024 environments (256 per scene, interleaved), 64x64
float32 depth.  Scenes and view-projection matrices are resident in HBM before the timed region.
Prints ONE JSON line.

How the headline is timed: the K steps cycle through four seeded sets of camera poses (the
workload's own and three more for the same scenes), the fourth with the environments' scene ids
permuted, so that consecutive requests differ and the work items are re-staged now and then.
Nothing but the requests is enqueued inside the timed region (no events); the region is bracketed
by synchronisations and `value` is B K / wall time.  Two separate short passes follow: one with a
HIP event per request (median and minimum time of a whole request), one with the library's events
around the raster kernel alone (kernel time for the roofline).

Two roofline objects are reported, both against the published HBM peak:
  roofline              the timed configuration (cluster culling on).  Algorithmic bytes are
                        recomputed for culling: bounds of every block / cluster that was tested plus
                        the mesh bytes of the clusters that reached the triangle phase, plus output.
  roofline_full_stream  the same request with culling off (every environment streams its whole
                        scene): 12 B per triangle + 12 B per vertex per environment, plus output.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
VALU_ISSUE_PEAK = 256 * 4 * 2.4e9 / 4      # wave64 vector instructions per second: 256 CUs x 4 SIMDs, 4 cycles each


def full_stream_bytes(w):
    """Every environment streams its scene's index and vertex arrays once (12 B per triangle +
    12 B per vertex), the frames are written once (4 B per pixel, +3 B with colour), and the
    request (scene id + matrix, 68 B) is read once."""
    geo = sum(12 * w.scenes[s].T + 12 * w.scenes[s].V for s in w.scene_ids)
    out = w.B * w.H * w.W * (7 if w.rgbd else 4)
    return geo + out + w.B * 68


def cpu_baseline(w, n_envs, textured=False):
    """Time the CPU oracle, as it stands, on a strided sample of the same workload."""
    import oracle
    stride = max(1, w.B // n_envs)
    sel = np.arange(0, w.B, stride)[:n_envs]
    t0 = time.perf_counter()
    r = oracle.render_batch(w.scenes, w.scene_ids[sel], w.view_proj[sel], w.H, w.W, rgbd=w.rgbd,
                            textured=textured and w.rgbd)
    dt = time.perf_counter() - t0
    return dict(value=len(sel) / dt, unit="frames/s", cores=int(r["threads"]), kind="oracle",
                sample=f"{len(sel)} of {w.B} environments (stride {stride}), same scenes and matrices, {dt:.2f} s wall")


def measured_traffic(key):
    """HBM bytes per launch from the rocprofv3 --pmc runs recorded under profiles/ (None if absent)."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as fh:
            return json.load(fh).get(key)
    except (OSError, ValueError):
        return None


def pose_cycle(torch, w, n_sets=4):
    """n_sets requests for one workload: (scene ids, device matrices).  Set 0 is the workload's own
    poses; the others are further seeded poses for the same scenes; the last one also permutes which
    environment uses which scene (same multiset of scenes, other order)."""
    import synth
    out = []
    for p in range(n_sets):
        vp = w.view_proj if p == 0 else synth.more_poses(w, p)
        ids = w.scene_ids
        if p == n_sets - 1 and n_sets > 1:
            perm = np.random.default_rng(7000 + w.number).permutation(w.B)
            ids, vp = w.scene_ids[perm], np.ascontiguousarray(vp[perm])
        out.append((ids, torch.from_numpy(np.ascontiguousarray(vp)).cuda()))
    return out


def timed_run(bps, torch, w, flags, steps, warmup, splits, threads, diagnostics=False, textured=False, n_sets=4,
              kernel_pass=24, request_pass=40):
    mode = bps.MODE_RGBD if w.rgbd else bps.MODE_DEPTH
    r = bps.Renderer(max_batch=w.B, height=w.H, width=w.W, mode=mode, splits=splits, threads=threads, flags=flags)
    if textured and w.rgbd:
        handles = [r.load_scene_textured(s.vertices, s.indices, s.uvs, s.texture) for s in w.scenes]
    else:
        handles = [r.load_scene(s.vertices, s.indices, s.colors if w.rgbd else None) for s in w.scenes]
    hmap = np.array(handles, np.int32)
    cycle = [(hmap[ids], vp) for ids, vp in pose_cycle(torch, w, n_sets)]
    depth = torch.empty((w.B, w.H, w.W), dtype=torch.float32, device="cuda")
    rgb = torch.empty((w.B, w.H, w.W, 3), dtype=torch.uint8, device="cuda") if w.rgbd else None
    stream = torch.cuda.current_stream()

    def submit(k):
        ids, vp = cycle[k % len(cycle)]
        bps.bps_render(r.handle, ids, vp, depth, out_rgb=rgb, stream=stream)

    # Before the W warm-up requests the device is brought out of idle: requests are issued for about
    # 50 ms, so that first-use allocations (the four staging slots, the planning stream) and the ramp of
    # the device's clocks lie outside the measurement whatever W is (a run with W = 5 came out 1.5 %
    # slower than one with W = 200 without this).
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < 0.05:
        for k in range(len(cycle)):
            submit(k)
        torch.cuda.synchronize()
    for k in range(max(warmup, len(cycle))):
        submit(k)
    # ---- the headline: K requests, nothing else enqueued, bracketed by synchronisations
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        submit(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # ---- whole requests one by one: an event after every request (these cost a few microseconds each,
    # which is why they are kept out of the headline)
    n = request_pass
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    ev[0].record(stream)
    for k in range(n):
        submit(k)
        ev[k + 1].record(stream)
    torch.cuda.synchronize()
    req_ms = np.array([ev[k].elapsed_time(ev[k + 1]) for k in range(n)])
    # ---- the raster kernel alone (library events around its launch)
    bps.bps_set_profiling(r.handle, 1)
    for k in range(kernel_pass):
        submit(k)
    torch.cuda.synchronize()
    each = bps.bps_kernel_ms_each(r.handle)
    bps.bps_set_profiling(r.handle, False)
    launches = len(each)
    res = dict(dt=dt, kernel_ms_avg=float(each.mean()) if launches else None, launches=launches,
               kernel_ms_median=float(np.median(each)) if launches else None,
               kernel_ms_min=float(each.min()) if launches else None,
               request_ms_median=float(np.median(req_ms)), request_ms_min=float(req_ms.min()), requests_timed=n,
               clusters=[bps.bps_query(r.handle, h, 0) for h in handles],
               splits=bps.bps_query(r.handle, handles[0], 4), groups=bps.bps_query(r.handle, handles[0], 5),
               threads=bps.bps_query(r.handle, handles[0], 6), lds=bps.bps_query(r.handle, handles[0], 7))
    if diagnostics:
        # work counts for the culling-aware byte accounting: averaged over the pose sets of the cycle
        bps.bps_set_diagnostics(r.handle, 1)
        diag = None
        for k in range(len(cycle)):
            submit(k)
            d = bps.bps_read_diagnostics(r.handle, 1 << 22).reshape(-1, 16).astype(np.float64)
            diag = d if diag is None else diag + d
        res["diag"] = diag / len(cycle)
        bps.bps_set_diagnostics(r.handle, 0)
    r.close()
    return res


def inputs_ready_run(bps, torch, w, steps, warmup):
    """The headline request with BPS_FLAG_INPUTS_READY: the matrices, resident on the device since before
    the timed region, are declared complete at every call, so the renderer stages and plans each
    request on its own stream while the previous one is still being drawn."""
    r = bps.Renderer(max_batch=w.B, height=w.H, width=w.W, flags=bps.FLAG_INPUTS_READY)
    hmap = np.array([r.load_scene(s.vertices, s.indices) for s in w.scenes], np.int32)
    cycle = [(hmap[ids], vp) for ids, vp in pose_cycle(torch, w)]
    depth = torch.empty((w.B, w.H, w.W), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    for k in range(max(warmup, len(cycle))):
        bps.bps_render(r.handle, *cycle[k % len(cycle)], depth, stream=stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        bps.bps_render(r.handle, *cycle[k % len(cycle)], depth, stream=stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    r.close()
    return {"value": w.B * steps / dt, "unit": "frames/s", "steps": steps, "ms_per_step": dt * 1e3 / steps}


def in_flight_run(bps, torch, w, steps, warmup, n_streams=2):
    """The same requests issued alternately on n_streams streams, each with its own output frames,
    so that consecutive requests overlap on the device and fill the compute units that the end of
    each launch leaves idle.  Reported beside the headline figure, which keeps one stream."""
    r = bps.Renderer(max_batch=w.B, height=w.H, width=w.W)
    hmap = np.array([r.load_scene(s.vertices, s.indices) for s in w.scenes], np.int32)
    cycle = [(hmap[ids], vp) for ids, vp in pose_cycle(torch, w)]
    depth = [torch.empty((w.B, w.H, w.W), dtype=torch.float32, device="cuda") for _ in range(n_streams)]
    streams = [torch.cuda.Stream() for _ in range(n_streams)]
    for k in range(max(warmup, len(cycle))):
        bps.bps_render(r.handle, *cycle[k % len(cycle)], depth[k % n_streams], stream=streams[k % n_streams])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        bps.bps_render(r.handle, *cycle[k % len(cycle)], depth[k % n_streams], stream=streams[k % n_streams])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # the same request on each stream must give the same frames
    for d, st in zip(depth, streams):
        bps.bps_render(r.handle, *cycle[0], d, stream=st)
    torch.cuda.synchronize()
    same = all(bool((d == depth[0]).all()) for d in depth[1:])
    r.close()
    return {"requests_in_flight": n_streams, "value": w.B * steps / dt, "unit": "frames/s", "steps": steps,
            "ms_per_step": dt * 1e3 / steps, "frames_identical_across_streams": same}


def rotation_run(bps, torch, w, steps, warmup):
    """Render while a loader thread keeps replacing scenes (asynchronous uploads on a side stream,
    retired scenes recycled): the paper's continuous rotation of the K resident assets (Sec. 3.2)."""
    import threading
    import synth
    r = bps.Renderer(max_batch=w.B, height=w.H, width=w.W)
    K = len(w.scenes)
    handles = [r.load_scene(s.vertices, s.indices) for s in w.scenes]
    spare = [synth.make_multiroom_scene(w.scenes[0].T, seed=1500 + k) for k in range(2)]
    pool = list(w.scenes) + spare
    state = {"ids": np.array([handles[k] for k in w.scene_ids], np.int32), "stop": False, "loaded": 0, "load_s": 0.0, "submitted": 0}
    lock = threading.Lock()
    copy_stream = torch.cuda.Stream()
    vp = torch.from_numpy(w.view_proj).cuda()
    depth = torch.empty((w.B, w.H, w.W), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def loader():
        slot_handles = list(handles)
        n = 0
        while not state["stop"]:
            k = n % K                                   # scene slot to replace
            mesh = pool[(n + K) % len(pool)]
            t0 = time.perf_counter()
            new = bps.bps_load_scene_async(r.handle, mesh.vertices, mesh.indices, None, copy_stream)
            state["load_s"] += time.perf_counter() - t0
            old = slot_handles[k]
            slot_handles[k] = new
            with lock:
                state["ids"] = np.array([slot_handles[j] for j in w.scene_ids], np.int32)
                mark = state["submitted"]
            # the render thread may have read the old ids just before the swap: the old scene is retired once
            # that request has been submitted (requests that use it may well still be queued: allowed)
            while state["submitted"] < mark + 2 and not state["stop"]:
                time.sleep(0.0002)
            bps.bps_unload_scene(r.handle, old)
            state["loaded"] += 1
            n += 1

    for _ in range(warmup):
        bps.bps_render(r.handle, state["ids"], vp, depth, stream=stream)
    torch.cuda.synchronize()
    th = threading.Thread(target=loader)
    th.start()
    t0 = time.perf_counter()
    for _ in range(steps):
        with lock:
            ids = state["ids"]
        bps.bps_render(r.handle, ids, vp, depth, stream=stream)
        state["submitted"] += 1
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    state["stop"] = True
    th.join()
    torch.cuda.synchronize()
    out = {"frames_per_s": w.B * steps / dt, "steps": steps, "scenes_loaded_meanwhile": state["loaded"],
           "host_ms_per_load": 1e3 * state["load_s"] / max(1, state["loaded"]),
           "device_blocks_allocated": bps.bps_query(r.handle, 0, 8),
           "note": "one loader thread replaces scenes back to back (cluster packing on the host, copy on a side stream) "
                   "while the render thread issues requests; every request after a swap uses the new scene"}
    r.close()
    return out


def sweep(bps, torch, steps, warmup):
    """Frames/s over batch size and resolution on the headline scenes (the shape of the paper's
    stand-alone renderer figure, App. A.2).  Prints one JSON object per point."""
    import synth
    base = synth.build_config(3)
    for res in (32, 64, 128):
        for B in (1, 8, 64, 256, 512, 1024, 2048):
            reps = (B + base.B - 1) // base.B
            w = synth.Workload(3, base.scenes, np.tile(base.scene_ids, reps)[:B], np.tile(base.view_proj, (reps, 1, 1))[:B],
                               res, res, False)
            run = timed_run(bps, torch, w, 0, steps, warmup, 0, 0, n_sets=1, request_pass=4)
            print(json.dumps({"sweep": True, "B": B, "H": res, "W": res, "frames_per_s": B * steps / run["dt"],
                              "ms_per_request": run["dt"] * 1e3 / steps, "kernel_ms": run["kernel_ms_avg"],
                              "work_groups": run["groups"], "splits": run["splits"]}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="workload number (3 = headline)")
    ap.add_argument("--batch", type=int, default=None, help="override the environment count")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--threads", type=int, default=0)
    ap.add_argument("--no-cull", action="store_true", help="stream every cluster (no culling of clusters)")
    ap.add_argument("--no-occlusion", action="store_true", help="frustum culling of clusters only")
    ap.add_argument("--no-dispatch-order", action="store_true", help="launch work-groups in batch order")
    ap.add_argument("--inputs-ready", action="store_true",
                    help="tell the renderer that the device-resident matrices are complete at every call, so that it plans "
                         "the launch on its own stream while the previous request is still being drawn")
    ap.add_argument("--sweep", action="store_true", help="batch-size x resolution sweep instead of the single benchmark line")
    ap.add_argument("--textured", action="store_true",
                    help="RGB-D workloads: colour from each scene's texture (uv + mip pyramid) instead of vertex colours")
    ap.add_argument("--rotate", action="store_true", help="also time rendering while scenes are being replaced")
    ap.add_argument("--jitter", type=float, default=0.0, metavar="CELLS",
                    help="time the workload on its irregular variant: furniture turned off-axis and every vertex displaced "
                         "by up to this many grid cells (multi-room workloads; 0 = the regular scenes)")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed run: no diagnostics request, no full-stream run (for profiler runs)")
    ap.add_argument("--cpu-envs", type=int, default=512, help="environments in the oracle timing sample (0 = skip)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="instead of rendering, run a plain device-to-device copy of this many MiB five times "
                         "(reference reading for the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.copy_calibration > 0:
        import torch
        n = args.copy_calibration * (1 << 20)
        a = torch.full((n // 4,), 1.0, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_MiB": args.copy_calibration, "reads_MiB": args.copy_calibration,
                          "writes_MiB": args.copy_calibration, "repeats": 5}))
        return
    if args.gpus != 1:
        sys.exit("bench.py: this build renders on ONE GPU; frames shard by environment with no exchange, "
                 "so run one process per GPU instead of --gpus %d" % args.gpus)

    import torch
    import synth
    import paper_2103_07013_amd as bps

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the renderer has no CPU path")

    if args.sweep:
        sweep(bps, torch, min(args.steps, 30), 5)
        return
    w = synth.build_config(args.config, B=args.batch, jitter=args.jitter)
    flags = ((bps.FLAG_NO_CLUSTER_CULL if args.no_cull else 0) | (bps.FLAG_NO_OCCLUSION_CULL if args.no_occlusion else 0) |
             (bps.FLAG_NO_DISPATCH_ORDER if args.no_dispatch_order else 0) |
             (bps.FLAG_INPUTS_READY if args.inputs_ready else 0))
    culling = not args.no_cull
    main_run = timed_run(bps, torch, w, flags, args.steps, args.warmup, args.splits, args.threads,
                         diagnostics=culling and not args.no_extras, textured=args.textured)
    dt = main_run["dt"]
    kernel_ms_avg = main_run["kernel_ms_avg"]
    variant = "full_stream" if args.no_cull else ("frustum_cull" if args.no_occlusion else "cull")

    fbytes = full_stream_bytes(w)
    if culling and "diag" in main_run:
        per_scene = [((12.0 * s.T + 12.0 * s.V) / c, c) for s, c in zip(w.scenes, main_run["clusters"])]
        diag = main_run["diag"]
        # the scenes of one workload have near-identical cluster sizes: use the average bytes per cluster
        avg_cluster_bytes = float(np.mean([p[0] for p in per_scene]))
        blocks = sum((per_scene[s][1] + 63) // 64 for s in w.scene_ids)
        abytes = (float(diag[:, 2].sum()) * avg_cluster_bytes + 24.0 * (blocks + float(diag[:, 0].sum())) +
                  w.B * w.H * w.W * (7 if w.rgbd else 4) + w.B * 68)
        accounting = ("culling: 24 B bounds per block and per tested cluster + mesh bytes (12 B/triangle + 12 B/vertex, "
                      "scene average per cluster) of clusters that reached the triangle phase + output + request")
        extra = {"clusters_tested": int(diag[:, 0].sum()), "clusters_kept_by_bounds_tests": int(diag[:, 1].sum()),
                 "clusters_drawn": int(diag[:, 2].sum()), "clusters_skipped_as_occluded": int(diag[:, 4].sum()),
                 "clusters_in_batch": int(sum(per_scene[s][1] for s in w.scene_ids))}
    elif culling:
        abytes, accounting, extra = None, "culling on; diagnostics skipped (--no-extras)", {}
    else:
        abytes = fbytes
        accounting = "full stream: 12 B/triangle + 12 B/vertex per environment + output + request"
        extra = {}

    def roofline(nbytes, ms, note, traffic_key):
        if nbytes is None:
            return None
        achieved = nbytes / (ms * 1e-3) / 1e9
        traffic = measured_traffic(traffic_key)
        out = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
               "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
               # what the counters say really crossed between L2 and the memory side, as a rate and against the peak
               "traffic_GBs": None if traffic is None else traffic / (ms * 1e-3) / 1e9,
               "traffic_frac": None if traffic is None else traffic / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
               "kernel": "k_raster", "kernel_ms_avg": ms, "algorithmic_bytes_per_launch": nbytes, "accounting": note}
        valu = measured_traffic(traffic_key + "_valu_insts")
        if valu:
            # what the counters say binds the kernel: vector-ALU issue (1024 SIMDs, 4 cycles per wave64 instruction)
            peak = VALU_ISSUE_PEAK
            out["valu_issue"] = {"insts_per_launch": valu, "achieved_Ginst_s": valu / (ms * 1e-3) / 1e9,
                                 "peak_Ginst_s": peak / 1e9, "frac": valu / (ms * 1e-3) / peak,
                                 "note": "SQ_INSTS_VALU from the rocprofv3 run under profiles/ over this run's kernel time"}
        return out

    def copy_ceiling_gbs():
        """Read + write rate of a plain 1 GiB device-to-device copy: what a pure streaming kernel gets."""
        n = 1 << 30
        a = torch.empty(n, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            b.copy_(a)
        e1.record()
        torch.cuda.synchronize()
        return 2.0 * n * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9

    out = {
        "metric": f"rendered frames/sec ({w.H}x{w.W} {'RGB-D' if w.rgbd else 'depth'}, {w.B} envs) on 1 MI355X",
        "value": w.B * args.steps / dt,
        "unit": "frames/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": dt * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"config{w.number}: {len(w.scenes)} procedural {'multi-room' if w.number > 1 else 'room'} scenes x "
                        f"~{w.scenes[0].T} triangles, {w.B} environments (scene = b mod {len(w.scenes)}), "
                        f"{w.H}x{w.W} {('textured RGB-D' if args.textured else 'RGB-D') if w.rgbd else 'float32 depth'}",
            "variant": variant + (f", irregular geometry (jitter {args.jitter})" if args.jitter else ""),
            "B": w.B, "H": w.H, "W": w.W, "scenes": len(w.scenes),
            "triangles_per_scene": [s.T for s in w.scenes],
            "env_triangles_per_step": w.env_triangles,
            "splits": main_run["splits"], "work_groups": main_run["groups"], "threads": main_run["threads"],
            "lds_bytes": main_run["lds"],
        },
        "env_triangles_per_s": w.env_triangles * args.steps / dt,
        "request_ms_median": main_run["request_ms_median"], "request_ms_min": main_run["request_ms_min"],
        "requests_timed_one_by_one": main_run["requests_timed"],
        "timing": "value = B x steps / wall time of the steps (bracketed by synchronisations; requests cycle through 4 "
                  "pose sets, one of them with permuted scene ids); request_ms_* from a separate pass with a HIP event "
                  "after every request; roofline.kernel_ms_* from a third pass with events around the raster kernel",
        "roofline": roofline(abytes, kernel_ms_avg, accounting, f"config{w.number}_{variant}"),
    }
    if out["roofline"] is not None:
        out["roofline"].update(extra)
        out["roofline"]["launches_timed"] = main_run["launches"]
        out["roofline"]["kernel_ms_median"] = main_run["kernel_ms_median"]
        out["roofline"]["kernel_ms_min"] = main_run["kernel_ms_min"]
        if not args.no_extras:
            ceiling = copy_ceiling_gbs()
            out["roofline"]["copy_ceiling_GBs"] = ceiling
            out["roofline"]["frac_of_copy_ceiling"] = out["roofline"]["achieved"] / ceiling
    if culling and not args.no_extras:
        steps2 = max(5, args.steps // 5)
        fs = timed_run(bps, torch, w, bps.FLAG_NO_CLUSTER_CULL, steps2, 3, args.splits, args.threads,
                       textured=args.textured)
        rl = roofline(fbytes, fs["kernel_ms_avg"],
                      "full stream: 12 B/triangle + 12 B/vertex per environment + output + request; same request "
                      "with cluster culling switched off", f"config{w.number}_full_stream")
        rl["frames_per_s"] = w.B * steps2 / fs["dt"]
        rl["launches_timed"] = fs["launches"]
        rl["kernel_ms_median"] = fs["kernel_ms_median"]
        rl["kernel_ms_min"] = fs["kernel_ms_min"]
        if out["roofline"] is not None and "copy_ceiling_GBs" in out["roofline"]:
            rl["frac_of_copy_ceiling"] = rl["achieved"] / out["roofline"]["copy_ceiling_GBs"]
        out["roofline_full_stream"] = rl
    if culling and not args.no_extras and not w.rgbd and args.splits <= 1:
        out["two_requests_in_flight"] = in_flight_run(bps, torch, w, args.steps, args.warmup)
        if not args.inputs_ready:
            out["inputs_declared_ready"] = inputs_ready_run(bps, torch, w, args.steps, args.warmup)
    if culling and not args.no_extras and not w.rgbd and w.number > 1 and not args.jitter:
        # the same workload on irregular geometry (furniture turned off-axis, every vertex displaced by up to 0.3 grid
        # cells): shows what the cluster packing and the culling owe to axis-aligned, regular grids
        wj = synth.build_config(args.config, B=args.batch, jitter=0.3)
        steps2 = max(10, args.steps // 2)
        rj = timed_run(bps, torch, wj, flags, steps2, 5, args.splits, args.threads, diagnostics=True)
        dj = rj["diag"]
        out["irregular_geometry"] = {
            "what": "same configuration with the scenes' furniture turned about its vertical axis by random angles and "
                    "every vertex displaced by up to 0.3 grid cells per axis (bench.py --jitter 0.3 times it alone)",
            "value": wj.B * steps2 / rj["dt"], "unit": "frames/s", "ms_per_step": rj["dt"] * 1e3 / steps2,
            "kernel_ms_median": rj["kernel_ms_median"], "clusters_drawn": int(dj[:, 2].sum()),
            "clusters_in_batch": int(sum(rj["clusters"][s] for s in wj.scene_ids)),
            "triangles_per_scene": [s.T for s in wj.scenes]}
    if args.rotate and not w.rgbd:
        out["rotation"] = rotation_run(bps, torch, w, max(2000, args.steps), args.warmup)
    if args.cpu_envs > 0:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_envs, args.textured)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
