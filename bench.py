#!/usr/bin/env python3
"""Benchmark of the batch renderer hot path on one MI355X.

A step is one complete render request (request staging + the fused raster kernel, plus the
resolve kernel when frames are split) for the headline workload: 4 procedural multi-room
scenes of ~500k triangles, 1024 environments (256 per scene, interleaved), 64x64 float32
depth.  Scenes and view-projection matrices are resident in HBM before the timed region.
Prints ONE JSON line.
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


def algorithmic_bytes(w):
    """Bytes the method itself must move per request: every environment streams its scene's
    index and vertex arrays once (12 B per triangle + 12 B per vertex), the frames are written
    once (4 B per pixel), and the request (scene id + matrix, 68 B) is read once."""
    geo = sum(12 * w.scenes[s].T + 12 * w.scenes[s].V for s in w.scene_ids)
    out = w.B * w.H * w.W * 4
    return geo + out + w.B * 68


def cpu_baseline(w, n_envs):
    """Time the CPU oracle, as it stands, on a strided sample of the same workload."""
    import oracle
    stride = max(1, w.B // n_envs)
    sel = np.arange(0, w.B, stride)[:n_envs]
    t0 = time.perf_counter()
    r = oracle.render_batch(w.scenes, w.scene_ids[sel], w.view_proj[sel], w.H, w.W)
    dt = time.perf_counter() - t0
    return dict(value=len(sel) / dt, unit="frames/s", cores=int(r["threads"]), kind="oracle",
                sample=f"{len(sel)} of {w.B} environments (every {stride}th), same scenes and matrices, {dt:.2f} s wall")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="workload number (3 = headline)")
    ap.add_argument("--batch", type=int, default=None, help="override the environment count")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--threads", type=int, default=0)
    ap.add_argument("--no-cull", action="store_true", help="stream every cluster (no frustum culling of clusters)")
    ap.add_argument("--no-occlusion", action="store_true", help="frustum culling of clusters only")
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

    w = synth.build_config(args.config, B=args.batch)
    if w.rgbd:
        sys.exit("bench.py: RGB-D workloads are not wired into the benchmark yet")
    r = bps.Renderer(max_batch=w.B, height=w.H, width=w.W, splits=args.splits, threads=args.threads,
                     flags=(bps.FLAG_NO_CLUSTER_CULL if args.no_cull else 0) |
                           (bps.FLAG_NO_OCCLUSION_CULL if args.no_occlusion else 0))
    handles = [r.load_scene(s.vertices, s.indices, None) for s in w.scenes]
    ids = np.array([handles[k] for k in w.scene_ids], np.int32)
    vp = torch.from_numpy(w.view_proj).cuda()
    depth = torch.empty((w.B, w.H, w.W), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    for _ in range(args.warmup):
        bps.bps_render(r.handle, ids, vp, depth, stream=stream)
    torch.cuda.synchronize()
    bps.bps_set_profiling(r.handle, True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        bps.bps_render(r.handle, ids, vp, depth, stream=stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    launches, kernel_ms = bps.bps_kernel_ms_total(r.handle)
    bps.bps_set_profiling(r.handle, False)

    ms_per_step = dt * 1e3 / args.steps
    kernel_ms_avg = kernel_ms / max(launches, 1)
    abytes = algorithmic_bytes(w)
    achieved = abytes / (kernel_ms_avg * 1e-3) / 1e9
    clusters = sum(bps.bps_query(r.handle, h, 0) for h in handles)
    out = {
        "metric": "rendered frames/sec (64x64 depth, 1024 envs) on 1 MI355X",
        "value": w.B * args.steps / dt,
        "unit": "frames/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"config{w.number}: {len(w.scenes)} procedural multi-room scenes x ~{w.scenes[0].T} triangles, "
                        f"{w.B} environments (scene = b mod {len(w.scenes)}), {w.H}x{w.W} float32 depth",
            "B": w.B, "H": w.H, "W": w.W, "scenes": len(w.scenes),
            "triangles_per_scene": [s.T for s in w.scenes],
            "env_triangles_per_step": w.env_triangles,
            "clusters_total": clusters,
            "splits": bps.bps_query(r.handle, handles[0], 4),
            "work_groups": bps.bps_query(r.handle, handles[0], 5),
            "threads": bps.bps_query(r.handle, handles[0], 6),
            "lds_bytes": bps.bps_query(r.handle, handles[0], 7),
        },
        "env_triangles_per_s": w.env_triangles * args.steps / dt,
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": None,
            "kernel": "k_raster",
            "kernel_ms_avg": kernel_ms_avg,
            "launches_timed": launches,
            "algorithmic_bytes_per_launch": abytes,
        },
    }
    if args.cpu_envs > 0:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_envs)
    r.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
