"""The five benchmark / parity workloads, each fully determined by its number and seeds."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from .cameras import make_cameras
from .scenes import make_multiroom_scene, make_room_scene

# number -> (scene kind, K scenes, triangles per scene, B environments, H, W, rgbd)
CONFIGS = {
    1: dict(kind="room", K=1, T=10_000, B=16, H=64, W=64, rgbd=False),
    2: dict(kind="multiroom", K=1, T=200_000, B=256, H=64, W=64, rgbd=False),
    3: dict(kind="multiroom", K=4, T=500_000, B=1024, H=64, W=64, rgbd=False),
    4: dict(kind="multiroom", K=8, T=1_000_000, B=1024, H=64, W=64, rgbd=True),
    5: dict(kind="multiroom", K=16, T=1_000_000, B=4096, H=128, W=128, rgbd=False),
}


@dataclass
class Workload:
    number: int
    scenes: list                 # list[Scene], K entries
    scene_ids: np.ndarray        # int32 [B], index into scenes (interleaved: b mod K)
    view_proj: np.ndarray        # float32 [B,4,4]
    H: int
    W: int
    rgbd: bool

    @property
    def B(self):
        return int(self.scene_ids.shape[0])

    @property
    def env_triangles(self):
        return int(sum(self.scenes[s].T for s in self.scene_ids))

    def describe(self):
        return (f"config{self.number}: K={len(self.scenes)} scenes x ~{self.scenes[0].T} tris, "
                f"B={self.B}, {self.H}x{self.W} {'rgbd' if self.rgbd else 'depth'}")


def build_config(number, B=None, scale=1.0, jitter=0.0, pose_set=0):
    """Build workload `number`.  B overrides the environment count; scale < 1 shrinks the
    per-scene triangle target (for quick CPU tests of the same structure); jitter > 0 gives the
    irregular variant of the multi-room scenes (furniture turned off-axis, vertices displaced by
    up to jitter x the grid cell); pose_set > 0 draws another seeded set of camera poses for the
    same scenes (pose_set 0 is the workload's own)."""
    c = CONFIGS[number]
    K = c["K"]
    B = c["B"] if B is None else B
    T = max(500, int(c["T"] * scale))
    scenes = []
    for k in range(K):
        if c["kind"] == "room":
            scenes.append(make_room_scene(T, seed=1000 + k))
        else:
            scenes.append(make_multiroom_scene(T, seed=1000 + k, jitter=jitter))
    scene_ids = (np.arange(B) % K).astype(np.int32)
    vp = np.empty((B, 4, 4), np.float32)
    aspect = c["W"] / c["H"]
    for k in range(K):
        sel = np.nonzero(scene_ids == k)[0]
        if sel.size:
            m, _ = make_cameras(scenes[k], sel.size, seed=(2000 + number) * 100 + k + 100_000 * pose_set, aspect=aspect)
            vp[sel] = m
    return Workload(number, scenes, scene_ids, vp, c["H"], c["W"], c["rgbd"])


def more_poses(w, pose_set):
    """Another seeded set of camera poses [B,4,4] for the scenes and scene ids of workload w."""
    vp = np.empty_like(w.view_proj)
    K = len(w.scenes)
    for k in range(K):
        sel = np.nonzero(w.scene_ids == k)[0]
        if sel.size:
            m, _ = make_cameras(w.scenes[k], sel.size, seed=(2000 + w.number) * 100 + k + 100_000 * pose_set, aspect=w.W / w.H)
            vp[sel] = m
    return vp
