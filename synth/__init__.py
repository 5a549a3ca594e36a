"""Seeded synthetic inputs: procedural indoor scenes and camera poses.

This package only manufactures inputs (triangle meshes, colours, camera
matrices).  It contains none of the renderer's arithmetic and is the one piece
shared by the CPU oracle's tests and the GPU path's tests and benchmark.

The scenes stand in for the scanned indoor datasets the paper renders (Sec. 3.2,
Sec. 4.1): tens of thousands to about a million triangles per scene, most of
them sub-pixel at 64x64, viewed by an agent camera at fixed height that only
yaws (Appendix A.3, agent actions).
"""
from .scenes import Scene, make_room_scene, make_multiroom_scene
from .cameras import make_cameras, perspective, look_yaw, view_proj_from_pose
from .configs import CONFIGS, build_config, more_poses, Workload

__all__ = [
    "Scene", "make_room_scene", "make_multiroom_scene", "make_cameras",
    "perspective", "look_yaw", "view_proj_from_pose", "CONFIGS",
    "build_config", "more_poses", "Workload",
]
