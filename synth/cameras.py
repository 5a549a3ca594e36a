"""Seeded agent cameras and their view-projection matrices.

Conventions (the request format of the renderer): row-major 4x4 matrix M,
clip = M @ (x, y, z, 1); normalised x right, y DOWN, z in [0, 1]; clip w is the
eye-space depth.  Matrices are composed in float64 and rounded once to float32.
"""
from __future__ import annotations

import math

import numpy as np


def perspective(hfov_deg=90.0, aspect=1.0, near=0.01, far=20.0):
    """Projection from a right-handed eye frame looking down -z (y up) to clip space."""
    f = 1.0 / math.tan(math.radians(hfov_deg) / 2.0)
    P = np.zeros((4, 4), np.float64)
    P[0, 0] = f
    P[1, 1] = -f * aspect                   # flip: image y grows downwards
    P[2, 2] = far / (near - far)
    P[2, 3] = near * far / (near - far)
    P[3, 2] = -1.0                          # w_clip = -z_eye = distance along the view axis
    return P


def look_yaw(pos, yaw, pitch=0.0):
    """World -> eye matrix for a camera at pos, rotated yaw about +Y then pitch about eye x."""
    cy, sy = math.cos(yaw), math.sin(yaw)
    cp, sp = math.cos(pitch), math.sin(pitch)
    # eye axes in world coordinates (yaw = 0 looks down world -z)
    right = np.array([cy, 0.0, -sy])
    fwd = np.array([-sy * cp, sp, -cy * cp])
    up = np.cross(right, fwd)
    R = np.stack([right, up, -fwd], 0)      # rows: eye x, y, z axes
    V = np.eye(4)
    V[:3, :3] = R
    V[:3, 3] = -R @ np.asarray(pos, np.float64)
    return V


def view_proj_from_pose(pos, yaw, pitch=0.0, hfov_deg=90.0, aspect=1.0, near=0.01, far=20.0):
    return (perspective(hfov_deg, aspect, near, far) @ look_yaw(pos, yaw, pitch)).astype(np.float32)


def _free(scene, x, z):
    for wx in scene.wall_x:
        if abs(x - wx) < 0.1:
            return False
    for wz in scene.wall_z:
        if abs(z - wz) < 0.1:
            return False
    b = scene.boxes
    if b.shape[0] and np.any((x > b[:, 0] - 0.1) & (x < b[:, 2] + 0.1) & (z > b[:, 1] - 0.1) & (z < b[:, 3] + 0.1)):
        return False
    c = scene.cylinders
    if c.shape[0] and np.any((x - c[:, 0]) ** 2 + (z - c[:, 1]) ** 2 < (c[:, 2] + 0.1) ** 2):
        return False
    return True


def make_cameras(scene, n, seed, height=1.25, hfov_deg=90.0, near=0.01, far=20.0, aspect=1.0):
    """n poses: uniform floor position (rejection-sampled to free space), uniform yaw, level.

    Returns (view_proj float32 [n,4,4], poses float64 [n,3] = x, z, yaw)."""
    rng = np.random.default_rng(seed)
    SX, SZ = scene.extent
    out = np.empty((n, 4, 4), np.float32)
    poses = np.empty((n, 3), np.float64)
    k = 0
    while k < n:
        x = rng.uniform(0.3, SX - 0.3)
        z = rng.uniform(0.3, SZ - 0.3)
        yaw = rng.uniform(0.0, 2.0 * math.pi)
        if not _free(scene, x, z):
            continue
        out[k] = view_proj_from_pose((x, height, z), yaw, 0.0, hfov_deg, aspect, near, far)
        poses[k] = (x, z, yaw)
        k += 1
    return out, poses
