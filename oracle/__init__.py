"""CPU oracle for the batch renderer -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

A plain C rasteriser (raster_oracle.c) that states, step by step, what one
`render` request must produce (paper Sec. 3 and Sec. 3.2: one request per
environment in, one frame per environment out, scenes shared by reference).
Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It neither imports nor is imported by the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "raster_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared"]


def build(force=False):
    """Compile the oracle with gcc (no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        f32p, u32p, u8p, i32p = (ctypes.POINTER(t) for t in (ctypes.c_float, ctypes.c_uint32, ctypes.c_uint8, ctypes.c_int32))
        lib.oracle_render.restype = ctypes.c_int
        lib.oracle_render.argtypes = [f32p, ctypes.c_uint32, u32p, ctypes.c_uint32, u8p, f32p, ctypes.c_uint32,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_float, f32p, u32p, u8p, u32p, ctypes.c_int]
        lib.oracle_render_textured.restype = ctypes.c_int
        lib.oracle_render_textured.argtypes = [f32p, ctypes.c_uint32, u32p, ctypes.c_uint32, u8p, f32p, u8p, ctypes.c_int,
                                               ctypes.c_int, f32p, ctypes.c_uint32, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_float, f32p, u32p, u8p, u32p, ctypes.c_int]
        lib.oracle_render_filtered.restype = ctypes.c_int
        lib.oracle_render_filtered.argtypes = [f32p, ctypes.c_uint32, u32p, ctypes.c_uint32, u8p, f32p, u8p, ctypes.c_int,
                                               ctypes.c_int, ctypes.c_int, f32p, ctypes.c_uint32, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_float, f32p, u32p, u8p, u32p, ctypes.c_int]
        lib.oracle_sample_filtered.restype = None
        lib.oracle_sample_filtered.argtypes = [u8p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_float,
                                               ctypes.c_int, u8p]
        lib.oracle_sample.restype = None
        lib.oracle_sample.argtypes = [u8p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_float, u8p]
        lib.oracle_cover_fixed.restype = None
        lib.oracle_cover_fixed.argtypes = [i32p, ctypes.c_uint32, ctypes.c_int, ctypes.c_int, u32p]
        lib.oracle_clip.restype = ctypes.c_int
        lib.oracle_clip.argtypes = [f32p, f32p, f32p]
        lib.oracle_clip_stats.restype = None
        lib.oracle_clip_stats.argtypes = [i32p, i32p, ctypes.c_int]
        lib.oracle_downsample2.restype = None
        lib.oracle_downsample2.argtypes = [f32p, u8p, ctypes.c_uint32, ctypes.c_int, ctypes.c_int, f32p, u8p]
        _lib = lib
    return _lib


def _p(a, t):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(t))


def render_scene(vertices, indices, view_proj, H, W, colors=None, background=0.0, want_cover=False, nthreads=0,
                 uvs=None, texture=None, bilinear=False):
    """Render every matrix in view_proj[B,4,4] against one mesh.  With uvs [V,2] and texture
    [th,tw,3] uint8 the colour output is sampled from the texture (rule N10, or N11 with bilinear).

    Returns dict(depth f32 [B,H,W], tri_id u32 [B,H,W], rgb u8 [B,H,W,3] | None,
    cover u32 [B,H,W] | None, threads int)."""
    lib = _load()
    v = np.ascontiguousarray(vertices, np.float32).reshape(-1, 3)
    i = np.ascontiguousarray(indices, np.uint32).reshape(-1, 3)
    m = np.ascontiguousarray(view_proj, np.float32).reshape(-1, 4, 4)
    if i.size and int(i.max()) >= v.shape[0]:
        raise ValueError("index out of range")
    B = m.shape[0]
    c = None if colors is None else np.ascontiguousarray(colors, np.uint8).reshape(-1, 3)
    uv = None if uvs is None else np.ascontiguousarray(uvs, np.float32).reshape(-1, 2)
    tex = None if texture is None else np.ascontiguousarray(texture, np.uint8)
    if (uv is None) != (tex is None):
        raise ValueError("uvs and texture go together")
    depth = np.empty((B, H, W), np.float32)
    tid = np.empty((B, H, W), np.uint32)
    rgb = np.zeros((B, H, W, 3), np.uint8) if (c is not None or tex is not None) else None
    cover = np.zeros((B, H, W), np.uint32) if want_cover else None
    used = lib.oracle_render_filtered(_p(v, ctypes.c_float), v.shape[0], _p(i, ctypes.c_uint32), i.shape[0],
                                      _p(c, ctypes.c_uint8), _p(uv, ctypes.c_float), _p(tex, ctypes.c_uint8),
                                      0 if tex is None else tex.shape[1], 0 if tex is None else tex.shape[0],
                                      1 if bilinear else 0, _p(m, ctypes.c_float), B, H, W, float(background),
                                      _p(depth, ctypes.c_float), _p(tid, ctypes.c_uint32), _p(rgb, ctypes.c_uint8),
                                      _p(cover, ctypes.c_uint32), int(nthreads))
    if used < 0:
        raise RuntimeError("oracle: a clipped polygon needed more corners than the clipper holds")
    return dict(depth=depth, tri_id=tid, rgb=rgb, cover=cover, threads=used)


def clip_stats(reset=False):
    """(polygons that outgrew the clipper, largest corner count reached) since the last reset."""
    lib = _load()
    a, b = ctypes.c_int32(0), ctypes.c_int32(0)
    lib.oracle_clip_stats(ctypes.byref(a), ctypes.byref(b), 1 if reset else 0)
    return int(a.value), int(b.value)


def downsample2(depth, rgb=None):
    """2x2 box filter of supersampled frames: depth f32 [B,2H,2W] (and rgb u8 [B,2H,2W,3]) ->
    (depth [B,H,W], rgb [B,H,W,3] | None)."""
    lib = _load()
    d = np.ascontiguousarray(depth, np.float32)
    B, H2, W2 = d.shape
    H, W = H2 // 2, W2 // 2
    c = None if rgb is None else np.ascontiguousarray(rgb, np.uint8)
    od = np.empty((B, H, W), np.float32)
    oc = None if c is None else np.empty((B, H, W, 3), np.uint8)
    lib.oracle_downsample2(_p(d, ctypes.c_float), _p(c, ctypes.c_uint8), B, H, W, _p(od, ctypes.c_float), _p(oc, ctypes.c_uint8))
    return od, oc


def render_batch(scenes, scene_ids, view_proj, H, W, rgbd=False, background=0.0, nthreads=0, want_cover=False,
                 textured=False, bilinear=False):
    """Render a mixed batch: env b uses scenes[scene_ids[b]] (objects with .vertices/.indices/.colors,
    and .uvs/.texture when textured)."""
    scene_ids = np.asarray(scene_ids)
    B = scene_ids.shape[0]
    depth = np.empty((B, H, W), np.float32)
    tid = np.empty((B, H, W), np.uint32)
    rgb = np.zeros((B, H, W, 3), np.uint8) if rgbd else None
    cover = np.zeros((B, H, W), np.uint32) if want_cover else None
    threads = 1
    for k in np.unique(scene_ids):
        sel = np.nonzero(scene_ids == k)[0]
        s = scenes[int(k)]
        r = render_scene(s.vertices, s.indices, view_proj[sel], H, W, colors=s.colors if (rgbd and not textured) else None,
                         background=background, nthreads=nthreads, want_cover=want_cover,
                         uvs=s.uvs if textured else None, texture=s.texture if textured else None, bilinear=bilinear)
        depth[sel], tid[sel] = r["depth"], r["tri_id"]
        if rgbd:
            rgb[sel] = r["rgb"]
        if want_cover:
            cover[sel] = r["cover"]
        threads = r["threads"]
    return dict(depth=depth, tri_id=tid, rgb=rgb, cover=cover, threads=threads)


def sample(texture, level, u, v, bilinear=False):
    """The RGB colour rule N10 (nearest texel) or N11 (bilinear) gives for (u, v) at mip level `level`."""
    lib = _load()
    tex = np.ascontiguousarray(texture, np.uint8)
    out = np.zeros(3, np.uint8)
    lib.oracle_sample_filtered(_p(tex, ctypes.c_uint8), tex.shape[1], tex.shape[0], int(level), float(u), float(v),
                               1 if bilinear else 0, _p(out, ctypes.c_uint8))
    return out


def cover_fixed(xy, H, W):
    """Coverage counts of triangles given in 1/256-pixel integer coordinates xy[n,3,2]."""
    lib = _load()
    a = np.ascontiguousarray(xy, np.int32).reshape(-1, 3, 2)
    cover = np.zeros((H, W), np.uint32)
    lib.oracle_cover_fixed(_p(a, ctypes.c_int32), a.shape[0], H, W, _p(cover, ctypes.c_uint32))
    return cover


def clip(view_proj, tri_xyz):
    """Clip-space polygon (n,4) of one world-space triangle after transform and frustum clipping."""
    lib = _load()
    m = np.ascontiguousarray(view_proj, np.float32).reshape(4, 4)
    t = np.ascontiguousarray(tri_xyz, np.float32).reshape(3, 3)
    out = np.zeros((16, 4), np.float32)
    n = lib.oracle_clip(_p(m, ctypes.c_float), _p(t, ctypes.c_float), _p(out, ctypes.c_float))
    return out[:n].copy()
