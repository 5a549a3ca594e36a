"""ctypes binding with the same names as the C ABI (include/bps.h).  Marshalling only."""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

MODE_DEPTH, MODE_RGBD = 0, 1
FLAG_NO_CLUSTER_CULL = 1
FLAG_NO_OCCLUSION_CULL = 2
FLAG_NO_DISPATCH_ORDER = 4
FLAG_INPUTS_READY = 8
FLAG_BILINEAR = 16
EXPORTS = ["bps_create", "bps_destroy", "bps_load_scene", "bps_load_scene_async", "bps_load_scene_textured", "bps_scene_ready", "bps_pack_clusters", "bps_unload_scene", "bps_render", "bps_render_static", "bps_set_profiling",
           "bps_last_kernel_ms", "bps_kernel_ms_total", "bps_kernel_ms_each", "bps_set_diagnostics", "bps_read_diagnostics", "bps_query", "bps_last_error"]


class BpsError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"bps status {status}: {text}")
        self.status = status


class bps_config(ctypes.Structure):
    _fields_ = [("device", ctypes.c_int32), ("max_batch", ctypes.c_int32), ("height", ctypes.c_int32),
                ("width", ctypes.c_int32), ("mode", ctypes.c_int32), ("background_depth", ctypes.c_float),
                ("splits", ctypes.c_int32), ("threads", ctypes.c_int32), ("flags", ctypes.c_uint32), ("supersample", ctypes.c_int32)]


_lib = None


def load_library():
    """Load libbps.so, building it first only if no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build(force=True)
    lib = ctypes.CDLL(_build.LIB)
    vp = ctypes.c_void_p
    lib.bps_create.restype = ctypes.c_int32
    lib.bps_create.argtypes = [ctypes.POINTER(bps_config), ctypes.POINTER(vp)]
    lib.bps_destroy.restype = None
    lib.bps_destroy.argtypes = [vp]
    lib.bps_load_scene.restype = ctypes.c_int32
    lib.bps_load_scene.argtypes = [vp, vp, ctypes.c_uint32, vp, ctypes.c_uint32, vp, ctypes.POINTER(ctypes.c_int32)]
    lib.bps_load_scene_async.restype = ctypes.c_int32
    lib.bps_load_scene_async.argtypes = [vp, vp, ctypes.c_uint32, vp, ctypes.c_uint32, vp, vp, ctypes.POINTER(ctypes.c_int32)]
    lib.bps_load_scene_textured.restype = ctypes.c_int32
    lib.bps_load_scene_textured.argtypes = [vp, vp, ctypes.c_uint32, vp, ctypes.c_uint32, vp, vp, ctypes.c_uint32,
                                            ctypes.c_uint32, vp, ctypes.POINTER(ctypes.c_int32)]
    lib.bps_scene_ready.restype = ctypes.c_int32
    lib.bps_scene_ready.argtypes = [vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    lib.bps_pack_clusters.restype = ctypes.c_int32
    lib.bps_pack_clusters.argtypes = [vp, ctypes.c_uint32, vp, ctypes.c_uint32, ctypes.POINTER(ctypes.c_uint32), vp, vp, vp]
    lib.bps_unload_scene.restype = ctypes.c_int32
    lib.bps_unload_scene.argtypes = [vp, ctypes.c_int32]
    lib.bps_render.restype = ctypes.c_int32
    lib.bps_render.argtypes = [vp, vp, vp, ctypes.c_uint32, vp, vp, vp, vp]
    lib.bps_render_static.restype = ctypes.c_int32
    lib.bps_render_static.argtypes = [vp, vp, vp, ctypes.c_uint32, vp, vp, vp]
    lib.bps_set_profiling.restype = ctypes.c_int32
    lib.bps_set_profiling.argtypes = [vp, ctypes.c_int32]
    lib.bps_last_kernel_ms.restype = ctypes.c_int32
    lib.bps_last_kernel_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
    lib.bps_kernel_ms_each.restype = ctypes.c_int32
    lib.bps_kernel_ms_each.argtypes = [vp, vp, ctypes.c_uint32, ctypes.POINTER(ctypes.c_uint32)]
    lib.bps_kernel_ms_total.restype = ctypes.c_int32
    lib.bps_kernel_ms_total.argtypes = [vp, ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(ctypes.c_float)]
    lib.bps_set_diagnostics.restype = ctypes.c_int32
    lib.bps_set_diagnostics.argtypes = [vp, ctypes.c_int32]
    lib.bps_read_diagnostics.restype = ctypes.c_int32
    lib.bps_read_diagnostics.argtypes = [vp, vp, ctypes.c_uint32, ctypes.POINTER(ctypes.c_uint32)]
    lib.bps_query.restype = ctypes.c_int32
    lib.bps_query.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_uint64)]
    lib.bps_last_error.restype = ctypes.c_char_p
    lib.bps_last_error.argtypes = [vp]
    _lib = lib
    return lib


def bps_last_error(handle=None):
    return load_library().bps_last_error(handle).decode()


def _check(status, handle):
    if status != 0:
        raise BpsError(status, bps_last_error(handle))


def bps_create(device=0, max_batch=1024, height=64, width=64, mode=MODE_DEPTH, background_depth=0.0, splits=0,
               threads=0, flags=0, supersample=0):
    lib = load_library()
    cfg = bps_config(device, max_batch, height, width, mode, background_depth, splits, threads, flags, supersample)
    h = ctypes.c_void_p()
    _check(lib.bps_create(ctypes.byref(cfg), ctypes.byref(h)), None)
    return h


def bps_destroy(handle):
    load_library().bps_destroy(handle)


def bps_load_scene(handle, vertices, indices, colors=None):
    """vertices float32 [V,3], indices uint32 [T,3], colors uint8 [V,3] | None (host arrays)."""
    lib = load_library()
    v = np.ascontiguousarray(vertices, np.float32).reshape(-1, 3)
    i = np.ascontiguousarray(indices, np.uint32).reshape(-1, 3)
    c = None if colors is None else np.ascontiguousarray(colors, np.uint8).reshape(-1, 3)
    if c is not None and c.shape[0] != v.shape[0]:
        raise ValueError("colors must have one row per vertex")
    out = ctypes.c_int32(-1)
    _check(lib.bps_load_scene(handle, v.ctypes.data, v.shape[0], i.ctypes.data, i.shape[0],
                              None if c is None else c.ctypes.data, ctypes.byref(out)), handle)
    return int(out.value)


def bps_load_scene_async(handle, vertices, indices, colors=None, copy_stream=None):
    """Like bps_load_scene but only enqueues the device copy on copy_stream (torch stream or raw handle)."""
    lib = load_library()
    v = np.ascontiguousarray(vertices, np.float32).reshape(-1, 3)
    i = np.ascontiguousarray(indices, np.uint32).reshape(-1, 3)
    c = None if colors is None else np.ascontiguousarray(colors, np.uint8).reshape(-1, 3)
    s = copy_stream if isinstance(copy_stream, int) or copy_stream is None else copy_stream.cuda_stream
    out = ctypes.c_int32(-1)
    _check(lib.bps_load_scene_async(handle, v.ctypes.data, v.shape[0], i.ctypes.data, i.shape[0],
                                    None if c is None else c.ctypes.data, ctypes.c_void_p(s or 0), ctypes.byref(out)), handle)
    return int(out.value)


def bps_load_scene_textured(handle, vertices, indices, uvs, texture, copy_stream=None):
    """vertices f32 [V,3], indices u32 [T,3], uvs f32 [V,2], texture u8 [h,w,3] with power-of-two sides."""
    lib = load_library()
    v = np.ascontiguousarray(vertices, np.float32).reshape(-1, 3)
    i = np.ascontiguousarray(indices, np.uint32).reshape(-1, 3)
    uv = np.ascontiguousarray(uvs, np.float32).reshape(-1, 2)
    tex = np.ascontiguousarray(texture, np.uint8)
    if uv.shape[0] != v.shape[0] or tex.ndim != 3 or tex.shape[2] != 3:
        raise ValueError("uvs must have one row per vertex and texture must be [h,w,3]")
    s = copy_stream if isinstance(copy_stream, int) or copy_stream is None else copy_stream.cuda_stream
    out = ctypes.c_int32(-1)
    _check(lib.bps_load_scene_textured(handle, v.ctypes.data, v.shape[0], i.ctypes.data, i.shape[0], uv.ctypes.data,
                                       tex.ctypes.data, tex.shape[1], tex.shape[0], ctypes.c_void_p(s or 0),
                                       ctypes.byref(out)), handle)
    return int(out.value)


def bps_scene_ready(handle, scene):
    flag = ctypes.c_int32(0)
    _check(load_library().bps_scene_ready(handle, int(scene), ctypes.byref(flag)), handle)
    return bool(flag.value)


def bps_pack_clusters(vertices, indices):
    """Host-only: (verts [C,3,64] f32, tris [C,128] u32, ids [C,128] u32) as bps_load_scene would upload."""
    lib = load_library()
    v = np.ascontiguousarray(vertices, np.float32).reshape(-1, 3)
    i = np.ascontiguousarray(indices, np.uint32).reshape(-1, 3)
    n = ctypes.c_uint32(0)
    st = lib.bps_pack_clusters(v.ctypes.data, v.shape[0], i.ctypes.data, i.shape[0], ctypes.byref(n), None, None, None)
    if st != 0:
        raise BpsError(st, "bps_pack_clusters rejected the mesh")
    C = int(n.value)
    verts = np.empty((C, 3, 64), np.float32)
    tris = np.empty((C, 128), np.uint32)
    ids = np.empty((C, 128), np.uint32)
    st = lib.bps_pack_clusters(v.ctypes.data, v.shape[0], i.ctypes.data, i.shape[0], ctypes.byref(n),
                               verts.ctypes.data, tris.ctypes.data, ids.ctypes.data)
    if st != 0:
        raise BpsError(st, "bps_pack_clusters failed")
    return verts, tris, ids


def bps_unload_scene(handle, scene):
    _check(load_library().bps_unload_scene(handle, int(scene)), handle)


def bps_render(handle, scene_ids, view_proj, out_depth, out_rgb=None, out_tri_id=None, stream=None):
    """scene_ids: host int32 [B]; view_proj: numpy float32 [B,4,4] or a CUDA torch tensor;
    out_*: CUDA torch tensors (depth float32 [B,H,W], rgb uint8 [B,H,W,3], tri_id int32/uint32 [B,H,W]);
    stream: a torch.cuda.Stream, a raw hipStream_t integer, or None for torch's current stream."""
    import torch
    lib = load_library()
    ids = np.ascontiguousarray(scene_ids, np.int32).reshape(-1)
    B = ids.shape[0]
    keep = None
    if isinstance(view_proj, torch.Tensor):
        if view_proj.dtype != torch.float32 or not view_proj.is_contiguous() or view_proj.numel() != B * 16:
            raise ValueError("view_proj tensor must be contiguous float32 [B,4,4]")
        vp_ptr = view_proj.data_ptr()
    else:
        keep = np.ascontiguousarray(view_proj, np.float32).reshape(B, 4, 4)
        vp_ptr = keep.ctypes.data

    def dev_ptr(t, dtype_ok, numel, name):
        if t is None:
            return None
        if not t.is_cuda or not t.is_contiguous() or t.dtype not in dtype_ok or t.numel() != numel:
            raise ValueError(f"{name}: need a contiguous CUDA tensor of {numel} elements, dtype in {dtype_ok}")
        return t.data_ptr()

    hw = out_depth.shape[-2] * out_depth.shape[-1] if out_depth is not None and out_depth.dim() >= 2 else 0
    d_ptr = dev_ptr(out_depth, (torch.float32,), B * hw, "out_depth")
    rgb_ptr = dev_ptr(out_rgb, (torch.uint8,), B * hw * 3, "out_rgb")
    id_ptr = dev_ptr(out_tri_id, (torch.int32, torch.uint32), B * hw, "out_tri_id")
    if stream is None:
        s = torch.cuda.current_stream(out_depth.device).cuda_stream
    elif isinstance(stream, int):
        s = stream
    else:
        s = stream.cuda_stream
    _check(lib.bps_render(handle, ids.ctypes.data, vp_ptr, B, d_ptr, rgb_ptr, id_ptr, ctypes.c_void_p(s)), handle)


def bps_render_static(handle, scene_ids, view_proj, out_depth, out_tri_id=None, stream=None):
    """bps_render without any allocation: scene_ids host int32 [B]; view_proj a CUDA float32 tensor [B,4,4];
    out_depth / out_tri_id CUDA tensors [B,H,W]; stream as in bps_render."""
    import torch
    lib = load_library()
    ids = np.ascontiguousarray(scene_ids, np.int32).reshape(-1)
    B = ids.shape[0]
    if not isinstance(view_proj, torch.Tensor) or not view_proj.is_cuda or view_proj.dtype != torch.float32 or \
            not view_proj.is_contiguous() or view_proj.numel() != B * 16:
        raise ValueError("view_proj must be a contiguous CUDA float32 tensor [B,4,4]")
    hw = out_depth.shape[-2] * out_depth.shape[-1]
    for t, ok, name in ((out_depth, (torch.float32,), "out_depth"), (out_tri_id, (torch.int32, torch.uint32), "out_tri_id")):
        if t is not None and (not t.is_cuda or not t.is_contiguous() or t.dtype not in ok or t.numel() != B * hw):
            raise ValueError(f"{name}: need a contiguous CUDA tensor of {B * hw} elements, dtype in {ok}")
    if stream is None:
        s = torch.cuda.current_stream(out_depth.device).cuda_stream
    elif isinstance(stream, int):
        s = stream
    else:
        s = stream.cuda_stream
    _check(lib.bps_render_static(handle, ids.ctypes.data, view_proj.data_ptr(), B, out_depth.data_ptr(),
                                 None if out_tri_id is None else out_tri_id.data_ptr(), ctypes.c_void_p(s)), handle)


def bps_set_profiling(handle, enable=True):
    """enable: False / 0 = off, True / 1 = time every request, n > 1 = time every n-th request."""
    _check(load_library().bps_set_profiling(handle, int(enable)), handle)


def bps_last_kernel_ms(handle):
    ms = ctypes.c_float(0.0)
    _check(load_library().bps_last_kernel_ms(handle, ctypes.byref(ms)), handle)
    return float(ms.value)


def bps_kernel_ms_each(handle, capacity=4096):
    """Durations (ms) of the requests profiled since the last call, oldest first, as a float32 array."""
    out = np.zeros(capacity, np.float32)
    n = ctypes.c_uint32(0)
    _check(load_library().bps_kernel_ms_each(handle, out.ctypes.data, capacity, ctypes.byref(n)), handle)
    return out[:int(n.value)].copy()


def bps_kernel_ms_total(handle):
    """(launches, total_ms) of every request profiled since the previous call."""
    n, ms = ctypes.c_uint32(0), ctypes.c_float(0.0)
    _check(load_library().bps_kernel_ms_total(handle, ctypes.byref(n), ctypes.byref(ms)), handle)
    return int(n.value), float(ms.value)


def bps_set_diagnostics(handle, enable=1):
    _check(load_library().bps_set_diagnostics(handle, int(enable)), handle)


def bps_read_diagnostics(handle, capacity=1 << 16):
    """uint64 array: 8 counters then one duration per work-group (see include/bps.h)."""
    out = np.zeros(capacity, np.uint64)
    n = ctypes.c_uint32(0)
    _check(load_library().bps_read_diagnostics(handle, out.ctypes.data, capacity, ctypes.byref(n)), handle)
    return out[:int(n.value)]


def bps_query(handle, scene, what):
    v = ctypes.c_uint64(0)
    _check(load_library().bps_query(handle, int(scene), int(what), ctypes.byref(v)), handle)
    return int(v.value)


class Renderer:
    """Convenience owner of one bps_renderer handle (same calls, object style)."""

    def __init__(self, max_batch, height=64, width=64, mode=MODE_DEPTH, device=0, background_depth=0.0, splits=0,
                 threads=0, flags=0, supersample=0):
        self.H, self.W, self.mode, self.device = height, width, mode, device
        self.handle = bps_create(device, max_batch, height, width, mode, background_depth, splits, threads, flags,
                                 supersample)

    def load_scene(self, vertices, indices, colors=None):
        return bps_load_scene(self.handle, vertices, indices, colors)

    def load_scene_textured(self, vertices, indices, uvs, texture, copy_stream=None):
        return bps_load_scene_textured(self.handle, vertices, indices, uvs, texture, copy_stream)

    def load_scene_async(self, vertices, indices, colors=None, copy_stream=None):
        return bps_load_scene_async(self.handle, vertices, indices, colors, copy_stream)

    def unload_scene(self, scene):
        bps_unload_scene(self.handle, scene)

    def render(self, scene_ids, view_proj, out_depth=None, out_rgb=None, out_tri_id=None, want_tri_id=False,
               stream=None):
        import torch
        B = len(scene_ids)
        dev = torch.device("cuda", self.device)
        if out_depth is None:
            out_depth = torch.empty((B, self.H, self.W), dtype=torch.float32, device=dev)
        if out_rgb is None and self.mode == MODE_RGBD:
            out_rgb = torch.empty((B, self.H, self.W, 3), dtype=torch.uint8, device=dev)
        if out_tri_id is None and want_tri_id:
            out_tri_id = torch.empty((B, self.H, self.W), dtype=torch.int32, device=dev)
        bps_render(self.handle, scene_ids, view_proj, out_depth, out_rgb, out_tri_id, stream)
        return out_depth, out_rgb, out_tri_id

    def close(self):
        if self.handle is not None:
            bps_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
