"""MI355X-native batch renderer for large-batch simulation (arXiv 2103.07013, Sec. 3.2).

Thin ctypes binding over libbps.so, the C-ABI library declared in include/bps.h.  Every
step of rendering runs in the library's HIP kernels; this module only marshals arguments.
PyTorch is used for device memory and streams.  There is no CPU fallback: if the library
is missing or no GPU is present, calls raise.
"""
from .binding import (BpsError, Renderer, bps_create, bps_destroy, bps_last_error, bps_last_kernel_ms, bps_kernel_ms_total, bps_kernel_ms_each, bps_set_diagnostics, bps_read_diagnostics,
                      bps_load_scene, bps_load_scene_async, bps_load_scene_textured, bps_scene_ready, bps_pack_clusters, bps_query, bps_render, bps_render_static, bps_set_profiling, bps_unload_scene, load_library,
                      MODE_DEPTH, MODE_RGBD, FLAG_NO_CLUSTER_CULL, FLAG_NO_OCCLUSION_CULL, FLAG_NO_DISPATCH_ORDER, FLAG_INPUTS_READY, FLAG_BILINEAR, EXPORTS)

__all__ = ["BpsError", "Renderer", "bps_create", "bps_destroy", "bps_last_error", "bps_last_kernel_ms", "bps_kernel_ms_total", "bps_kernel_ms_each", "bps_set_diagnostics", "bps_read_diagnostics",
           "bps_load_scene", "bps_load_scene_async", "bps_load_scene_textured", "bps_scene_ready", "bps_pack_clusters", "bps_query", "bps_render", "bps_render_static", "bps_set_profiling", "bps_unload_scene", "load_library",
           "MODE_DEPTH", "MODE_RGBD", "FLAG_NO_CLUSTER_CULL", "FLAG_NO_OCCLUSION_CULL", "FLAG_NO_DISPATCH_ORDER", "FLAG_INPUTS_READY", "FLAG_BILINEAR", "EXPORTS"]
