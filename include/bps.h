/*
 * bps.h -- C ABI of the batch renderer for large-batch simulation on AMD MI355X (gfx950).
 *
 * The operation (paper Sec. 3, Fig. 2, Sec. 3.2 "Batch Rendering"): a batch of N environment
 * states goes in as ONE request, N low-resolution frames come out in GPU memory; the K << N
 * scene assets are uploaded once and every environment refers to one of them by id
 * (Sec. 3.2 "Scene asset sharing").  Here an environment state is a scene handle plus a 4x4
 * view-projection matrix and a frame is H x W float32 eye depth (optionally RGB-D).
 *
 * The paper leaves rasterisation to the graphics API; this library fixes the rule:
 *   clip = M * (x, y, z, 1)^T with M row-major, normalised x right, y DOWN, z in [0,1];
 *   triangles are clipped against the six planes |x| <= w, |y| <= w, 0 <= z <= w;
 *   screen positions are snapped to 1/256 pixel; a pixel belongs to a triangle when its centre
 *   passes the three integer edge tests under the top-left fill rule (two-sided, no culling by
 *   winding); depth is perspective-correct clip-space w; the frame keeps, per pixel, the
 *   minimum of (depth bits << 32 | triangle id), i.e. nearest surface, ties to the lower id.
 *
 * All functions return a status; none throws or aborts.  Unless stated otherwise pointers are
 * HOST memory.  bps_render, the scene calls and bps_scene_ready may be called from different
 * threads (typically one render thread and one loader thread; the library serialises its
 * bookkeeping and keeps the long host-side part of a load outside the lock); everything else
 * must not overlap other calls on the same renderer.  Different renderers are independent.
 * There is no CPU fallback: without a usable GPU bps_create fails.
 */
#ifndef BPS_H
#define BPS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bps_renderer bps_renderer; /* opaque; bound to one device and one frame format */
typedef int32_t bps_scene;                /* handle >= 0; names one load: after bps_unload_scene it stays invalid even
                                             when the library reuses its table slot for a later scene */
typedef int32_t bps_status;

enum {
    BPS_OK = 0,
    BPS_ERR_INVALID_ARG = -1,     /* null pointer, zero size, bad resolution, index out of range ... */
    BPS_ERR_BAD_HANDLE = -2,      /* scene handle not live in this renderer */
    BPS_ERR_OOM = -3,             /* host or device allocation failed */
    BPS_ERR_HIP = -4,             /* a HIP runtime call failed; text in bps_last_error */
    BPS_ERR_UNSUPPORTED = -5      /* frame does not fit the on-chip visibility buffer of this device */
};

enum { BPS_MODE_DEPTH = 0, BPS_MODE_RGBD = 1 };

/* bps_config.flags.  Cluster culling is the paper's frustum culling of geometry chunks
 * (Sec. 3.2 "Pipelined geometry culling"); it never changes a frame, only the work done. */
enum {
    BPS_FLAG_NO_CLUSTER_CULL = 1,   /* stream every cluster of the scene for every environment */
    BPS_FLAG_NO_OCCLUSION_CULL = 2, /* frustum culling only: do not skip clusters hidden behind nearer geometry */
    BPS_FLAG_NO_DISPATCH_ORDER = 4, /* launch work-groups in batch order instead of costliest first */
    BPS_FLAG_INPUTS_READY = 8       /* the caller vouches that device-resident view_proj arrays are complete
                                       when bps_render is called (no pending work on any stream still writes
                                       them): staging and launch planning may then start at once, on a stream
                                       of the renderer, instead of queuing behind the caller's stream.  Host
                                       arrays are consumed during the call and always get this treatment. */
    ,
    BPS_FLAG_BILINEAR = 16          /* textured scenes: blend the four texels around the sample position
                                       (see bps_load_scene_textured) instead of taking the nearest one */
};

typedef struct {
    int32_t device;          /* HIP device ordinal */
    int32_t max_batch;       /* largest B accepted by bps_render (>= 1) */
    int32_t height, width;   /* output frame size; multiples of 8, 8..128 */
    int32_t mode;            /* BPS_MODE_DEPTH or BPS_MODE_RGBD */
    float background_depth;  /* written where no triangle covers the pixel centre */
    int32_t splits;          /* work-groups per environment; 0 = choose from B and the device */
    int32_t threads;         /* work-group size: 0 = default, else 256, 384, 512 or 1024 */
    uint32_t flags;          /* BPS_FLAG_* bits, 0 = defaults */
    int32_t supersample;     /* 0 or 1 = off; 2 = render at 2 height x 2 width and average 2x2 blocks into the
                                output (depth: ((a+b)+(c+d))/4 in float32; colour: (a+b+c+d+2)>>2); then
                                2 height and 2 width must be <= 128 and out_tri_id must be NULL */
} bps_config;

/* Create a renderer on cfg->device (Sec. 3.2: the renderer is set up once and then serves one batched
 * request per simulation step; its frame size is the policy's input resolution, Sec. 4.1).  *out
 * receives the handle.  Allocates the device scene table, the events of the request staging ring
 * and (lazily, in the first requests that need them) the staging buffers, the global visibility
 * buffer used when an environment is split over several work-groups, and the colour pass's buffers. */
bps_status bps_create(const bps_config *cfg, bps_renderer **out);

/* Waits for the device, frees every scene and buffer.  NULL is ignored. */
void bps_destroy(bps_renderer *r);

/* Scene asset upload (Sec. 3.2 "Scene asset sharing": K unique assets resident in GPU memory,
 * referenced by many environments).
 *   vertices  float32 [V][3]  world positions
 *   indices   uint32  [T][3]  vertex indices; triangle id = row number
 *   colors    uint8   [V][3]  per-vertex RGB or NULL (required for RGB-D rendering)
 * The mesh is validated (every index < V, every coordinate finite), re-packed on the host into
 * clusters of <= 64 vertices / <= 128 triangles, and copied to the device; the caller may free
 * its arrays on return.  Synchronous.  *out_handle receives the scene id. */
bps_status bps_load_scene(bps_renderer *r, const float *vertices, uint32_t V, const uint32_t *indices, uint32_t T,
                          const uint8_t *colors, bps_scene *out_handle);

/* Asynchronous scene upload (Sec. 3.2: new scenes are streamed into GPU memory while rollouts
 * and learning continue, and scenes no longer referenced are dropped).  Same arguments and
 * host-side work (validation, re-packing into a pinned image) as bps_load_scene, but the copy to
 * the device is only enqueued on `copy_stream` (a hipStream_t other than the render stream) and the
 * call returns without waiting; the caller's arrays may be freed on return.  The handle may be
 * passed to bps_render at once: a request that references a scene still in flight is ordered
 * after its copy on the device, the host never blocks.  bps_scene_ready reports (without
 * waiting) whether the copy has finished. */
bps_status bps_load_scene_async(bps_renderer *r, const float *vertices, uint32_t V, const uint32_t *indices,
                                uint32_t T, const uint8_t *colors, void *copy_stream, bps_scene *out_handle);
bps_status bps_scene_ready(bps_renderer *r, bps_scene scene, int32_t *ready);

/* Textured scene (the paper's RGB sensor renders textured scans, Sec. 4.1).  As bps_load_scene,
 * with per-vertex texture coordinates and one RGB8 texture per scene instead of vertex colours:
 *   uvs     float32 [V][2]              texture coordinates, any range (the texture repeats)
 *   texels  uint8   [tex_h][tex_w][3]   tex_w, tex_h powers of two up to 4096
 * In RGB-D mode a pixel then shows one texel, chosen as follows: (u, v) are interpolated
 * perspective-correctly like colours; the library builds a mip pyramid (each level halves both
 * sides, a texel is (a+b+c+d+2)>>2 of its 2x2 parents); each rasterised triangle uses the level
 * at which one pixel covers fewer than four texels (from its uv area and pixel area); the texel
 * is the one containing (u - floor u, v - floor v).  With BPS_FLAG_BILINEAR the four texels of
 * that level around the sample position are blended instead: x = fu lw - 0.5, x0 = floor x,
 * tx = x - x0, texels x0 and x0 + 1 wrapped around the texture's sides (likewise y), per channel
 * top = fma(tx, c01 - c00, c00), bot = fma(tx, c11 - c10, c10), out = rint(fma(ty, bot - top, top))
 * in float32, so colours stay reproducible bit for bit.  copy_stream NULL = wait for the upload,
 * otherwise the copy is only enqueued there (see bps_load_scene_async). */
bps_status bps_load_scene_textured(bps_renderer *r, const float *vertices, uint32_t V, const uint32_t *indices,
                                   uint32_t T, const float *uvs, const uint8_t *texels, uint32_t tex_w,
                                   uint32_t tex_h, void *copy_stream, bps_scene *out_handle);

/* Host-only helper (no GPU needed): re-pack a mesh exactly as bps_load_scene does and copy the
 * cluster arrays out, for tests and tools.  On entry *count is the capacity of the output
 * arrays in clusters (ignored when all three are NULL); on return it is the cluster count.
 *   verts_out [count][3][64] float32   x, y, z planes; unused lanes repeat the first vertex
 *   tris_out  [count][128]   uint32    i0 | i1 << 8 | i2 << 16, used-slot count in bits 24..31 of word 0
 *   ids_out   [count][128]   uint32    row in `indices`, 0xFFFFFFFF for unused slots */
bps_status bps_pack_clusters(const float *vertices, uint32_t V, const uint32_t *indices, uint32_t T, uint32_t *count,
                             float *verts_out, uint32_t *tris_out, uint32_t *ids_out);

/* Retires a scene (Sec. 3.2 "Scene asset sharing": the K resident assets are rotated, a scene that
 * no environment uses any more makes room for the next one).  Safe while requests that reference
 * it are still queued, and while its own asynchronous upload is still in flight: its device block and
 * table slot are only reused after those have finished.  Never waits for the device.  The handle is
 * invalid for new requests from this call on (BPS_ERR_BAD_HANDLE), also after its slot has been reused. */
bps_status bps_unload_scene(bps_renderer *r, bps_scene scene);

/* One batched render request (Sec. 3: the whole batch of N environment states is rendered at
 * once and the N frames are left in GPU memory for the consumer).
 *   scene_ids   host   int32 [B]          scene of each environment
 *   view_proj   host or device float32 [B][4][4], row-major
 *   out_depth   DEVICE float32 [B][H][W]  eye depth, background_depth where nothing is hit
 *   out_rgb     DEVICE uint8 [B][H][W][3] or NULL; required in RGB-D mode
 *   out_tri_id  DEVICE uint32 [B][H][W] or NULL; winning triangle id, 0xFFFFFFFF = none
 *   stream      hipStream_t (NULL = default stream)
 * Only enqueues work on `stream` and returns; host arrays are consumed before return, output
 * buffers must stay alive until the stream reaches the end of the request.  The one host wait: at
 * most four requests of a renderer are in flight; a fifth call waits for the oldest to finish
 * (its staging slot is reused).
 * Requests on one stream run in order.  Requests on different streams may overlap on the device
 * (two requests in flight fill the compute units that the end of a launch leaves idle); the library
 * itself orders those that use its internal buffers (RGB-D requests, split frames,
 * supersampling, diagnostics). */
bps_status bps_render(bps_renderer *r, const bps_scene *scene_ids, const float *view_proj, uint32_t B,
                      float *out_depth, uint8_t *out_rgb, uint32_t *out_tri_id, void *stream);

/* bps_render for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  It calls no hipMalloc / hipFree / hipHostMalloc and copies nothing
 * from host memory: the work items travel as kernel arguments, and the launch plan (work items, work
 * items in launch order, cost words) lives in a file-scope __device__ array of the library, 576 KiB on every GPU the
 * library runs on, held until the process ends.  Same frames as bps_render, bit for bit.
 * Limits: depth renderers without supersampling, forced splits or diagnostics; view_proj must be
 * DEVICE memory; B x (64x64-pixel tiles per frame) <= 16384 work-groups (e.g. 16384 environments at
 * 64x64, 4096 at 128x128), otherwise BPS_ERR_INVALID_ARG / BPS_ERR_UNSUPPORTED and nothing is enqueued.
 * One environment is never split over several work-groups here, so very small batches run slower
 * than through bps_render.  scene_ids is host memory as in bps_render.
 * Every call on a GPU, from any renderer and stream, uses that GPU's one array: calls on one stream
 * are ordered and safe; calls that overlap on one GPU (different streams or renderers) race.  Nothing
 * in the array needs clearing: each call overwrites what it reads. */
bps_status bps_render_static(bps_renderer *r, const bps_scene *scene_ids, const float *view_proj, uint32_t B,
                             float *out_depth, uint32_t *out_tri_id, void *stream);

/* Timing aid for benchmarks: when enabled, bps_render brackets its raster kernel (the one launch
 * of k_raster) with HIP events on the caller's stream; request staging, the two planning kernels
 * and the resolve / colour / downsample kernels are outside the bracket.  enable = 1 times every
 * request, enable = n > 1 every n-th one (the first, the (n+1)-th, ...: the events themselves cost a
 * few microseconds per request), 0 switches it off.
 * bps_last_kernel_ms waits for the most recent request's events and returns its duration in
 * milliseconds.  bps_kernel_ms_total waits for every request profiled since the last call (or
 * since profiling was enabled; at most 4096 are remembered), returns their count and summed
 * duration, and forgets them.  bps_kernel_ms_each does the same but writes the individual
 * durations (at most `capacity`, oldest first) to the host array `out` and their count to *written. */
bps_status bps_set_profiling(bps_renderer *r, int32_t enable);
bps_status bps_last_kernel_ms(bps_renderer *r, float *ms);
bps_status bps_kernel_ms_total(bps_renderer *r, uint32_t *launches, float *total_ms);
bps_status bps_kernel_ms_each(bps_renderer *r, float *out, uint32_t capacity, uint32_t *written);

/* Diagnostics: when enabled (1), the raster kernel tallies its work into a device block that
 * bps_read_diagnostics copies out after waiting for the device: 16 words per work-group g,
 *   out[16 g + 0] clusters whose bounds were tested      [1] clusters that passed the bounds tests
 *   [2] clusters that reached the triangle phase           [3] triangles sent to the clipper
 *   [4] clusters skipped because nearer geometry already covered their footprint
 *   [5] run time of the group's slowest wavefront in 100 MHz ticks
 *   [6] small triangles queued for per-lane rasterisation   [7] large triangles rasterised by a wavefront
 *   [8] clusters rejected against the coarse depth tiles before being queued
 *   [9..15] with enable = 2 only (this slows the kernel): time summed over the group's wavefronts
 *           in the bounds testing, barrier, depth sort, prologue (set-up and block ordering),
 *           cluster processing, barrier and final flush phases.
 *           with enable = 3: how often each path ran, summed over the wavefronts: drains of the
 *           small-triangle queue, their pixel steps, the steps in which some pixel was covered, calls that
 *           handed triangles on, passes over medium triangles, 8x8 steps of large ones, appends to the queue.
 *           with enable = 4: clipper runs, their plane passes, fan steps, occlusion-test passes when
 *           clusters are taken off the list, passes over 64 triangles, clusters taken off the list,
 *           passes of the bounds tests.
 *   with enable = 1 instead: [11] environment index, [12] run times of all the group's wavefronts
 *           summed, [13] start and [14] end of the group on the device-wide 100 MHz clock (low 32
 *           bits), [15] hardware id of the compute unit that ran it (die in the top byte).
 * `capacity` is the room in `out` (in words), *written the number of words copied. */
bps_status bps_set_diagnostics(bps_renderer *r, int32_t enable);
bps_status bps_read_diagnostics(bps_renderer *r, uint64_t *out, uint32_t capacity, uint32_t *written);

/* Facts about a loaded scene and the launch plan, for benchmarks and tests.
 * what: 0 = clusters in the scene, 1 = triangles, 2 = vertices, 3 = device bytes held,
 *       4 = splits used by the last request, 5 = work-groups of the last request,
 *       6 = work-group size, 7 = LDS bytes per work-group, 8 = device blocks allocated for scenes so
 *       far, 9 = retired scene blocks waiting for reuse. */
bps_status bps_query(bps_renderer *r, bps_scene scene, int32_t what, uint64_t *value);

/* Text of the last error on this renderer (owned by the renderer; never NULL).
 * With r == NULL returns the text of the last failed bps_create on this thread. */
const char *bps_last_error(const bps_renderer *r);

#ifdef __cplusplus
}
#endif
#endif /* BPS_H */
