// Device side of the batch renderer: one fused geometry + rasterisation kernel and a resolve
// kernel, written for gfx950 (64-lane wavefronts, 160 KB LDS per CU).
//
// One work-group renders (a slice of) one environment's frame (paper Sec. 3.2: every
// environment of the batch is drawn in a single request).  The frame's visibility buffer --
// H*W packed keys (depth bits << 32 | triangle id) -- lives in LDS for the whole kernel, so the
// z-test is a 64-bit LDS atomic min and the frame is written to HBM exactly once.  Each wavefront
// streams clusters of <= 64 vertices / <= 128 triangles:
//   vertex phase   one lane per vertex: clip = M v, six-plane outcodes, projection, 1/256-px snap
//   cluster cull   all 64 vertices outside one plane (wave ballot)  -> next cluster
//   triangle phase two triangles per lane: outcode reject, bounding box vs pixel centres
//   compaction     survivors are appended to LDS queues with ballot + prefix count so
//                  that the expensive steps run on full wavefronts:
//                    small queue  (per wavefront) triangles touching <= 12 pixel centres, one lane per triangle
//                    clip ring    (per work-group) triangles straddling a frustum plane, one lane per triangle
//                  large triangles are rasterised by the whole wavefront, 8x8 pixels at a time.
// All float arithmetic follows one fixed IEEE sequence (explicit fmaf, no contraction, exact
// division) so that coverage and ids are reproducible bit for bit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bps {

struct SceneDev {
    const float* cverts;       // [C][3][64] cluster vertex positions, x then y then z
    const uint32_t* ctris;     // [C][128]   packed local indices, count in bits 24..31 of word 0
    const uint32_t* ctri_id;   // [C][128]   original triangle row
    const float* cbounds;      // [6][c_stride] cluster bounds: min x, y, z then max x, y, z
    const float* bbounds;      // [6][b_stride] bounds of each block of 64 consecutive clusters
    const float* verts;        // [V][3]     original arrays, used when shading
    const uint32_t* indices;   // [T][3]
    const uint8_t* colors;     // [V][3] or null
    const float* uvs;          // [V][2] or null (textured scenes)
    const uint32_t* texels;    // RGBA8 mip pyramid, level after level, or null
    const float* tri_rec;      // [T][16]    per-triangle shading record (scenes with colours or a texture), or null:
                               //            x0 y0 z0 x1 y1 z1 x2 y2 z2, then three packed RGB words or u0 v0 u1 v1 u2 v2
    uint32_t tex_w, tex_h, tex_levels, pad2;
    uint32_t n_clusters, n_tris, n_verts, c_stride, b_stride, pad;
};

// One work-group's share: tile `tile` of environment `env`'s frame, and of its scene the
// 64-cluster blocks split, split + n_splits, split + 2 n_splits, ... (split_of = n_splits << 16 | split)
struct WorkItem {
    uint32_t env, scene, split_of, tile;
};

struct FrameParams {
    int32_t H, W;
    int32_t tile_w, tile_h; // a work-group owns one tile of the frame (the whole frame when it fits)
    float sx, sy;          // 128*W, 128*H
    float xmax, ymax;      // 2*sx + 64, 2*sy + 64
    float background;
    int32_t merge;         // 0: resolve straight to the output; 1: atomic-min into the global buffer
    int32_t cull;          // 0: stream every cluster; 1: frustum-cull clusters; 2: frustum + occlusion cull
    int32_t list_cap;      // capacity of the work-group's survivor list, in clusters
    int32_t round_target;  // survivors queued before a round's testing stops
    int32_t first_round;   // the same for an environment's first round (kept short when occlusion culling is on)
    int32_t phase_timers;  // diagnostics: 1 also time the kernel's phases (slows it down), 2 / 3 path tallies
    int32_t bilinear;      // colour pass: sample textures with bilinear filtering instead of the nearest texel
};

constexpr unsigned long long kEmptyKey = ~0ull;
constexpr int kOrigin = 16384;         // packed screen coordinates are stored relative to pixel 64
constexpr int kSmallMax = 12;          // pixel centres a "small" triangle may touch (one lane rasterises it)
constexpr uint32_t kInvalid = 0x40u;   // outcode bit: vertex unusable, drop its triangles
constexpr uint32_t kNoProject = 0x80u; // outcode bit: vertex has no finite screen position (w <= 0 or overflow)

// per-wave LDS block: 64 staged vertices (8 B + 4 B outcode each), small queue 8 x 64 words
constexpr uint32_t kListCap64 = 1216;   // survivor-list capacity of the 64x64 instance (two groups per compute unit)
constexpr uint32_t kWaveLdsBytes = 64 * 12 + 8 * 64 * 4;

// The work-group's ring of triangles waiting for the clipper.  A wavefront adds at most 128 entries
// between two looks at the ring and then drains it below 64, and at most 64 entries per wavefront are
// claimed but not yet read: never more than 64 + 192 per wavefront in use, so 256 per wavefront
// (rounded up to a power of two) cannot wrap onto a live entry.
__host__ __device__ constexpr uint32_t clip_ring_entries(int threads) {
    uint32_t need = 256u * (uint32_t)(threads / 64), n = 256u;
    while (n < need) n *= 2u;
    return n;
}

constexpr int kOrderCap = 1024;        // blocks of one item that can be depth-sorted
constexpr int kHizTiles = 64;          // 8x8-pixel tiles of a window of at most 64x64 pixels
constexpr int kDepthBins = 128;        // bins of the per-round depth sort of surviving clusters

// visibility buffer, per-wave blocks, survivor list (8 B record + two 2 B sort words per cluster),
// block order, depth histogram and its prefix, eight counters, clip ring
__host__ __device__ inline size_t lds_bytes(int tile_h, int tile_w, int threads, int list_cap) {
    return (size_t)tile_h * tile_w * 8 + (size_t)(threads / 64) * kWaveLdsBytes + (size_t)list_cap * 12 + kOrderCap * 2 +
           2 * kDepthBins * 4 + kHizTiles * 4 + 32 + (size_t)clip_ring_entries(threads) * 4;
}

// DIAG = true is the instance launched while diagnostics are on; it alone keeps counters and timers.
// CULL = FrameParams::cull of the launch (0 none, 1 frustum, 2 frustum + occlusion).
// FRAME = 64 or 128: the frame is square of that size and drawn as 64x64 windows; 0 = any frame.
template <int NT, bool DIAG, int CULL, int FRAME>
__global__ void k_raster(const SceneDev* __restrict__ scenes, const WorkItem* __restrict__ items,
                         const float* __restrict__ view_proj, FrameParams fp, unsigned long long* __restrict__ gvis,
                         float* __restrict__ out_depth, uint32_t* __restrict__ out_id,
                         unsigned long long* __restrict__ stats);

__global__ void k_resolve(unsigned long long* __restrict__ gvis, size_t n, float background,
                          float* __restrict__ out_depth, uint32_t* __restrict__ out_id);

__global__ void k_fill_keys(unsigned long long* __restrict__ gvis, size_t n);
__global__ void k_zero_words(unsigned long long* __restrict__ p, size_t n);

void launch_raster(int threads, dim3 grid, size_t lds, hipStream_t stream, const SceneDev* scenes, const WorkItem* items,
                   const float* view_proj, const FrameParams& fp, unsigned long long* gvis, float* out_depth,
                   uint32_t* out_id, unsigned long long* stats);
// Fills ordered[n_items] with the items in launch order, costliest first; cost is scratch, one word
// per item.
constexpr uint32_t kMaxPlannedItems = 16384;
void launch_plan(hipStream_t stream, const SceneDev* scenes, const WorkItem* items, const float* view_proj,
                 const FrameParams& fp, uint32_t n_items, uint32_t* cost, WorkItem* ordered);
hipError_t prepare_raster(int threads, size_t lds);
// Work items handed over as kernel arguments (no host-to-device copy, no staging memory): up to
// kPackedItemsPerLaunch items per launch, each packed as env | scene << 16 | tile << 28 (one
// work-group per environment and tile, i.e. split_of = 1 << 16).
constexpr uint32_t kPackedItemsPerLaunch = 960;
struct PackedItems {
    uint32_t word[kPackedItemsPerLaunch];
};
void launch_unpack_items(hipStream_t stream, const PackedItems& packed, uint32_t first, uint32_t count, WorkItem* items);
void launch_downsample(hipStream_t stream, const float* depth, const uint8_t* rgb, uint32_t B, int H, int W,
                       float* out_depth, uint8_t* out_rgb);
// Colour pass.  Pixels whose winning triangle needs the clipper go through kShadeQueues queues (work-group g
// of the first kernel appends to queue g % kShadeQueues); shade_queue_cap(pixels) words per queue hold the
// worst case.  queue: kShadeQueues * shade_queue_cap(pixels) words; count / next_count: this request's
// counters (32 * kShadeQueues words, all zero) and the next request's (cleared by the launch).
constexpr uint32_t kShadeQueues = 64;
inline uint32_t shade_queue_cap(size_t pixels) {
    const size_t groups = (pixels + 255) / 256;
    return (uint32_t)((groups + kShadeQueues - 1) / kShadeQueues * 256);
}
// Fills sc.tri_rec from the scene's original arrays (once per scene, on the stream that uploads it).
void launch_build_shade_records(hipStream_t stream, const SceneDev& sc, float* tri_rec);
void launch_shade(hipStream_t stream, const SceneDev* scenes, const uint32_t* env_scene, const float* view_proj,
                  const FrameParams& fp, uint32_t B, const uint32_t* tri_id, uint8_t* out_rgb, uint32_t* queue,
                  uint32_t* count, uint32_t* next_count);

}  // namespace bps
