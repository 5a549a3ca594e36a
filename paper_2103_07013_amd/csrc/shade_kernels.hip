// Colour resolve for RGB-D frames (stand-in for the paper's textured RGB sensor, Sec. 4.1):
// per-vertex uint8 colours, perspective-correct interpolation at the pixel centre of the
// triangle that won the z-test.  Runs after k_raster, one thread per pixel: the winner's
// three vertices are transformed, clipped and set up again with exactly the arithmetic of
// the raster kernel, so the barycentric weights are the ones the z-test used.
//   cn = fma(e2/w2, c2, fma(e1/w1, c1, (e0/w0) c0)),  out = clamp(rint(cn / num), 0, 255)
#include <algorithm>

#include "raster_device.h"
#include "raster_kernels.h"

namespace bps {
namespace {

using namespace dev;

struct CVert {
    Clip4 c;
    float r, g, b;
};

struct SVert {
    uint32_t xy;
    float iw, r, g, b;
};

// Field-by-field choice (choosing between whole objects goes through their addresses and would
// put both into private memory).
__device__ __forceinline__ CVert pick(bool first, const CVert& x, const CVert& y) {
    CVert o;
    o.c.x = first ? x.c.x : y.c.x; o.c.y = first ? x.c.y : y.c.y; o.c.z = first ? x.c.z : y.c.z; o.c.w = first ? x.c.w : y.c.w;
    o.r = first ? x.r : y.r; o.g = first ? x.g : y.g; o.b = first ? x.b : y.b;
    return o;
}

// Colour of pixel (i, j) from one snapped fan triangle; returns false when it does not cover the pixel.
__device__ __forceinline__ bool piece_colour(const SVert& v0, const SVert& v1, const SVert& v2, int i, int j,
                                             float& depth, float (&rgb)[3], float& uv_area2, int& area2) {
    Setup s = make_setup(v0.xy, v1.xy, v2.xy, v0.iw, v1.iw, v2.iw);
    if (s.A2 == 0) return false;
    // (values are selected one by one: choosing between two objects by reference would force both
    // into private memory)
    struct Attr { float r, g, b; };
    const Attr a = {v0.r, v0.g, v0.b};
    const Attr b = {s.swapped ? v2.r : v1.r, s.swapped ? v2.g : v1.g, s.swapped ? v2.b : v1.b};
    const Attr c = {s.swapped ? v1.r : v2.r, s.swapped ? v1.g : v2.g, s.swapped ? v1.b : v2.b};
    int px = (i << 8) + 128 - kOrigin, py = (j << 8) + 128 - kOrigin;
    int E0 = __mul24(s.dx0, py - s.Y1) - __mul24(s.dy0, px - s.X1);
    int E1 = __mul24(s.dx1, py - s.Y2) - __mul24(s.dy1, px - s.X2);
    int E2 = __mul24(s.dx2, py - s.Y0) - __mul24(s.dy2, px - s.X0);
    if (((E0 + s.b0) | (E1 + s.b1) | (E2 + s.b2)) < 0) return false;
    float e0 = (float)E0, e1 = (float)E1, e2 = (float)E2;
    float num = fmaf(e2, s.iw2, fmaf(e1, s.iw1, e0 * s.iw0));
    depth = (float)s.A2 / num;
    float w0 = e0 * s.iw0, w1 = e1 * s.iw1, w2 = e2 * s.iw2;
    rgb[0] = fmaf(w2, c.r, fmaf(w1, b.r, w0 * a.r)) / num;
    rgb[1] = fmaf(w2, c.g, fmaf(w1, b.g, w0 * a.g)) / num;
    rgb[2] = fmaf(w2, c.b, fmaf(w1, b.b, w0 * a.b)) / num;
    // for textured scenes slots r, g hold (u, v): twice the triangle's uv area over its pixel area
    float du1 = b.r - a.r, dv1 = b.g - a.g, du2 = c.r - a.r, dv2 = c.g - a.g;
    uv_area2 = fabsf(fmaf(du1, dv2, -(du2 * dv1)));
    area2 = s.A2;
    return true;
}

__device__ __forceinline__ uint8_t to_u8(float v) {
    if (!(v == v)) return 0;
    int q = __float2int_rn(fminf(fmaxf(v, -1.0f), 256.0f));
    return (uint8_t)min(max(q, 0), 255);
}

// Texel or interpolated colour of one covering fan piece (rgb holds (u, v, -) for textured scenes).
__device__ __forceinline__ void piece_output(const SceneDev& sc, bool textured, bool bilinear, const float (&rgb)[3],
                                             float uv_area2, int area2, uint8_t (&out)[3]) {
    if (textured) {
        // mip level: quarter the texels-per-pixel ratio while it is at least 4
        float ratio = ((uv_area2 * (float)sc.tex_w) * (float)sc.tex_h) * 65536.0f / (float)area2;
        uint32_t L = 0, lw = sc.tex_w, lh = sc.tex_h;
        size_t off = 0;
        while (L + 1 < sc.tex_levels && ratio >= 4.0f) {
            ratio *= 0.25f;
            off += (size_t)lw * lh;
            lw = lw > 1 ? lw / 2 : 1;
            lh = lh > 1 ? lh / 2 : 1;
            ++L;
        }
        float fu = rgb[0] - floorf(rgb[0]), fv = rgb[1] - floorf(rgb[1]);
        if (!(fu >= 0.0f && fu < 1.0f)) fu = 0.0f;
        if (!(fv >= 0.0f && fv < 1.0f)) fv = 0.0f;
        if (bilinear) {
            // the four texels around the sample position, wrapped around the texture's (power-of-two) sides
            const float x = fu * (float)lw - 0.5f, y = fv * (float)lh - 0.5f;
            const float fx0 = floorf(x), fy0 = floorf(y);
            const float tx = x - fx0, ty = y - fy0;
            const uint32_t x0 = (uint32_t)(int)fx0 & (lw - 1), x1 = (uint32_t)((int)fx0 + 1) & (lw - 1);
            const uint32_t y0 = (uint32_t)(int)fy0 & (lh - 1), y1 = (uint32_t)((int)fy0 + 1) & (lh - 1);
            const uint32_t t00 = sc.texels[off + (size_t)y0 * lw + x0], t01 = sc.texels[off + (size_t)y0 * lw + x1];
            const uint32_t t10 = sc.texels[off + (size_t)y1 * lw + x0], t11 = sc.texels[off + (size_t)y1 * lw + x1];
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                const float c00 = (float)((t00 >> (8 * c)) & 0xFFu), c01 = (float)((t01 >> (8 * c)) & 0xFFu);
                const float c10 = (float)((t10 >> (8 * c)) & 0xFFu), c11 = (float)((t11 >> (8 * c)) & 0xFFu);
                const float top = fmaf(tx, c01 - c00, c00), bot = fmaf(tx, c11 - c10, c10);
                out[c] = to_u8(fmaf(ty, bot - top, top));
            }
            return;
        }
        uint32_t x = min((uint32_t)(fu * (float)lw), lw - 1), y = min((uint32_t)(fv * (float)lh), lh - 1);
        uint32_t texel = sc.texels[off + (size_t)y * lw + x];
        out[0] = (uint8_t)(texel & 0xFFu);
        out[1] = (uint8_t)((texel >> 8) & 0xFFu);
        out[2] = (uint8_t)((texel >> 16) & 0xFFu);
    } else {
        out[0] = to_u8(rgb[0]);
        out[1] = to_u8(rgb[1]);
        out[2] = to_u8(rgb[2]);
    }
}

// Vertex k of a triangle from its shading record: one 64-byte record per triangle holds the three
// positions and the three colours (or texture coordinates), so a pixel's gather is one cache line
// instead of one per index, position and colour.
__device__ __forceinline__ CVert record_vertex(const float4 (&rec)[4], bool textured, const float (&M)[16], int k) {
    const float f[16] = {rec[0].x, rec[0].y, rec[0].z, rec[0].w, rec[1].x, rec[1].y, rec[1].z, rec[1].w,
                         rec[2].x, rec[2].y, rec[2].z, rec[2].w, rec[3].x, rec[3].y, rec[3].z, rec[3].w};
    CVert o;
    o.c = to_clip(M, f[3 * k], f[3 * k + 1], f[3 * k + 2]);
    if (textured) {
        o.r = f[9 + 2 * k];
        o.g = f[10 + 2 * k];
        o.b = 0.0f;
    } else {
        const uint32_t rgb = __float_as_uint(f[9 + k]);
        o.r = (float)(rgb & 0xFFu);
        o.g = (float)((rgb >> 8) & 0xFFu);
        o.b = (float)((rgb >> 16) & 0xFFu);
    }
    return o;
}

// Fetches the records of a wavefront's 64 pixels.  A lane that read its own 64-byte record with four
// 16-byte loads would hit one cache line four times while it is still on its way, and the cache
// handles such hits on a pending line one after the other.  So four lanes share a record instead:
// each load instruction of the wavefront then fetches sixteen whole records (sixteen different
// lines), and the pieces change hands through `stage` ([64][4] float4 of this wavefront, LDS).
__device__ __forceinline__ void load_records(const SceneDev& sc, uint32_t id, bool valid, int lane, float4* stage,
                                             float4 (&rec)[4]) {
    // the address of this lane's own record (lanes of one wavefront may belong to different scenes)
    const u64 mine = valid ? (u64)(reinterpret_cast<const float4*>(sc.tri_rec) + 4 * (size_t)id) : 0ull;
    const int part = lane & 3;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int from = 16 * s + (lane >> 2);
        const u64 at = (u64)(uint32_t)__shfl((int)(uint32_t)mine, from, 64) |
                       ((u64)(uint32_t)__shfl((int)(uint32_t)(mine >> 32), from, 64) << 32);
        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (at != 0ull) v = reinterpret_cast<const float4*>(at)[part];
        stage[4 * from + part] = v;
    }
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < 4; ++k) rec[k] = stage[4 * lane + k];
    wave_lds_sync();     // the stage may be refilled (k_shade_clipped loops)
}

// Pixel of thread p: frames are walked in 8x8-pixel tiles, one tile per wavefront, so that the
// pixels of a wavefront share triangles (equal addresses are fetched once).
__device__ __forceinline__ void pixel_of(size_t p, const FrameParams& fp, uint32_t& env, int& i, int& j) {
    const int HW = fp.H * fp.W;
    env = (uint32_t)(p / HW);
    const int q = (int)(p - (size_t)env * HW);
    const int tile = q >> 6, lane = q & 63, tiles_x = fp.W >> 3;
    i = ((tile % tiles_x) << 3) + (lane & 7);
    j = ((tile / tiles_x) << 3) + (lane >> 3);
}

}  // namespace

// Colour pass, first kernel: one thread per pixel.  A winner whose three vertices lie inside every
// clip plane (nearly all of them) is projected and shaded from registers.  The others are appended
// to a queue (pixel numbers) and left to k_shade_clipped, so that the clipper, whose polygons need
// 56 KB of LDS per wavefront, runs on full wavefronts of the few pixels that need it.
// There are kShadeQueues queues, work-group g appends to queue g % kShadeQueues with ONE global atomic
// (its wavefronts first add up in LDS): atomics of the whole chip on a single word are served one
// after the other by the memory side and took longer than all the rest of the pass.  Queue q starts
// at q * queue_cap; count[32 q] counts its entries (zero on entry); next_count is the counter block of
// the next request and is cleared here (the host alternates between two blocks).
__global__ __launch_bounds__(256) void k_shade(const SceneDev* __restrict__ scenes, const uint32_t* __restrict__ env_scene,
                                               const float* __restrict__ view_proj, FrameParams fp, uint32_t B,
                                               const uint32_t* __restrict__ tri_id, uint8_t* __restrict__ out_rgb,
                                               uint32_t* __restrict__ queue, uint32_t queue_cap, uint32_t* __restrict__ count,
                                               uint32_t* __restrict__ next_count) {
    __shared__ float4 stage_all[4 * 256];
    __shared__ uint32_t group_count, group_base;
    const int HW = fp.H * fp.W;
    // Work-groups are dealt to the eight dies round-robin by index.  The groups of one frame are mapped
    // to one die, so that pixels of neighbouring tiles that show the same triangle find its record in
    // that die's L2 (frames in whole sets of eight, frames of whole 256-pixel groups; identity otherwise).
    uint32_t group = blockIdx.x;
    if (HW % 256 == 0) {
        const uint32_t per_frame = (uint32_t)HW / 256u, die = group % 8u, turn = group / 8u;
        if (turn < (B / 8u) * per_frame) group = ((turn / per_frame) * 8u + die) * per_frame + turn % per_frame;
    }
    const size_t t = (size_t)group * blockDim.x + threadIdx.x;
    if (blockIdx.x == 0 && threadIdx.x < kShadeQueues) next_count[32 * threadIdx.x] = 0u;
    if (threadIdx.x == 0) group_count = 0u;
    __syncthreads();
    const bool active = t < (size_t)B * HW;      // whole wavefronts: HW is a multiple of 64
    const int lane = (int)(threadIdx.x & 63u);
    uint32_t env = 0;
    int i = 0, j = 0;
    pixel_of(active ? t : 0, fp, env, i, j);
    env = __builtin_amdgcn_readfirstlane(env);
    const size_t p = (size_t)env * HW + (size_t)j * fp.W + i;
    uint8_t out[3] = {0, 0, 0};
    const SceneDev sc = scenes[env_scene[env]];
    const uint32_t id = active ? tri_id[p] : 0xFFFFFFFFu;
    const bool textured = sc.texels != nullptr;
    bool clipped = false;
    const bool valid = id != 0xFFFFFFFFu && sc.tri_rec != nullptr && id < sc.n_tris;
    float4 rec[4];
    load_records(sc, id, valid, lane, stage_all + 256 * (threadIdx.x >> 6), rec);
    if (valid) {
        float M[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) M[k] = view_proj[(size_t)env * 16 + k];
        const CVert a = record_vertex(rec, textured, M, 0), b = record_vertex(rec, textured, M, 1),
                    c = record_vertex(rec, textured, M, 2);
        const uint32_t oc_or = outcode(a.c) | outcode(b.c) | outcode(c.c);
        // Crossing exactly one plane (nine in ten of the winners that cross any) leaves three or four
        // corners, which fit in registers: clipped here, in the order and with the arithmetic of the
        // general clipper.  Whatever crosses more planes goes to the queue.
        const bool one_plane = oc_or != 0u && (oc_or & (oc_or - 1u)) == 0u && oc_or < kInvalid;
        clipped = oc_or != 0u && !one_plane;
        CVert o0 = a, o1 = b, o2 = c, o3 = c;
        int m = 3;
        if (one_plane) {
            const int k = __builtin_ctz(oc_or);
            m = 0;
            auto put = [&](const CVert& q) {
                o0 = pick(m == 0, q, o0); o1 = pick(m == 1, q, o1); o2 = pick(m == 2, q, o2); o3 = pick(m == 3, q, o3);
                ++m;
            };
            CVert prev = c;
            float dprev = plane_dist(prev.c, k);
            auto step = [&](const CVert& v) {
                const float dv = plane_dist(v.c, k);
                const bool cin = dv >= 0.0f, pin = dprev >= 0.0f;
                if (cin != pin) {
                    const CVert in = pick(cin, v, prev), outv = pick(cin, prev, v);      // always from the inside corner
                    const float da = cin ? dv : dprev, db = cin ? dprev : dv;
                    const float t = da / (da - db);
                    CVert q;
                    q.c.x = fmaf(t, outv.c.x - in.c.x, in.c.x);
                    q.c.y = fmaf(t, outv.c.y - in.c.y, in.c.y);
                    q.c.z = fmaf(t, outv.c.z - in.c.z, in.c.z);
                    q.c.w = fmaf(t, outv.c.w - in.c.w, in.c.w);
                    q.r = fmaf(t, outv.r - in.r, in.r);
                    q.g = fmaf(t, outv.g - in.g, in.g);
                    q.b = fmaf(t, outv.b - in.b, in.b);
                    put(q);
                }
                if (cin) put(v);
                prev = v;
                dprev = dv;
            };
            step(a);
            step(b);
            step(c);
        }
        if (!clipped && m >= 3) {
            SVert s0, s1, s2, s3;
            bool unused;
            bool ok = project(o0.c, fp, s0.xy, s0.iw, unused);
            ok = project(o1.c, fp, s1.xy, s1.iw, unused) && ok;
            ok = project(o2.c, fp, s2.xy, s2.iw, unused) && ok;
            s0.r = o0.r; s0.g = o0.g; s0.b = o0.b;
            s1.r = o1.r; s1.g = o1.g; s1.b = o1.b;
            s2.r = o2.r; s2.g = o2.g; s2.b = o2.b;
            s3 = s2;
            if (m == 4) {
                ok = project(o3.c, fp, s3.xy, s3.iw, unused) && ok;
                s3.r = o3.r; s3.g = o3.g; s3.b = o3.b;
            }
            float d = 0.0f, rgb[3], uv_area2;
            int area2;
            bool found = false;
            if (ok && piece_colour(s0, s1, s2, i, j, d, rgb, uv_area2, area2)) {
                found = true;
                piece_output(sc, textured, fp.bilinear != 0, rgb, uv_area2, area2, out);
            }
            // the second fan piece; should rounding ever make both cover this pixel, the nearer one is
            // the one the z-test kept (the first one on a tie)
            float d2;
            if (ok && m == 4 && piece_colour(s0, s2, s3, i, j, d2, rgb, uv_area2, area2) && (!found || d2 < d))
                piece_output(sc, textured, fp.bilinear != 0, rgb, uv_area2, area2, out);
        }
    }
    const u64 cm = ballot64(clipped);
    uint32_t wave_base = 0;
    if (cm != 0ull && lane == 0) wave_base = atomicAdd(&group_count, (uint32_t)__popcll(cm));
    wave_base = __builtin_amdgcn_readfirstlane(wave_base);
    __syncthreads();
    if (threadIdx.x == 0 && group_count != 0u) group_base = atomicAdd(&count[32 * (blockIdx.x % kShadeQueues)], group_count);
    __syncthreads();
    if (clipped)
        queue[(size_t)(blockIdx.x % kShadeQueues) * queue_cap + group_base + wave_base + rank_below(cm)] = (uint32_t)p;
    if (active && !clipped) {
        out_rgb[3 * p + 0] = out[0];
        out_rgb[3 * p + 1] = out[1];
        out_rgb[3 * p + 2] = out[2];
    }
}

// Colour pass, second kernel: the queued pixels, whose winning triangle crosses a clip plane.  The
// triangle is clipped exactly as the raster kernel clipped it, and the fan piece that covers the
// pixel centre gives the colour.
__global__ __launch_bounds__(64) void k_shade_clipped(const SceneDev* __restrict__ scenes, const uint32_t* __restrict__ env_scene,
                                                      const float* __restrict__ view_proj, FrameParams fp,
                                                      const uint32_t* __restrict__ tri_id, uint8_t* __restrict__ out_rgb,
                                                      const uint32_t* __restrict__ queue_all, uint32_t queue_cap,
                                                      const uint32_t* __restrict__ count) {
    __shared__ float4 stage[256];
    __shared__ float poly[2 * kMaxPoly * 7 * 64];
    const int HW = fp.H * fp.W;
    // work-group b serves queue b % kShadeQueues together with the other groups of the same residue
    const uint32_t q = blockIdx.x % kShadeQueues, worker = blockIdx.x / kShadeQueues, workers = gridDim.x / kShadeQueues;
    const uint32_t n = count[32 * q];
    const uint32_t* queue = queue_all + (size_t)q * queue_cap;
    const int lane = (int)threadIdx.x;
    for (uint32_t base = worker * 64u; base < n; base += workers * 64u) {
        const uint32_t q0 = base + threadIdx.x;
        const bool have = q0 < n;
        const size_t p = queue[have ? q0 : base];      // pixel number in the output's own order
        const uint32_t env = (uint32_t)(p / HW);
        const int pix = (int)(p - (size_t)env * HW);
        const int i = pix % fp.W, j = pix / fp.W;
        uint8_t out[3] = {0, 0, 0};
        const uint32_t id = tri_id[p];
        const SceneDev sc = scenes[env_scene[env]];
        const bool textured = sc.texels != nullptr;
        float M[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) M[k] = view_proj[(size_t)env * 16 + k];
        float4 rec[4];
        // (the queue only ever holds pixels with a valid winner; the check keeps a stray entry harmless)
        const bool valid = have && sc.tri_rec != nullptr && id < sc.n_tris;
        load_records(sc, id, valid, lane, stage, rec);
        if (!valid) continue;
        // Polygons live in LDS, one word per (buffer, corner, attribute, lane) with the lane running
        // fastest (no bank conflicts whatever corner each lane addresses); private arrays would be
        // indexed per lane and therefore sit in memory, a round trip per corner.
        auto put = [&](int buf, int q, const CVert& v) {
            float* at = poly + ((buf * kMaxPoly + q) * 7) * 64 + lane;
            at[0] = v.c.x; at[64] = v.c.y; at[128] = v.c.z; at[192] = v.c.w; at[256] = v.r; at[320] = v.g; at[384] = v.b;
        };
        auto get = [&](int buf, int q) {
            const float* at = poly + ((buf * kMaxPoly + q) * 7) * 64 + lane;
            CVert v;
            v.c.x = at[0]; v.c.y = at[64]; v.c.z = at[128]; v.c.w = at[192]; v.r = at[256]; v.g = at[320]; v.b = at[384];
            return v;
        };
        uint32_t oc_or = 0;
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const CVert v = record_vertex(rec, textured, M, k);
            put(0, k, v);
            oc_or |= outcode(v.c);
        }
        int cnt = 3, cur = 0;
        const int order[6] = {4, 5, 0, 1, 2, 3};
        for (int oi = 0; oi < 6; ++oi) {
            int k = order[oi];
            if (!((oc_or >> k) & 1u) || cnt < 3) continue;
            int m = 0;
            CVert prev = get(cur, cnt - 1);
            float dprev = plane_dist(prev.c, k);
            for (int q = 0; q < cnt; ++q) {
                CVert v = get(cur, q);
                float dv = plane_dist(v.c, k);
                bool cin = dv >= 0.0f, pin = dprev >= 0.0f;
                if (cin != pin && m < kMaxPoly) {
                    const CVert a = pick(cin, v, prev);      // inside
                    const CVert b = pick(cin, prev, v);      // outside
                    float da = cin ? dv : dprev, db = cin ? dprev : dv;
                    float t = da / (da - db);
                    CVert o;
                    o.c.x = fmaf(t, b.c.x - a.c.x, a.c.x);
                    o.c.y = fmaf(t, b.c.y - a.c.y, a.c.y);
                    o.c.z = fmaf(t, b.c.z - a.c.z, a.c.z);
                    o.c.w = fmaf(t, b.c.w - a.c.w, a.c.w);
                    o.r = fmaf(t, b.r - a.r, a.r);
                    o.g = fmaf(t, b.g - a.g, a.g);
                    o.b = fmaf(t, b.b - a.b, a.b);
                    put(cur ^ 1, m++, o);
                }
                if (cin && m < kMaxPoly) put(cur ^ 1, m++, v);
                prev = v;
                dprev = dv;
            }
            cnt = m;
            cur ^= 1;
        }
        if (cnt >= 3) {
            // projected corners go to the other buffer: snapped position, 1/w and the attributes
            auto get_s = [&](int q) {
                const float* at = poly + (((cur ^ 1) * kMaxPoly + q) * 7) * 64 + lane;
                SVert v;
                v.xy = __float_as_uint(at[0]); v.iw = at[64]; v.r = at[128]; v.g = at[192]; v.b = at[256];
                return v;
            };
            bool ok = true;
            for (int q = 0; q < cnt; ++q) {
                const CVert v = get(cur, q);
                bool unused;
                uint32_t xy;
                float iw;
                ok = project(v.c, fp, xy, iw, unused) && ok;
                float* at = poly + (((cur ^ 1) * kMaxPoly + q) * 7) * 64 + lane;
                at[0] = __uint_as_float(xy); at[64] = iw; at[128] = v.r; at[192] = v.g; at[256] = v.b;
            }
            if (ok) {
                // the fan pieces of one triangle tile it; should rounding ever make two of them
                // cover this pixel, the nearer one is the one the z-test kept (first one on a tie)
                float best = 0.0f;
                bool found = false;
                const SVert s0 = get_s(0);
                SVert s1 = get_s(1);
                for (int q = 1; q + 1 < cnt; ++q) {
                    const SVert s2 = get_s(q + 1);
                    float d, rgb[3], uv_area2;
                    int area2;
                    if (piece_colour(s0, s1, s2, i, j, d, rgb, uv_area2, area2) && (!found || d < best)) {
                        found = true;
                        best = d;
                        piece_output(sc, textured, fp.bilinear != 0, rgb, uv_area2, area2, out);
                    }
                    s1 = s2;
                }
            }
        }
        out_rgb[3 * p + 0] = out[0];
        out_rgb[3 * p + 1] = out[1];
        out_rgb[3 * p + 2] = out[2];
    }
}

// 2x2 box filter from the rendered frame to the output frame (the paper renders its 128-pixel
// observations at twice the resolution and downsamples, Sec. 4.1).  Depth: ((a + b) + (c + d)) / 4
// in float32 in that order; colour: (a + b + c + d + 2) >> 2 per channel.
__global__ __launch_bounds__(256) void k_downsample(const float* __restrict__ depth, const uint8_t* __restrict__ rgb,
                                                    uint32_t B, int H, int W, float* __restrict__ out_depth,
                                                    uint8_t* __restrict__ out_rgb) {
    const int oh = H >> 1, ow = W >> 1;
    size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= (size_t)B * oh * ow) return;
    const int x = (int)(p % ow), y = (int)((p / ow) % oh);
    const size_t b = p / ((size_t)ow * oh);
    const size_t s = b * H * W + (size_t)(2 * y) * W + 2 * x;
    out_depth[p] = ((depth[s] + depth[s + 1]) + (depth[s + W] + depth[s + W + 1])) * 0.25f;
    if (rgb && out_rgb)
        for (int c = 0; c < 3; ++c)
            out_rgb[3 * p + c] = (uint8_t)(((int)rgb[3 * s + c] + (int)rgb[3 * (s + 1) + c] + (int)rgb[3 * (s + W) + c] +
                                            (int)rgb[3 * (s + W + 1) + c] + 2) >> 2);
}

void launch_downsample(hipStream_t stream, const float* depth, const uint8_t* rgb, uint32_t B, int H, int W,
                       float* out_depth, uint8_t* out_rgb) {
    size_t n = (size_t)B * (H / 2) * (W / 2);
    hipLaunchKernelGGL(k_downsample, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, depth, rgb, B, H, W, out_depth,
                       out_rgb);
}

// One thread per triangle: gather its three positions and colours (or texture coordinates) from the
// uploaded arrays into its 64-byte shading record.
__global__ __launch_bounds__(256) void k_build_shade_records(SceneDev sc, float* __restrict__ tri_rec) {
    const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= sc.n_tris) return;
    float f[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) f[k] = 0.0f;
    for (int k = 0; k < 3; ++k) {
        const uint32_t vi = sc.indices[3 * t + k];
        f[3 * k] = sc.verts[3 * (size_t)vi];
        f[3 * k + 1] = sc.verts[3 * (size_t)vi + 1];
        f[3 * k + 2] = sc.verts[3 * (size_t)vi + 2];
        if (sc.uvs) {
            f[9 + 2 * k] = sc.uvs[2 * (size_t)vi];
            f[10 + 2 * k] = sc.uvs[2 * (size_t)vi + 1];
        } else if (sc.colors) {
            const uint8_t* col = sc.colors + 3 * (size_t)vi;
            f[9 + k] = __uint_as_float((uint32_t)col[0] | ((uint32_t)col[1] << 8) | ((uint32_t)col[2] << 16));
        }
    }
    float4* dst = reinterpret_cast<float4*>(tri_rec) + 4 * t;
#pragma unroll
    for (int k = 0; k < 4; ++k) dst[k] = make_float4(f[4 * k], f[4 * k + 1], f[4 * k + 2], f[4 * k + 3]);
}

void launch_build_shade_records(hipStream_t stream, const SceneDev& sc, float* tri_rec) {
    hipLaunchKernelGGL(k_build_shade_records, dim3((sc.n_tris + 255u) / 256u), dim3(256), 0, stream, sc, tri_rec);
}

void launch_shade(hipStream_t stream, const SceneDev* scenes, const uint32_t* env_scene, const float* view_proj,
                  const FrameParams& fp, uint32_t B, const uint32_t* tri_id, uint8_t* out_rgb, uint32_t* queue,
                  uint32_t* count, uint32_t* next_count) {
    const size_t n = (size_t)B * fp.H * fp.W;
    const unsigned groups = (unsigned)((n + 255) / 256);
    const uint32_t queue_cap = shade_queue_cap(n);
    hipLaunchKernelGGL(k_shade, dim3(groups), dim3(256), 0, stream, scenes, env_scene, view_proj, fp, B, tri_id, out_rgb, queue,
                       queue_cap, count, next_count);
    // a few wavefronts per queue, each striding over its queue (most find little or nothing to do)
    const unsigned workers = (unsigned)std::min<size_t>((n / kShadeQueues + 63) / 64 + 1, 32);
    hipLaunchKernelGGL(k_shade_clipped, dim3(kShadeQueues * workers), dim3(64), 0, stream, scenes, env_scene, view_proj, fp,
                       tri_id, out_rgb, queue, queue_cap, count);
}

}  // namespace bps
