// Fused geometry + rasterisation kernel for gfx950.  See raster_kernels.h for the plan.
//
// Numeric rule implemented here (the paper, Sec. 3.2, leaves it to the graphics API):
//   clip = M v by nested fma; planes w+x, w-x, w+y, w-y, z, w-z >= 0; Sutherland-Hodgman in the
//   order near, far, left, right, top, bottom with crossings interpolated from the inside vertex;
//   X = rint(fma(x/w, 128 W, 128 W)) in 1/256 px; integer edge functions with the top-left rule;
//   depth = A2 / (e0/w0 + e1/w1 + e2/w2); per pixel the minimum of (depth bits << 32 | id).
#include "raster_device.h"
#include "raster_kernels.h"

namespace bps {
namespace {

using namespace dev;

// ---------------------------------------------------------------------------------------------
// Per-wave state kept in LDS.
struct WaveLds {
    float2* stage;      // [64] staged vertices of the current cluster: (packed xy bits, 1/w)
    uint32_t* stage_oc; // [64] their outcodes
    uint32_t* smallq;   // [8][64] struct-of-arrays: xy0 xy1 xy2 iw0 iw1 iw2 id box
    uint32_t* tally;    // diagnostics (wave-private registers, dead code in the production instances): see kT*
};
// diagnostics tallies
enum { kTSmall = 0, kTLarge = 1, kTDrains = 2, kTDrainIters = 3, kTDrainDepth = 4, kTEmits = 5, kTMedPasses = 6, kTLargeSteps = 7,
       kTPushes = 8, kTClipDrains = 9, kTClipPasses = 10, kTFanIters = 11, kTPopPasses = 12, kTSlots = 13, kTClusters = 14,
       kTPhaseAPasses = 15, kTCount = 16 };

// One lane per queued small triangle: at most kSmallMax pixel centres each.
__device__ __forceinline__ void drain_small(const WaveLds& L, int n, int lane, u64* vis, const Window& win,
                                            const BPS_GLOBAL uint32_t* ctri_id) {
    bool have = lane < n;
    // the queue holds the triangle's slot in the cluster arrays; its id is fetched here, one
    // gather per 64 triangles, and arrives while the edge set-up is computed
    const uint32_t ref = have ? L.smallq[6 * 64 + lane] : 0u;
    const uint32_t id = ctri_id[ref];
    uint32_t xy0 = L.smallq[0 * 64 + lane], xy1 = L.smallq[1 * 64 + lane], xy2 = L.smallq[2 * 64 + lane];
    float iw0 = __uint_as_float(L.smallq[3 * 64 + lane]), iw1 = __uint_as_float(L.smallq[4 * 64 + lane]),
          iw2 = __uint_as_float(L.smallq[5 * 64 + lane]);
    uint32_t box = L.smallq[7 * 64 + lane];
    Setup s = make_setup(xy0, xy1, xy2, iw0, iw1, iw2);
    int i_lo = (int)(box & 0xFFu), j_lo = (int)((box >> 8) & 0xFFu);
    int nx = (int)((box >> 16) & 0xFFu), ny = (int)(box >> 24);
    int cnt = (have && s.A2 != 0) ? nx * ny : 0;
    // Edge functions at the first pixel centre, then stepped: one pixel to the right changes edge k by
    // -256 dy_k, and going from the end of a row to the start of the next by 256 dx_k + 256 (nx - 1) dy_k.
    // Same integers as evaluating each pixel afresh (all of them are areas inside the triangle's box).
    const int px = (i_lo << 8) + 128 - kOrigin, py = (j_lo << 8) + 128 - kOrigin;
    int E0 = __mul24(s.dx0, py - s.Y1) - __mul24(s.dy0, px - s.X1);
    int E1 = __mul24(s.dx1, py - s.Y2) - __mul24(s.dy1, px - s.X2);
    int E2 = __mul24(s.dx2, py - s.Y0) - __mul24(s.dy2, px - s.X0);
    const int right0 = -(s.dy0 << 8), right1 = -(s.dy1 << 8), right2 = -(s.dy2 << 8);
    const int wrap0 = (s.dx0 + __mul24(nx - 1, s.dy0)) << 8, wrap1 = (s.dx1 + __mul24(nx - 1, s.dy1)) << 8,
              wrap2 = (s.dx2 + __mul24(nx - 1, s.dy2)) << 8;
    int at = __mul24(j_lo - win.y0, win.w) + (i_lo - win.x0), col = 0;
    const int at_wrap = win.w - nx + 1;
    const float a2f = (float)s.A2;
    ++L.tally[kTDrains];
    for (int k = 0; k < kSmallMax; ++k) {
        const bool act = k < cnt;
        if (ballot64(act) == 0) break;
        ++L.tally[kTDrainIters];
        if (ballot64(act && (((E0 + s.b0) | (E1 + s.b1) | (E2 + s.b2)) >= 0)) != 0ull) ++L.tally[kTDrainDepth];
        if (act && (((E0 + s.b0) | (E1 + s.b1) | (E2 + s.b2)) >= 0)) {
            const float num = fmaf((float)E2, s.iw2, fmaf((float)E1, s.iw1, (float)E0 * s.iw0));
            const float depth = a2f / num;
            atomicMin(&vis[at], ((u64)__float_as_uint(depth) << 32) | (u64)id);
        }
        const bool row_end = ++col == nx;
        E0 += row_end ? wrap0 : right0;
        E1 += row_end ? wrap1 : right1;
        E2 += row_end ? wrap2 : right2;
        at += row_end ? at_wrap : 1;
        col = row_end ? 0 : col;
    }
}

// Append small triangles to the wave's queue; whenever it reaches 64 entries, drain them.
__device__ __forceinline__ void push_small(const WaveLds& L, int& count, bool want, uint32_t xy0, uint32_t xy1,
                                           uint32_t xy2, float iw0, float iw1, float iw2, uint32_t ref, uint32_t box,
                                           int lane, u64* vis, const Window& win,
                                           const BPS_GLOBAL uint32_t* ctri_id, u64 mask) {
    // mask = the lanes that want (handed in: callers build it from ballots of single comparisons,
    // which cost one compare each, instead of a ballot of the combined condition)
    if (mask == 0) return;
    int n = __popcll(mask);
    L.tally[kTSmall] += (uint32_t)n;
    ++L.tally[kTPushes];
    int rank = (int)rank_below(mask);
    int room = 64 - count;
    int pos = count + rank;            // position if the queue were unbounded
    bool first = want && rank < room;
    bool later = want && !first;
    if (first) {
        L.smallq[0 * 64 + pos] = xy0; L.smallq[1 * 64 + pos] = xy1; L.smallq[2 * 64 + pos] = xy2;
        L.smallq[3 * 64 + pos] = __float_as_uint(iw0); L.smallq[4 * 64 + pos] = __float_as_uint(iw1);
        L.smallq[5 * 64 + pos] = __float_as_uint(iw2);
        L.smallq[6 * 64 + pos] = ref; L.smallq[7 * 64 + pos] = box;
    }
    if (n >= room) {
        wave_lds_sync();
        drain_small(L, 64, lane, vis, win, ctri_id);
        wave_lds_sync();
        pos -= 64;
        if (later) {
            L.smallq[0 * 64 + pos] = xy0; L.smallq[1 * 64 + pos] = xy1; L.smallq[2 * 64 + pos] = xy2;
            L.smallq[3 * 64 + pos] = __float_as_uint(iw0); L.smallq[4 * 64 + pos] = __float_as_uint(iw1);
            L.smallq[5 * 64 + pos] = __float_as_uint(iw2);
            L.smallq[6 * 64 + pos] = ref; L.smallq[7 * 64 + pos] = box;
        }
        count = n - room;
    } else {
        count += n;
    }
}

// Whole wavefront on one large triangle: 8x8 pixel blocks over its bounding box.
__device__ __forceinline__ void raster_large(uint32_t xy0, uint32_t xy1, uint32_t xy2, float iw0, float iw1, float iw2,
                                             uint32_t id, int i_lo, int i_hi, int j_lo, int j_hi, int lane, u64* vis,
                                             const Window& win, uint32_t* tally) {
    Setup s = make_setup(xy0, xy1, xy2, iw0, iw1, iw2);
    int li = lane & 7, lj = lane >> 3;
    for (int by = j_lo >> 3; by <= (j_hi >> 3); ++by) {
        int j = (by << 3) + lj;
        bool jok = j >= j_lo && j <= j_hi;
        for (int bx = i_lo >> 3; bx <= (i_hi >> 3); ++bx) {
            int i = (bx << 3) + li;
            bool act = jok && i >= i_lo && i <= i_hi;
            ++tally[kTLargeSteps];
            shade_pixel(s, i, j, act, id, vis, win);
        }
    }
}

typedef short short2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ short2v as_s2(uint32_t v) { return __builtin_bit_cast(short2v, v); }
__device__ __forceinline__ uint32_t as_u32(short2v v) { return __builtin_bit_cast(uint32_t, v); }

// Pixel centres inside a triangle's bounding box, both axes at once with packed 16-bit
// arithmetic.  Pixel i has its centre at 256 (i - 64) + 128 in packed coordinates, so the first
// centre at or right of x is (x + 127) >> 8 and the last centre at or left of x is (x - 128) >> 8
// (both minus 64).  Returns false when the box, clamped to the work-group's window of the frame,
// holds no centre; otherwise lo = first pixel - 64 and ext = last - first per axis.
__device__ __forceinline__ bool centre_box(uint32_t xy0, uint32_t xy1, uint32_t xy2, const Window& win, short2v& lo,
                                           short2v& ext) {
    short2v a = as_s2(xy0), b = as_s2(xy1), c = as_s2(xy2);
    short2v mn = __builtin_elementwise_min(a, __builtin_elementwise_min(b, c));
    short2v mx = __builtin_elementwise_max(a, __builtin_elementwise_max(b, c));
    lo = (mn + (short)127) >> (short)8;
    short2v hi = (mx - (short)128) >> (short)8;
    short2v lo_clamp = {(short)(win.x0 - 64), (short)(win.y0 - 64)};
    short2v hi_clamp = {(short)(win.x0 + win.w - 65), (short)(win.y0 + win.h - 65)};
    lo = __builtin_elementwise_max(lo, lo_clamp);
    hi = __builtin_elementwise_min(hi, hi_clamp);
    ext = hi - lo;                              // both halves >= 0: some pixel centre is inside
    return (as_u32(ext) & 0x80008000u) == 0;
}

// Classification and hand-off of one candidate triangle per lane whose box holds a pixel centre.
// ref = cluster * 128 + slot addresses the triangle's original id in ctri_id; small triangles
// carry it through the queue, only large ones look the id up here.
__device__ __forceinline__ void emit(const WaveLds& L, int& small_count, bool valid, short2v lo, short2v ext,
                                     uint32_t xy0, uint32_t xy1, uint32_t xy2, float iw0, float iw1, float iw2,
                                     uint32_t ref, const BPS_GLOBAL uint32_t* ctri_id, int lane, u64* vis,
                                     const Window& win, u64 vmask) {
    // vmask = the lanes with valid set
    if (vmask == 0) return;
    ++L.tally[kTEmits];
    int nx = (int)ext.x + 1, ny = (int)ext.y + 1;
    int i_lo = (int)lo.x + 64, j_lo = (int)lo.y + 64;
    const bool few = nx * ny <= kSmallMax, narrow = nx <= 8, low = ny <= 8;
    const u64 small_mask = vmask & ballot64(few);
    const bool small = valid && few;
    uint32_t box = (uint32_t)i_lo | ((uint32_t)j_lo << 8) | ((uint32_t)nx << 16) | ((uint32_t)ny << 24);
    push_small(L, small_count, small, xy0, xy1, xy2, iw0, iw1, iw2, ref, box, lane, vis, win, ctri_id, small_mask);
    u64 med = vmask & ~small_mask & ballot64(narrow) & ballot64(low);
    u64 big = vmask & ~small_mask & ~med;
    L.tally[kTLarge] += (uint32_t)__popcll(med | big);
    const uint32_t id = (valid && !small) ? ctri_id[ref] : 0u;
    // medium triangles (box within 8x8 pixels): four per pass, sixteen lanes each, 4x4 pixels per step
    while (med) {
        ++L.tally[kTMedPasses];
        int src[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            src[k] = med ? __builtin_ctzll(med) : -1;
            med &= med - 1;     // 0 & anything stays 0
        }
        const int g = lane >> 4;
        const int from = g == 0 ? src[0] : g == 1 ? src[1] : g == 2 ? src[2] : src[3];
        const bool on = from >= 0;
        const int f = on ? from : 0;
        const uint32_t mxy0 = (uint32_t)__shfl((int)xy0, f, 64), mxy1 = (uint32_t)__shfl((int)xy1, f, 64),
                       mxy2 = (uint32_t)__shfl((int)xy2, f, 64);
        const float miw0 = __shfl(iw0, f, 64), miw1 = __shfl(iw1, f, 64), miw2 = __shfl(iw2, f, 64);
        const uint32_t mid = (uint32_t)__shfl((int)id, f, 64), mbox = (uint32_t)__shfl((int)box, f, 64);
        const Setup st = make_setup(mxy0, mxy1, mxy2, miw0, miw1, miw2);
        const int mi = (int)(mbox & 0xFFu), mj = (int)((mbox >> 8) & 0xFFu);
        const int mnx = (int)((mbox >> 16) & 0xFFu), mny = (int)(mbox >> 24);
        const int li = lane & 3, lj = (lane >> 2) & 3;
#pragma unroll
        for (int by = 0; by < 2; ++by)
#pragma unroll
            for (int bx = 0; bx < 2; ++bx) {
                const int di = bx * 4 + li, dj = by * 4 + lj;
                const bool act = on && di < mnx && dj < mny;
                if (ballot64(act) == 0) continue;
                shade_pixel(st, mi + di, mj + dj, act, mid, vis, win);
            }
    }
    while (big) {
        int src = __builtin_ctzll(big);
        big &= big - 1;
        int bi = bcast_i(i_lo, src), bj = bcast_i(j_lo, src);
        raster_large((uint32_t)bcast_i((int)xy0, src), (uint32_t)bcast_i((int)xy1, src), (uint32_t)bcast_i((int)xy2, src),
                     bcast_f(iw0, src), bcast_f(iw1, src), bcast_f(iw2, src), (uint32_t)bcast_i((int)id, src), bi,
                     bi + bcast_i(nx, src) - 1, bj, bj + bcast_i(ny, src) - 1, lane, vis, win, L.tally);
    }
}

// Conservative test of an axis-aligned box against the planes that bound the work-group's window
// of the frame, in world space: near z >= 0, far w - z >= 0 and the four side planes
// x - aL w >= 0, aR w - x >= 0, y - aT w >= 0, aB w - y >= 0 (aL = -1, aR = +1 for a whole frame,
// i.e. w + x >= 0 and w - x >= 0).  For each plane the largest value over the box is compared with a
// negative margin proportional to the magnitude of the terms, so that rounding in this test and
// in the per-vertex transform can never cull a box holding a vertex the exact rule keeps; window
// edges lie half a pixel outside the outermost pixel centres, far more than vertex snapping moves
// anything.  NaNs compare false and therefore never cull.
__device__ __forceinline__ bool box_outside_frustum(const float (&M)[16], const Window& win, float lx, float ly,
                                                    float lz, float hx, float hy, float hz) {
    const float eps = 1.52587890625e-05f;   // 2^-16
    float ax = fmaxf(fabsf(lx), fabsf(hx)), ay = fmaxf(fabsf(ly), fabsf(hy)), az = fmaxf(fabsf(lz), fabsf(hz));
    bool outside = false;
#pragma unroll
    for (int k = 0; k < 6; ++k) {
        float px, py, pz, pw, qx, qy, qz, qw;   // plane coefficients and their magnitudes
        if (k == 4) {
            px = M[8]; py = M[9]; pz = M[10]; pw = M[11];
            qx = fabsf(px); qy = fabsf(py); qz = fabsf(pz); qw = fabsf(pw);
        } else if (k == 5) {
            px = M[12] - M[8]; py = M[13] - M[9]; pz = M[14] - M[10]; pw = M[15] - M[11];
            qx = fabsf(M[12]) + fabsf(M[8]); qy = fabsf(M[13]) + fabsf(M[9]);
            qz = fabsf(M[14]) + fabsf(M[10]); qw = fabsf(M[15]) + fabsf(M[11]);
        } else {
            const int r = (k < 2) ? 0 : 1;
            // (row_r - a row_3) for the low side, (a row_3 - row_r) for the high side
            const float a = k == 0 ? win.aL : k == 1 ? win.aR : k == 2 ? win.aT : win.aB;
            const float sg = (k == 0 || k == 2) ? 1.0f : -1.0f;
            px = sg * (M[4 * r + 0] - a * M[12]); py = sg * (M[4 * r + 1] - a * M[13]);
            pz = sg * (M[4 * r + 2] - a * M[14]); pw = sg * (M[4 * r + 3] - a * M[15]);
            const float aa = fabsf(a);
            qx = fabsf(M[4 * r + 0]) + aa * fabsf(M[12]); qy = fabsf(M[4 * r + 1]) + aa * fabsf(M[13]);
            qz = fabsf(M[4 * r + 2]) + aa * fabsf(M[14]); qw = fabsf(M[4 * r + 3]) + aa * fabsf(M[15]);
        }
        float dmax = pw + fmaxf(px * lx, px * hx) + fmaxf(py * ly, py * hy) + fmaxf(pz * lz, pz * hz);
        float mag = fmaf(qx, ax, fmaf(qy, ay, fmaf(qz, az, qw)));
        outside = outside || (dmax < -eps * mag);
    }
    return outside;
}

constexpr uint32_t kNoPixel = 0xFFFFFFFFu;   // box_footprint: the box cannot cover any pixel centre

// Screen footprint and nearest possible depth of a box, for the occlusion test made when the
// cluster is popped.  Every triangle inside the box rasterises with a depth that is a convex
// combination of clip w values attained inside the box, onto pixels inside the projection of the
// box.  So if the smallest w over the box (minus a rounding margin) is larger than the depth
// already stored at every pixel whose centre the projected box can reach, nothing in the box can
// win the z-test.  Returns the packed test record, or 0 when no bound can be given (the box
// may reach the eye plane, or is more than 32 pixels wide or high):
//   bit 0 testable | x0 6 bits | y0 6 bits (both relative to the window) | width-1 5 bits |
//   height-1 5 bits, and in wbits18 the exponent and top ten mantissa bits of the w bound
//   (truncated, i.e. rounded towards the eye)
__device__ __forceinline__ uint32_t box_footprint(const float (&M)[16], const FrameParams& fp, const Window& win,
                                                 float lx, float ly, float lz, float hx, float hy, float hz,
                                                 uint32_t& wbits18) {
    const float eps = 1.52587890625e-05f;   // 2^-16
    wbits18 = 0u;
    float ax = fmaxf(fabsf(lx), fabsf(hx)), ay = fmaxf(fabsf(ly), fabsf(hy)), az = fmaxf(fabsf(lz), fabsf(hz));
    float wmin = M[15] + fminf(M[12] * lx, M[12] * hx) + fminf(M[13] * ly, M[13] * hy) + fminf(M[14] * lz, M[14] * hz);
    float wmag = fmaf(fabsf(M[12]), ax, fmaf(fabsf(M[13]), ay, fmaf(fabsf(M[14]), az, fabsf(M[15]))));
    float wcons = wmin - eps * wmag;
    if (!(wcons > 0.0f)) return 0u;
    float x0 = 3.0e38f, x1 = -3.0e38f, y0 = 3.0e38f, y1 = -3.0e38f;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float x = (k & 1) ? hx : lx, y = (k & 2) ? hy : ly, z = (k & 4) ? hz : lz;
        float cx = fmaf(M[2], z, fmaf(M[1], y, fmaf(M[0], x, M[3])));
        float cy = fmaf(M[6], z, fmaf(M[5], y, fmaf(M[4], x, M[7])));
        float cw = fmaf(M[14], z, fmaf(M[13], y, fmaf(M[12], x, M[15])));
        float rw = __builtin_amdgcn_rcpf(fmaxf(cw, wcons));   // approximate is fine: a whole pixel of slack follows
        float sx = cx * rw, sy = cy * rw;
        x0 = fminf(x0, sx); x1 = fmaxf(x1, sx);
        y0 = fminf(y0, sy); y1 = fmaxf(y1, sy);
    }
    // pixels whose centres (i + 0.5) lie inside the projected box, with 1/64 pixel of slack for
    // vertex snapping (1/512 px) and rounding; none at all means nothing in the box can cover a centre
    const float hw = 0.5f * (float)fp.W, hh = 0.5f * (float)fp.H, slack = 0.015625f;
    float fx0 = ceilf(fmaf(x0, hw, hw) - 0.5f - slack), fx1 = floorf(fmaf(x1, hw, hw) - 0.5f + slack);
    float fy0 = ceilf(fmaf(y0, hh, hh) - 0.5f - slack), fy1 = floorf(fmaf(y1, hh, hh) - 0.5f + slack);
    if (!(fx0 == fx0 && fx1 == fx1 && fy0 == fy0 && fy1 == fy1)) return 0u;   // NaN somewhere: no bound
    fx0 = fmaxf(fx0, (float)win.x0); fy0 = fmaxf(fy0, (float)win.y0);
    fx1 = fminf(fx1, (float)(win.x0 + win.w - 1)); fy1 = fminf(fy1, (float)(win.y0 + win.h - 1));
    if (fx0 > fx1 || fy0 > fy1) return kNoPixel;
    int ix0 = (int)fx0, ix1 = (int)fx1, iy0 = (int)fy0, iy1 = (int)fy1;
    int bw = ix1 - ix0, bh = iy1 - iy0;
    if (bw > 31 || bh > 31) return 0u;
    wbits18 = __float_as_uint(wcons) >> 13;      // positive: the sign bit is clear, 18 bits remain
    return 1u | ((uint32_t)(ix0 - win.x0) << 1) | ((uint32_t)(iy0 - win.y0) << 7) | ((uint32_t)bw << 13) | ((uint32_t)bh << 18);
}

// Depth bin of a survivor record: exponent and top three mantissa bits of its w bound, i.e.
// eight bins per octave from 2^-7 upwards; records without a bound (near or large boxes) go first.
__device__ __forceinline__ int depth_bin(u64 e) {
    if (!((e >> 23) & 1ull)) return 0;
    int k = (int)(e >> 53) - 120 * 8;     // exponent and three mantissa bits of the w bound
    return min(max(k, 0), kDepthBins - 1);
}

// The clip ring is shared by the work-group: with one ring a clipper pass of 64 triangles comes up
// eight times sooner than with a queue per wavefront, and what waits for the clipper are the triangles
// along the window's border, without which no footprint touching a border pixel can be found hidden.
//   tail  entries reserved by producers (one LDS atomic per wavefront and push)
//   head  entries claimed by consumers
// An entry is written right after its reservation and reads kClipEmpty until then; the consumer of a
// claimed entry waits for it to turn up and puts kClipEmpty back.
constexpr uint32_t kClipEmpty = 0xFFFFFFFFu;      // no entry: cluster << 7 | slot stays below 2^30
struct ClipRing {
    uint32_t* slot;      // [mask + 1]
    uint32_t* tail;
    uint32_t* head;
    uint32_t mask;
};

// tail_seen: the ring's tail right after this wavefront's reservation
__device__ __forceinline__ void push_clip(const ClipRing& R, bool want, uint32_t ref, u64 mask, int lane, uint32_t& tail_seen) {
    if (mask == 0) return;
    const uint32_t count = (uint32_t)__popcll(mask);
    uint32_t pos = 0;
    if (lane == 0) pos = atomicAdd(R.tail, count);
    pos = __builtin_amdgcn_readfirstlane(pos);
    if (want) R.slot[(pos + rank_below(mask)) & R.mask] = ref;
    tail_seen = pos + count;
}

// Claims up to 64 entries if at least `at_least` are waiting; returns how many (0: none) and hands
// lane k < n its entry.  head_seen, tail_seen: the ring's head and tail as last seen by this wavefront
// (the true head is never behind head_seen).
__device__ __forceinline__ int pop_clip(const ClipRing& R, uint32_t at_least, int lane, uint32_t& ref, uint32_t& head_seen,
                                        uint32_t& tail_seen) {
    uint32_t start = 0, n = 0, h = 0, t = 0;
    if (lane == 0) {
        h = __hip_atomic_load(R.head, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        for (;;) {
            t = __hip_atomic_load(R.tail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            const uint32_t waiting = t - h;
            if (waiting < at_least || waiting == 0u) break;
            const uint32_t take = min(waiting, 64u);
            const uint32_t seen = atomicCAS(R.head, h, h + take);
            if (seen == h) { start = h; n = take; h += take; break; }
            h = seen;
        }
    }
    start = __builtin_amdgcn_readfirstlane(start);
    n = __builtin_amdgcn_readfirstlane(n);
    head_seen = __builtin_amdgcn_readfirstlane(h);
    tail_seen = __builtin_amdgcn_readfirstlane(t);
    ref = kClipEmpty;
    if ((uint32_t)lane < n) {
        // The producer writes the entry right after reserving it and waits for nothing in between, so the
        // wait is a few cycles at most; it is bounded all the same, so that every wavefront leaves the
        // kernel whatever happens (a lane whose entry never turned up draws nothing).
        uint32_t* s = &R.slot[(start + (uint32_t)lane) & R.mask];
        for (int spin = 0; spin < (1 << 22); ++spin) {
            ref = __hip_atomic_load(s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (ref != kClipEmpty) break;
        }
        __hip_atomic_store(s, kClipEmpty, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    return (int)n;
}

// One lane per queued straddling triangle: clip, project, fan, hand the pieces to emit().
__device__ __forceinline__ void drain_clip(const WaveLds& L, uint32_t ref, int n, int& small_count, const SceneDev& sc,
                                           const float (&M)[16], const FrameParams& fp, const Window& win, int lane,
                                           u64* vis) {
    bool have = lane < n && ref != kClipEmpty;
    if (!have) ref = 0u;
    uint32_t c = ref >> 7, slot = ref & 127u;
    uint32_t t = gptr(sc.ctris)[(size_t)c * 128 + slot] & 0x00FFFFFFu;
    const BPS_GLOBAL float* cv = gptr(sc.cverts) + (size_t)c * 192;
    Clip4 tri[3];
    uint32_t oc_or = 0;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        uint32_t vi = (t >> (8 * k)) & 0xFFu;
        tri[k] = to_clip(M, cv[vi], cv[64 + vi], cv[128 + vi]);
        oc_or |= outcode(tri[k]);
    }
    // Polygons between passes live in private memory, and a value stored there comes back only after
    // a trip to L2.  So the first pass takes the triangle from registers, and a lane's last pass
    // projects the vertices it puts out at once (one failure drops the triangle) instead of storing
    // them for a separate projection loop: a triangle that crosses one plane never reads a polygon back.
    Clip4 px[2][kMaxPoly];
    uint32_t pxy[kMaxPoly];
    float piw[kMaxPoly];
    bool ok = true;
    int cnt = have ? 3 : 0;
    int cur = 0;
    // Planes are taken in the rule's order near, far, left, right, top, bottom, but every lane only
    // visits the planes its own triangle crosses: in pass j each lane clips against the j-th of
    // them, so a wavefront of triangles that each cross one (different) plane needs one pass, not six.
    // The plane is applied as c.x x + c.y y + c.z z + c.w w with coefficients 0 and +-1, which rounds
    // exactly like the written-out w + x, w - x, ..., z, w - z (products with 0 and +-1 and sums
    // with 0 are exact).
    uint32_t todo = ((oc_or >> 4) & 3u) | ((oc_or & 15u) << 2);      // bit p: p-th plane of the order
    if (cnt < 3) todo = 0u;
    if (ballot64(have && todo == 0u) != 0ull) {      // crosses no plane after all: the triangle as it is
        if (have && todo == 0u) {
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                bool unused;
                ok = project(tri[k], fp, pxy[k], piw[k], unused) && ok;
            }
        }
    }
    bool first_pass = true;
    ++L.tally[kTClipDrains];
    while (ballot64(todo != 0u) != 0ull) {
        ++L.tally[kTClipPasses];
        const bool active = todo != 0u;
        const int p = active ? __builtin_ctz(todo) : 0;
        todo &= todo - 1u;
        const bool last = todo == 0u;                                // this lane's final plane
        const int k = p < 2 ? p + 4 : p - 2;                         // plane number: 4 5 0 1 2 3
        const float cx = k == 0 ? 1.0f : k == 1 ? -1.0f : 0.0f, cy = k == 2 ? 1.0f : k == 3 ? -1.0f : 0.0f;
        const float cz = k == 4 ? 1.0f : k == 5 ? -1.0f : 0.0f, cw = k == 4 ? 0.0f : 1.0f;
        auto dist = [&](const Clip4& q) { return fmaf(cx, q.x, fmaf(cy, q.y, fmaf(cz, q.z, cw * q.w))); };
        if (active) {
            int m = 0;
            auto put = [&](const Clip4& q) {
                if (m < kMaxPoly) {
                    if (last) {
                        bool unused;
                        uint32_t xy;
                        float iw;
                        ok = project(q, fp, xy, iw, unused) && ok;
                        pxy[m] = xy;
                        piw[m] = iw;
                    } else {
                        px[cur ^ 1][m] = q;
                    }
                    ++m;
                }
            };
            auto step = [&](const Clip4& v, Clip4& prev, float& dprev) {
                const float dv = dist(v);
                const bool cin = dv >= 0.0f, pin = dprev >= 0.0f;
                if (cin != pin) {
                    // always from the inside vertex a to the outside vertex b
                    const Clip4 a = cin ? v : prev, b = cin ? prev : v;
                    const float da = cin ? dv : dprev, db = cin ? dprev : dv;
                    const float tt = da / (da - db);
                    Clip4 o;
                    o.x = fmaf(tt, b.x - a.x, a.x);
                    o.y = fmaf(tt, b.y - a.y, a.y);
                    o.z = fmaf(tt, b.z - a.z, a.z);
                    o.w = fmaf(tt, b.w - a.w, a.w);
                    put(o);
                }
                if (cin) put(v);
                prev = v;
                dprev = dv;
            };
            if (first_pass) {
                Clip4 prev = tri[2];
                float dprev = dist(prev);
                step(tri[0], prev, dprev);
                step(tri[1], prev, dprev);
                step(tri[2], prev, dprev);
            } else {
                Clip4 prev = px[cur][cnt - 1];
                float dprev = dist(prev);
                Clip4 ahead = px[cur][0];            // fetch one vertex ahead of its use
                for (int i = 0; i < cnt; ++i) {
                    const Clip4 v = ahead;
                    ahead = px[cur][min(i + 1, kMaxPoly - 1)];
                    step(v, prev, dprev);
                }
            }
            cnt = m;
            cur ^= 1;
            if (cnt < 3) todo = 0u;
        }
        first_pass = false;
    }
    if (cnt < 3 || !ok) cnt = 0;
    const BPS_GLOBAL uint32_t* ctri_id = gptr(sc.ctri_id);
    const uint32_t tri_ref = c * 128u + slot;
    // fan (0, i, i + 1): vertex i is the previous piece's last one, and the next one is fetched ahead
    const uint32_t a = pxy[0];
    const float wa = piw[0];
    uint32_t b = pxy[1], d_ahead = pxy[2];
    float wb = piw[1], wd_ahead = piw[2];
    for (int i = 1; ; ++i) {
        bool v = i + 1 < cnt;
        const u64 vm = ballot64(v);
        if (vm == 0) break;
        ++L.tally[kTFanIters];
        const uint32_t d = d_ahead;
        const float wd = wd_ahead;
        d_ahead = pxy[min(i + 2, kMaxPoly - 1)];
        wd_ahead = piw[min(i + 2, kMaxPoly - 1)];
        short2v lo, ext;
        const bool has = v && centre_box(a, b, d, win, lo, ext);
        emit(L, small_count, has, lo, ext, a, b, d, wa, wb, wd, tri_ref, ctri_id, lane, vis, win, ballot64(has));
        b = d;
        wb = wd;
    }
}

}  // namespace

// =============================================================================================
template <int NT, bool DIAG, int CULL, int FRAME>
__global__ __launch_bounds__(NT, 4) void k_raster(const SceneDev* __restrict__ scenes, const WorkItem* __restrict__ items,
                                               const float* __restrict__ view_proj, FrameParams fp,
                                               unsigned long long* __restrict__ gvis, float* __restrict__ out_depth,
                                               uint32_t* __restrict__ out_id, unsigned long long* __restrict__ stats_block) {
    extern __shared__ __align__(16) unsigned char smem[];
    // The DIAG = false instance carries no counters or timers at all: everything below that feeds
    // only the diagnostics record is dead code there and costs neither registers nor instructions.
    unsigned long long* const stats = DIAG ? stats_block : nullptr;
    const bool phase_timers = DIAG && fp.phase_timers == 1;
    constexpr int NW = NT / 64;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // LDS is sized for a full tile; edge tiles may be smaller.  The 64x64 instance also fixes the
    // capacity of the survivor list, so that every LDS address below is a compile-time constant.
    // FRAME = 64 or 128: an instance for square frames of that size, drawn as 64x64 windows (the
    // paper's two resolutions).  The frame parameters the loops use are constants there.
    FrameParams fq = fp;
    if (FRAME) {
        fq.H = FRAME; fq.W = FRAME; fq.tile_w = 64; fq.tile_h = 64;
        fq.sx = 128.0f * FRAME; fq.sy = 128.0f * FRAME; fq.xmax = 256.0f * FRAME + 64.0f; fq.ymax = 256.0f * FRAME + 64.0f;
    }
    const int HW = FRAME ? 64 * 64 : fp.tile_w * fp.tile_h;
    const int list_cap = FRAME ? (int)kListCap64 : fp.list_cap;

    u64* vis = reinterpret_cast<u64*>(smem);
    unsigned char* wbase = smem + (size_t)HW * 8 + (size_t)wave * kWaveLdsBytes;
    uint32_t tally[kTCount] = {};
    WaveLds L;
    L.tally = tally;
    L.stage = reinterpret_cast<float2*>(wbase);
    L.stage_oc = reinterpret_cast<uint32_t*>(wbase + 64 * 8);
    L.smallq = reinterpret_cast<uint32_t*>(wbase + 64 * 12);

    unsigned char* shared = smem + (size_t)HW * 8 + (size_t)NW * kWaveLdsBytes;
    u64* list = reinterpret_cast<u64*>(shared);                                 // [list_cap] surviving clusters
    uint16_t* order = reinterpret_cast<uint16_t*>(shared + (size_t)list_cap * 8);   // [kOrderCap] blocks, near to far
    uint16_t* perm = reinterpret_cast<uint16_t*>(shared + (size_t)list_cap * 8 + kOrderCap * 2);   // [list_cap] pop order
    uint16_t* slot_in_bin = perm + list_cap;                                                       // [list_cap]
    uint32_t* hist = reinterpret_cast<uint32_t*>(slot_in_bin + list_cap);                          // [2][kDepthBins]
    uint32_t* hiz = hist + 2 * kDepthBins;                                                            // [kHizTiles]
    uint32_t* counters = hiz + kHizTiles;
    uint32_t* list_count = counters;       // survivors appended in this round
    uint32_t* pop_count = counters + 1;    // survivors handed out in this round
    uint32_t* next_block = counters + 2;   // blocks handed out so far (whole item)
    uint32_t* reserved = counters + 3;     // upper bound on list_count once every tester has appended
    uint32_t* blocks_in_view = counters + 4;   // blocks of the item that are not wholly outside the frustum
    ClipRing ring;
    ring.tail = counters + 5;
    ring.head = counters + 6;
    ring.slot = counters + 8;
    ring.mask = clip_ring_entries(NT) - 1u;

    const WorkItem item = items[blockIdx.x];     // the host or the planner has put the items in launch order
    const SceneDev sc = scenes[item.scene];
    float M[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) M[k] = view_proj[(size_t)item.env * 16 + k];

    // this work-group's window of the frame
    const int tiles_x = (fp.W + fp.tile_w - 1) / fp.tile_w;
    Window win;
    if (FRAME == 64) {
        // the instance for 64x64 frames (the paper's main resolution): the window is the frame, and
        // with its origin and size known to the compiler the pixel arithmetic of every loop shrinks
        win.x0 = 0; win.y0 = 0; win.w = 64; win.h = 64;
        win.aL = -1.0f; win.aR = 1.0f; win.aT = -1.0f; win.aB = 1.0f;
    } else if (FRAME == 128) {
        // 128x128 frames: four windows of known size; only the origin depends on the item
        win.x0 = (int)(item.tile & 1u) * 64; win.y0 = (int)(item.tile >> 1) * 64; win.w = 64; win.h = 64;
        win.aL = (float)win.x0 * (1.0f / 64.0f) - 1.0f; win.aR = win.aL + 1.0f;
        win.aT = (float)win.y0 * (1.0f / 64.0f) - 1.0f; win.aB = win.aT + 1.0f;
    } else {
        win.x0 = (int)(item.tile % (uint32_t)tiles_x) * fp.tile_w;
        win.y0 = (int)(item.tile / (uint32_t)tiles_x) * fp.tile_h;
        win.w = min(fp.tile_w, fp.W - win.x0);
        win.h = min(fp.tile_h, fp.H - win.y0);
        win.aL = 2.0f * (float)win.x0 / (float)fp.W - 1.0f;
        win.aR = 2.0f * (float)(win.x0 + win.w) / (float)fp.W - 1.0f;
        win.aT = 2.0f * (float)win.y0 / (float)fp.H - 1.0f;
        win.aB = 2.0f * (float)(win.y0 + win.h) / (float)fp.H - 1.0f;
    }
    const int npix = win.w * win.h;
    for (int p = tid; p < npix; p += NT) vis[p] = kEmptyKey;

    int small_count = 0;
    uint32_t clip_tail_seen = 0u, clip_head_seen = 0u;    // this wavefront's last view of the clip ring
    // diagnostics (only when the host passes a counter block): per-wave tallies, one atomic each at the end
    uint32_t st_tested = 0, st_boxed = 0, st_drawn = 0, st_straddle = 0, st_hidden = 0, st_hiz = 0;
    const unsigned long long t_start = stats ? wall_clock64() : 0ull;
    // phase timers (diagnostics only): ticks[k] accumulates the time since the previous TICK
    unsigned long long t_prev = t_start;
    uint32_t ticks[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#define TICK(k) do { if (phase_timers) { unsigned long long t_ = wall_clock64(); ticks[k] += (uint32_t)(t_ - t_prev); t_prev = t_; } } while (0)
    const uint32_t full_tri_mask = 0x00FFFFFFu;
    const BPS_GLOBAL float* g_cverts = gptr(sc.cverts);
    const BPS_GLOBAL uint32_t* g_ctris = gptr(sc.ctris);
    const BPS_GLOBAL uint32_t* g_ctri_id = gptr(sc.ctri_id);
    const BPS_GLOBAL float* g_bounds = gptr(sc.cbounds);
    const uint32_t S = item.split_of >> 16, item_split = item.split_of & 0xFFFFu;
    const uint32_t nblocks_total = (sc.n_clusters + 63u) / 64u;
    const uint32_t nb_item = nblocks_total > item_split ? (nblocks_total - item_split + S - 1u) / S : 0u;
    const BPS_GLOBAL float* g_bbounds = gptr(sc.bbounds);
    // CULL is the culling level the instance is compiled for: 0 none (every cluster of the scene is
    // streamed), 1 frustum tests only, 2 frustum and occlusion tests (the default)
    constexpr bool occlusion = CULL > 1;
    const uint32_t* vis_hi = reinterpret_cast<const uint32_t*>(vis) + 1;   // depth word of pixel p is vis_hi[2 p]

    // ---- prologue: counters, and the item's blocks ordered near to far
    const bool sorted = CULL != 0 && nb_item <= kOrderCap && nb_item <= 2u * (uint32_t)list_cap && nb_item > 1;
    if (tid < 8) counters[tid] = 0u;
    for (int t = tid; t < kHizTiles; t += NT) hiz[t] = 0xFFFFFFFFu;   // nothing drawn yet: no tile hides anything
    for (uint32_t t = tid; t <= ring.mask; t += NT) ring.slot[t] = kClipEmpty;
    // the bin counts of the two counting sorts below: zero whenever no sort is under way (the wavefront
    // that turns them into offsets clears them again)
    for (int t = tid; t < kDepthBins; t += NT) hist[t] = 0u;
    __syncthreads();
    if (sorted) {
        // Counting sort of the blocks in view on the smallest clip w over the block's bounding box
        // (exactly attained at a corner), in the logarithmic depth bins of the survivor sort: any order
        // is a correct one, near to far lets occluders come first.  Blocks wholly outside one frustum
        // plane get no place in the order and are never visited.
        uint32_t* keys = reinterpret_cast<uint32_t*>(list);     // [nb_item]: bin | place in the bin << 8, or all ones
        for (uint32_t b = tid; b < nb_item; b += NT) {
            const uint32_t gb = b * S + item_split;
            float lo[3], hi[3];
#pragma unroll
            for (int a = 0; a < 3; ++a) {
                lo[a] = g_bbounds[(size_t)a * sc.b_stride + gb];
                hi[a] = g_bbounds[(size_t)(a + 3) * sc.b_stride + gb];
            }
            float wmin = M[15];
#pragma unroll
            for (int a = 0; a < 3; ++a) wmin += fminf(M[12 + a] * lo[a], M[12 + a] * hi[a]);
            uint32_t key = 0xFFFFFFFFu;
            if (!box_outside_frustum(M, win, lo[0], lo[1], lo[2], hi[0], hi[1], hi[2])) {
                // exponent and top three mantissa bits from 2^-7 upwards; boxes reaching the eye plane first
                const int k = wmin > 0.0f ? (int)(__float_as_uint(wmin) >> 20) - 120 * 8 : 0;
                const uint32_t bin = (uint32_t)min(max(k, 0), kDepthBins - 1);
                key = bin | (atomicAdd(&hist[bin], 1u) << 8);
            }
            keys[b] = key;
        }
        __syncthreads();
        if (wave == 0) {   // exclusive prefix sums of the bins: two bins per lane, shuffle scan of the pair sums
            const uint32_t h0 = hist[2 * lane], h1 = hist[2 * lane + 1];
            hist[2 * lane] = 0u;
            hist[2 * lane + 1] = 0u;
            uint32_t incl = h0 + h1;
#pragma unroll
            for (int step = 1; step < 64; step <<= 1) {
                const uint32_t up = (uint32_t)__shfl_up((int)incl, step, 64);
                if (lane >= step) incl += up;
            }
            const uint32_t before = incl - (h0 + h1);
            hist[kDepthBins + 2 * lane] = before;
            hist[kDepthBins + 2 * lane + 1] = before + h0;
            if (lane == 63) *blocks_in_view = incl;
        }
        __syncthreads();
        for (uint32_t b = tid; b < nb_item; b += NT) {
            const uint32_t key = keys[b];
            if (key != 0xFFFFFFFFu) order[hist[kDepthBins + (key & 0xFFu)] + (key >> 8)] = (uint16_t)b;
        }
    }
    __syncthreads();
    const uint32_t nb_visit = sorted ? *blocks_in_view : nb_item;

    // The item's clusters are the 64-cluster blocks split, split + S, ... of its scene, visited
    // near to far in rounds:
    //   phase A  wavefronts take blocks from the ordered list; every lane tests one cluster's
    //            bounds against the frustum and works out its screen footprint; survivors are
    //            appended (ballot + prefix count, one LDS atomic per wavefront) to the work-group's
    //            list until enough are queued or the list could overflow
    //   phase B  wavefronts pop clusters from the list one at a time; a cluster whose footprint
    //            pixels all hold nearer depths by then is skipped (one lane per footprint pixel)
    TICK(4);
    // the first round is kept short: what it draws (the nearest blocks) lets later rounds reject
    // hidden clusters before they are queued
    uint32_t round_target = occlusion ? min((uint32_t)fp.round_target, (uint32_t)fp.first_round) : (uint32_t)fp.round_target;
    const int htx = (win.w + 7) >> 3;     // Hi-Z tiles per row of the window
    bool later_round = false;             // something has been drawn: the depth buffer can reject
    for (;;) {
        for (;;) {
            if (*list_count >= round_target) break;
            uint32_t r0 = 0, blk = 0;
            if (lane == 0) r0 = atomicAdd(reserved, 64u);
            r0 = __builtin_amdgcn_readfirstlane(r0);
            if (r0 + 64u > (uint32_t)list_cap) {
                if (lane == 0) atomicSub(reserved, 64u);
                break;
            }
            if (lane == 0) blk = atomicAdd(next_block, 1u);
            blk = __builtin_amdgcn_readfirstlane(blk);
            if (blk >= nb_visit) {
                if (lane == 0) atomicSub(reserved, 64u);
                break;
            }
            const uint32_t jb = sorted ? (uint32_t)order[blk] : blk;
            if (occlusion && sorted && jb == 0xFFFFu) {      // struck out: the whole block is hidden
                if (lane == 0) atomicSub(reserved, 64u);
                continue;
            }
            ++tally[kTPhaseAPasses];
            const uint32_t cl = (jb * S + item_split) * 64u + (uint32_t)lane;
            bool visible = cl < sc.n_clusters;
            uint32_t foot = 0u, wb18 = 0u;
            st_tested += (uint32_t)__popcll(ballot64(visible));
            if (CULL != 0) {
                const uint32_t cc = visible ? cl : 0u;
                float lx = g_bounds[cc], ly = g_bounds[sc.c_stride + cc], lz = g_bounds[2 * sc.c_stride + cc];
                float hx = g_bounds[3 * sc.c_stride + cc], hy = g_bounds[4 * sc.c_stride + cc],
                      hz = g_bounds[5 * sc.c_stride + cc];
                visible = visible && !box_outside_frustum(M, win, lx, ly, lz, hx, hy, hz);
                if (occlusion && visible) {
                    foot = box_footprint(M, fq, win, lx, ly, lz, hx, hy, hz, wb18);
                    visible = foot != kNoPixel;
                    if (visible && (foot & 1u)) {
                        // coarse test against the largest depth per 8x8 tile as of the end of the last round
                        const int fx = (int)((foot >> 1) & 63u), fy = (int)((foot >> 7) & 63u);     // window-relative
                        const int bw = (int)((foot >> 13) & 31u), bh = (int)((foot >> 18) & 31u);
                        if (bw <= 7 && bh <= 7) {     // at most 2 x 2 tiles: their corners are all of them
                            const int tx0 = fx >> 3, tx1 = (fx + bw) >> 3;
                            const int ty0 = fy >> 3, ty1 = (fy + bh) >> 3;
                            uint32_t zmax = max(max(hiz[ty0 * htx + tx0], hiz[ty0 * htx + tx1]),
                                                max(hiz[ty1 * htx + tx0], hiz[ty1 * htx + tx1]));
                            if ((wb18 << 13) > zmax) visible = false;
                        }
                        // Footprints of at most 4x4 pixels are then checked pixel by pixel, all 64 clusters
                        // at once (no wavefront is drawing during this phase): the same test a wavefront
                        // would make alone when it pops the cluster, at a fortieth of the cost.
                        const bool fine = visible && later_round && bw <= 3 && bh <= 3;
                        if (ballot64(fine) != 0ull) {
                            // one footprint row per step: its up to four depth words are read together
                            const uint32_t bound = wb18 << 13;
                            int at = __mul24(fy, win.w) + fx;
                            uint32_t farthest = 0u;
                            for (int row = 0; row < 4; ++row) {
                                const bool act = fine && row <= bh;
                                if (ballot64(act) == 0ull) break;
                                const uint32_t d0 = act ? vis_hi[2 * at] : 0u;
                                const uint32_t d1 = act && bw >= 1 ? vis_hi[2 * (at + 1)] : 0u;
                                const uint32_t d2 = act && bw >= 2 ? vis_hi[2 * (at + 2)] : 0u;
                                const uint32_t d3 = act && bw >= 3 ? vis_hi[2 * (at + 3)] : 0u;
                                farthest = max(farthest, max(max(d0, d1), max(d2, d3)));
                                at += win.w;
                            }
                            if (fine && farthest < bound) visible = false;
                        }
                    }
                    st_hiz += (uint32_t)__popcll(ballot64(!visible && foot != kNoPixel));
                }
            }
            const u64 keep = ballot64(visible);
            const uint32_t n_keep = (uint32_t)__popcll(keep);
            uint32_t base = 0;
            if (lane == 0) {
                base = atomicAdd(list_count, n_keep);
                atomicSub(reserved, 64u - n_keep);
            }
            base = __builtin_amdgcn_readfirstlane(base);
            // record: cluster 23 bits | footprint 23 bits | w bound 18 bits
            if (visible) list[base + rank_below(keep)] = (u64)cl | ((u64)foot << 23) | ((u64)wb18 << 46);
        }
        TICK(1);
        __syncthreads();
        TICK(2);
        const uint32_t n_list = *list_count;
        // every block has been handed out: this is the last round (the same for all wavefronts:
        // next_block only moves during phase A)
        const bool last_round = *next_block >= nb_visit;
        if (n_list == 0 && last_round) break;
        st_boxed += wave == 0 ? n_list : 0u;

        // Order the round's survivors near to far (counting sort on a logarithmic depth key, eight
        // bins per octave) so that occluders are drawn before what they hide.
        const bool by_depth = occlusion && n_list > 64u;
        if (by_depth) {
            for (uint32_t i = tid; i < n_list; i += NT)
                slot_in_bin[i] = (uint16_t)atomicAdd(&hist[depth_bin(list[i])], 1u);
            __syncthreads();
            if (wave == 0) {   // exclusive prefix sums of the bins: two bins per lane, shuffle scan of the pair sums
                static_assert(kDepthBins == 128, "one wavefront scans two bins per lane");
                const uint32_t h0 = hist[2 * lane], h1 = hist[2 * lane + 1];
                hist[2 * lane] = 0u;      // zero again for the next sort
                hist[2 * lane + 1] = 0u;
                uint32_t incl = h0 + h1;
#pragma unroll
                for (int step = 1; step < 64; step <<= 1) {
                    const uint32_t up = (uint32_t)__shfl_up((int)incl, step, 64);
                    if (lane >= step) incl += up;
                }
                const uint32_t before = incl - (h0 + h1);
                hist[kDepthBins + 2 * lane] = before;
                hist[kDepthBins + 2 * lane + 1] = before + h0;
            }
            __syncthreads();
            if (FRAME) {
                // the instances with a fixed list capacity put the records themselves in order (every thread
                // carries its few records over a barrier), so that taking a cluster off the list is one read
                constexpr int kPerThread = ((int)kListCap64 + NT - 1) / NT;
                u64 rec[kPerThread];
                uint32_t dst[kPerThread];
#pragma unroll
                for (int k = 0; k < kPerThread; ++k) {
                    const uint32_t i = (uint32_t)tid + (uint32_t)(k * NT);
                    const bool mine = i < n_list;
                    rec[k] = mine ? list[i] : 0ull;
                    dst[k] = mine ? hist[kDepthBins + depth_bin(rec[k])] + slot_in_bin[i] : 0xFFFFFFFFu;
                }
                __syncthreads();
#pragma unroll
                for (int k = 0; k < kPerThread; ++k)
                    if (dst[k] != 0xFFFFFFFFu) list[dst[k]] = rec[k];
            } else {
                for (uint32_t i = tid; i < n_list; i += NT)
                    perm[hist[kDepthBins + depth_bin(list[i])] + slot_in_bin[i]] = (uint16_t)i;
            }
            __syncthreads();
            TICK(3);
        }

        // pop one ahead so that the next cluster's words are in flight while this one is processed;
        // a cluster whose footprint pixels all hold nearer depths by now cannot win anywhere and is
        // dropped here (one lane per footprint pixel)
        uint32_t pop = 0;
        float nx_ = 0, ny_ = 0, nz_ = 0;
        uint32_t nt0 = 0, nt1 = 0, c_next = 0;
        auto pop_visible = [&]() {
            for (;;) {
                if (lane == 0) pop = atomicAdd(pop_count, 1u);
                pop = __builtin_amdgcn_readfirstlane(pop);
                if (pop >= n_list) return;
                const u64 e = list[(by_depth && !FRAME) ? (uint32_t)perm[pop] : pop];
                const uint32_t lo32 = __builtin_amdgcn_readfirstlane((uint32_t)e);
                const uint32_t hi32 = __builtin_amdgcn_readfirstlane((uint32_t)(e >> 32));
                c_next = lo32 & 0x007FFFFFu;
                const uint32_t foot = (lo32 >> 23) | (hi32 << 9);
                if (foot & 1u) {
                    const int fx = (int)((foot >> 1) & 63u), fy = (int)((foot >> 7) & 63u);
                    const int bw = (int)((foot >> 13) & 31u), bh = (int)((foot >> 18) & 31u);
                    const uint32_t wbits = (hi32 >> 14) << 13;
                    // the wavefront covers the footprint in passes of 64 pixels: rows of 1, 2, 4, ... 32
                    // pixels (the smallest power of two that holds the width), as many rows as fit
                    const int cols_log2 = bw == 0 ? 0 : 32 - __builtin_clz((uint32_t)bw);
                    const int qx = lane & ((1 << cols_log2) - 1), qy = lane >> cols_log2;
                    const int rows_per_pass = 64 >> cols_log2;
                    bool shows = false;
                    for (int row0 = 0; row0 <= bh && !shows; row0 += rows_per_pass) {
                        ++tally[kTPopPasses];
                        const bool in = qx <= bw && row0 + qy <= bh;
                        const uint32_t d = in ? vis_hi[2 * (__mul24(fy + row0 + qy, win.w) + fx + qx)] : 0u;
                        // lanes outside the footprint read d = 0, below every bound (the bound is a positive float)
                        shows = ballot64(d >= wbits) != 0ull;
                    }
                    if (!shows) { ++st_hidden; continue; }
                }
                const BPS_GLOBAL float* cv = g_cverts + (size_t)c_next * 192;
                nx_ = cv[lane]; ny_ = cv[64 + lane]; nz_ = cv[128 + lane];
                const BPS_GLOBAL uint32_t* ct = g_ctris + (size_t)c_next * 128;
                nt0 = ct[lane]; nt1 = ct[64 + lane];
                return;
            }
        };
        pop_visible();
        while (pop < n_list) {
            const uint32_t c = c_next;
            float x = nx_, y = ny_, z = nz_;
            uint32_t t0 = nt0, t1 = nt1;
            pop_visible();

            // ---- vertex phase
            Clip4 cp = to_clip(M, x, y, z);
            bool o0 = !(cp.w + cp.x >= 0.0f), o1 = !(cp.w - cp.x >= 0.0f);
            bool o2 = !(cp.w + cp.y >= 0.0f), o3 = !(cp.w - cp.y >= 0.0f);
            bool o4 = !(cp.z >= 0.0f), o5 = !(cp.w - cp.z >= 0.0f);
            bool culled = ballot64(o0) == ~0ull || ballot64(o1) == ~0ull || ballot64(o2) == ~0ull ||
                          ballot64(o3) == ~0ull || ballot64(o4) == ~0ull || ballot64(o5) == ~0ull;
            ++tally[kTClusters];
            if (culled) continue;
            ++st_drawn;
            uint32_t oc = (o0 ? 1u : 0u) | (o1 ? 2u : 0u) | (o2 ? 4u : 0u) | (o3 ? 8u : 0u) | (o4 ? 16u : 0u) |
                          (o5 ? 32u : 0u);
            if (!all_finite(cp)) oc |= kInvalid;
            uint32_t xy;
            float iw;
            bool can_project;
            bool ok = project(cp, fq, xy, iw, can_project);
            if (oc == 0 && !ok) oc = kInvalid;
            if (!can_project) oc |= kNoProject;
            const bool all_inside = ballot64(oc != 0) == 0;
            wave_lds_sync();   // earlier reads of the stage are done
            // the slot index is laundered so that its LDS address is recomputed here (one add) rather
            // than kept in a register across the whole loop, where it was spilled and its reload
            // made the wavefront wait for the cluster prefetch as well
            int stage_slot = lane;
            asm volatile("" : "+v"(stage_slot));
            L.stage[stage_slot] = make_float2(__uint_as_float(xy), iw);
            if (!all_inside) L.stage_oc[stage_slot] = oc;
            wave_lds_sync();

            // ---- triangle phase: two slots per lane
            const int ntri = __builtin_amdgcn_readfirstlane((int)(t0 >> 24));
#pragma unroll 1
            for (int slot = 0; slot < 2; ++slot) {
                if (slot == 1 && ntri <= 64) break;
                ++tally[kTSlots];
                uint32_t t = (slot == 0 ? t0 : t1) & full_tri_mask;
                const uint32_t i0 = t & 0xFFu, i1 = (t >> 8) & 0xFFu, i2 = t >> 16;
                float2 a = L.stage[i0], b = L.stage[i1], d = L.stage[i2];
                bool fast = slot * 64 + lane < ntri;
                u64 fast_mask = ballot64(fast);      // masks are combined on the scalar unit
                short2v lo, ext;
                const bool has = centre_box(__float_as_uint(a.x), __float_as_uint(b.x), __float_as_uint(d.x), win, lo, ext);
                const u64 has_mask = ballot64(has);
                if (!all_inside) {
                    uint32_t oa = L.stage_oc[i0], ob = L.stage_oc[i1], od = L.stage_oc[i2];
                    uint32_t o_or = oa | ob | od, o_and = oa & ob & od;
                    const bool sound = (o_or & kInvalid) == 0, apart = (o_and & 0x3Fu) == 0, crossing = (o_or & 0x3Fu) != 0;
                    const bool behind = (o_or & kNoProject) != 0;
                    const bool live = fast && sound && apart;
                    const u64 live_mask = fast_mask & ballot64(sound) & ballot64(apart), crossing_mask = ballot64(crossing);
                    fast = live && !crossing;
                    fast_mask = live_mask & ~crossing_mask;
                    // A straddler whose three vertices all project (w > 0) cannot reach a pixel centre
                    // outside the box of its projected vertices: only the others need the clipper.
                    const bool straddle = live && crossing && (has || behind);
                    const u64 straddle_mask = live_mask & crossing_mask & (has_mask | ballot64(behind));
                    st_straddle += (uint32_t)__popcll(straddle_mask);
                    push_clip(ring, straddle, (c << 7) | (uint32_t)(slot * 64 + lane), straddle_mask, lane, clip_tail_seen);
                }
                emit(L, small_count, fast && has, lo, ext, __float_as_uint(a.x), __float_as_uint(b.x),
                     __float_as_uint(d.x), a.y, b.y, d.y, c * 128u + (uint32_t)(slot * 64 + lane), g_ctri_id, lane, vis,
                     win, fast_mask & has_mask);
            }
            // ---- clip ring: full wavefronts only while streaming.  The ring is looked at only when this
            // wavefront's own view says 64 may be waiting: its view of the tail dates from its last push, its
            // view of the head is never ahead of the head, so every push that leaves 64 or more waiting is
            // followed by a look.
            while (clip_tail_seen - clip_head_seen >= 64u) {
                uint32_t ref;
                const int n = pop_clip(ring, 64u, lane, ref, clip_head_seen, clip_tail_seen);
                if (n == 0) break;
                wave_lds_sync();
                drain_clip(L, ref, n, small_count, sc, M, fq, win, lane, vis);
            }
        }
        TICK(5);
        // After the last round a wavefront goes straight on to flush its queues, without waiting for
        // the others: the flush (one pass of the clipper, mostly waiting for memory) then overlaps the
        // clusters the slower wavefronts are still drawing.
        if (last_round) break;
        // What the wavefront has queued goes into the depth buffer now, so that the depth tiles and the
        // next round's tests see everything this round drew.  Triangles waiting for the clipper are the
        // ones along the window's border: until they are drawn, no footprint that touches a border
        // pixel can be found hidden.
        if (occlusion) {
            for (;;) {
                uint32_t ref;
                const int n = pop_clip(ring, 1u, lane, ref, clip_head_seen, clip_tail_seen);
                if (n == 0) break;
                wave_lds_sync();
                drain_clip(L, ref, n, small_count, sc, M, fq, win, lane, vis);
            }
        }
        if (occlusion && small_count > 0) {
            wave_lds_sync();
            drain_small(L, small_count, lane, vis, win, g_ctri_id);
            wave_lds_sync();
            small_count = 0;
        }
        __syncthreads();
        if (tid == 0) { *list_count = 0u; *pop_count = 0u; *reserved = 0u; }
        if (occlusion) {   // (more blocks are waiting, or the loop would have ended above)
            // Whole blocks are tested against the new depth tiles as well: thread k takes the k-th block
            // still waiting.  Its bounds are fetched now and arrive while the tiles are being built.
            const uint32_t waiting_from = *next_block;      // stable: it only moves during phase A
            float blo[3] = {0.0f, 0.0f, 0.0f}, bhi[3] = {0.0f, 0.0f, 0.0f};
            uint32_t my_rank = waiting_from + (uint32_t)tid;
            bool my_block = sorted && my_rank < nb_visit && order[my_rank] != 0xFFFFu;
            if (my_block) {
                const uint32_t gb = (uint32_t)order[my_rank] * S + item_split;
#pragma unroll
                for (int a = 0; a < 3; ++a) {
                    blo[a] = g_bbounds[(size_t)a * sc.b_stride + gb];
                    bhi[a] = g_bbounds[(size_t)(a + 3) * sc.b_stride + gb];
                }
            }
            // Hi-Z: largest stored depth word per 8x8-pixel tile of the window (empty pixels read as
            // 0xFFFFFFFF); one thread per tile row reads its eight words, eight neighbouring lanes hold the
            // rows of one tile (a 64x64 window is one pass of the 512 threads)
            const int hty = (win.h + 7) >> 3;
            for (int u = tid; u < htx * hty * 8; u += NT) {
                const int t = u >> 3, py = ((t / htx) << 3) + (u & 7), px0 = (t % htx) << 3;
                uint32_t dbits = 0u;
                if (py < win.h) {
                    const uint32_t* row = vis_hi + 2 * (__mul24(py, win.w) + px0);
#pragma unroll
                    for (int k = 0; k < 8; ++k) dbits = max(dbits, px0 + k < win.w ? row[2 * k] : 0u);
                }
#pragma unroll
                for (int sh = 4; sh >= 1; sh >>= 1) dbits = max(dbits, (uint32_t)__shfl_xor((int)dbits, sh, 64));
                if ((u & 7) == 0) hiz[t] = dbits;
            }
            __syncthreads();
            // A block whose box lies behind the largest depth of every tile its footprint touches hides
            // all of its clusters (their boxes are inside it; depths only ever decrease): its entry in
            // the visiting order is struck out and phase A passes over it.
            if (my_block) {
                uint32_t wb18 = 0u;
                const uint32_t foot = box_footprint(M, fq, win, blo[0], blo[1], blo[2], bhi[0], bhi[1], bhi[2], wb18);
                bool dead = foot == kNoPixel;
                if (!dead && (foot & 1u)) {
                    const int fx = (int)((foot >> 1) & 63u), fy = (int)((foot >> 7) & 63u);
                    const int bw = (int)((foot >> 13) & 31u), bh = (int)((foot >> 18) & 31u);
                    uint32_t zmax = 0u;
                    for (int ty = fy >> 3; ty <= (fy + bh) >> 3; ++ty)
                        for (int tx = fx >> 3; tx <= (fx + bw) >> 3; ++tx) zmax = max(zmax, hiz[ty * htx + tx]);
                    dead = (wb18 << 13) > zmax;
                }
                if (dead) order[my_rank] = 0xFFFFu;
            }
        }
        round_target = (uint32_t)fp.round_target;
        later_round = true;
        __syncthreads();
        TICK(6);
    }
    // whatever a wavefront that is still drawing adds later, that wavefront takes when it gets here
    for (;;) {
        uint32_t ref;
        const int n = pop_clip(ring, 1u, lane, ref, clip_head_seen, clip_tail_seen);
        if (n == 0) break;
        wave_lds_sync();
        drain_clip(L, ref, n, small_count, sc, M, fq, win, lane, vis);
    }
    if (small_count > 0) {
        wave_lds_sync();
        drain_small(L, small_count, lane, vis, win, g_ctri_id);
    }
    TICK(7);
    if (stats) __syncthreads();   // the record below reuses the survivor list: every wavefront must be done with it
    // diagnostics: per-wave tallies go through LDS (the survivor list is free by now) and leave as
    // one record of 16 words per work-group, without atomics
    if (stats && lane == 0) {
        uint32_t* rec = reinterpret_cast<uint32_t*>(list) + wave * 16;
        const uint32_t dt = (uint32_t)(wall_clock64() - t_start);
        rec[0] = st_tested; rec[1] = st_boxed; rec[2] = st_drawn; rec[3] = st_straddle; rec[4] = st_hidden; rec[5] = dt;
        rec[6] = tally[kTSmall]; rec[7] = tally[kTLarge]; rec[8] = st_hiz;
        for (int k = 1; k < 8; ++k) rec[8 + k] = ticks[k];
        // path tallies instead of the phase timers: first or second half of them
        if (fp.phase_timers == 2) for (int k = 0; k < 7; ++k) rec[9 + k] = tally[2 + k];
        if (fp.phase_timers == 3) for (int k = 0; k < 7; ++k) rec[9 + k] = tally[9 + k];
        if (fp.phase_timers == 0) {
            // without phase timers the last words tell where and when the group ran: the sum of the
            // wavefronts' durations (against word 5: how unevenly they finish), the environment, start
            // and end on the device-wide 100 MHz clock, and the hardware id (compute unit, shader
            // engine in the low 24 bits, die above)
            rec[12] = dt;
            if (wave == 0) {
                rec[11] = item.env;
                rec[13] = (uint32_t)t_start;
                rec[14] = (uint32_t)wall_clock64();
                rec[15] = (__builtin_amdgcn_s_getreg((31 << 11) | 4) & 0xFFFFFFu) |
                          (__builtin_amdgcn_s_getreg((3 << 11) | 20) << 24);
            }
        }
    }
    __syncthreads();
    if (stats && tid < 16) {
        const uint32_t* rec = reinterpret_cast<const uint32_t*>(list);
        unsigned long long sum = 0, mx = 0;
        for (int w = 0; w < NW; ++w) { sum += rec[w * 16 + tid]; mx = max(mx, (unsigned long long)rec[w * 16 + tid]); }
        stats[(size_t)blockIdx.x * 16 + tid] = tid == 5 ? mx : sum;      // word 5: longest wavefront of the group
    }

    // ---- resolve this work-group's frame
    const size_t base = (size_t)item.env * fq.H * fq.W;
    for (int p = tid; p < npix; p += NT) {
        const int y = p / win.w, x = p - y * win.w;
        const size_t o = base + (size_t)(win.y0 + y) * fq.W + (size_t)(win.x0 + x);
        const u64 key = vis[p];
        const bool hit = key != kEmptyKey;
        if (fp.merge) {
            if (hit) atomicMin(&gvis[o], key);
        } else {
            out_depth[o] = hit ? __uint_as_float((uint32_t)(key >> 32)) : fp.background;
            if (out_id) out_id[o] = hit ? (uint32_t)key : 0xFFFFFFFFu;
        }
    }
}

// Resolve of the global visibility buffer (used when an environment was split over several
// work-groups); leaves the buffer cleared for the next request.
__global__ void k_resolve(unsigned long long* __restrict__ gvis, size_t n, float background,
                          float* __restrict__ out_depth, uint32_t* __restrict__ out_id) {
    size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n) return;
    u64 key = gvis[p];
    bool hit = key != kEmptyKey;
    out_depth[p] = hit ? __uint_as_float((uint32_t)(key >> 32)) : background;
    if (out_id) out_id[p] = hit ? (uint32_t)key : 0xFFFFFFFFu;
    if (hit) gvis[p] = kEmptyKey;
}

// Launch planning.  Work-groups are dispatched in index order, so handing out the most expensive
// items first (longest processing time first) shortens the tail of the launch.  An item's cost
// is estimated as the number of its scene's 64-cluster blocks that are not wholly outside the
// environment's frustum; k_dispatch_order then sorts all items by decreasing cost.
__global__ __launch_bounds__(64) void k_item_cost(const SceneDev* __restrict__ scenes, const WorkItem* __restrict__ items,
                                                  const float* __restrict__ view_proj, FrameParams fp, uint32_t n_items,
                                                  uint32_t* __restrict__ cost) {
    const uint32_t i = blockIdx.x;
    if (i >= n_items) return;
    const WorkItem item = items[i];
    const SceneDev sc = scenes[item.scene];
    float M[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) M[k] = view_proj[(size_t)item.env * 16 + k];
    const BPS_GLOBAL float* bb = gptr(sc.bbounds);
    const uint32_t nblocks = (sc.n_clusters + 63u) / 64u;
    const uint32_t S = item.split_of >> 16, item_split = item.split_of & 0xFFFFu;
    const int tiles_x = (fp.W + fp.tile_w - 1) / fp.tile_w;
    Window win;
    win.x0 = (int)(item.tile % (uint32_t)tiles_x) * fp.tile_w;
    win.y0 = (int)(item.tile / (uint32_t)tiles_x) * fp.tile_h;
    win.w = min(fp.tile_w, fp.W - win.x0);
    win.h = min(fp.tile_h, fp.H - win.y0);
    win.aL = 2.0f * (float)win.x0 / (float)fp.W - 1.0f;
    win.aR = 2.0f * (float)(win.x0 + win.w) / (float)fp.W - 1.0f;
    win.aT = 2.0f * (float)win.y0 / (float)fp.H - 1.0f;
    win.aB = 2.0f * (float)(win.y0 + win.h) / (float)fp.H - 1.0f;
    uint32_t count = 0;
    for (uint32_t gb = item_split + S * threadIdx.x; gb < nblocks; gb += S * 64u) {
        float lx = bb[gb], ly = bb[sc.b_stride + gb], lz = bb[2 * sc.b_stride + gb];
        float hx = bb[3 * sc.b_stride + gb], hy = bb[4 * sc.b_stride + gb], hz = bb[5 * sc.b_stride + gb];
        count += box_outside_frustum(M, win, lx, ly, lz, hx, hy, hz) ? 0u : 1u;
    }
#pragma unroll
    for (int sh = 32; sh >= 1; sh >>= 1) count += (uint32_t)__shfl_xor((int)count, sh, 64);
    if (threadIdx.x == 0) cost[i] = count;
}

// Dispatch order = all items by decreasing estimated cost (counting sort over 2048 linear cost
// buckets): consecutive work-group indices go to consecutive dies, so every die receives an even
// sample of the cost distribution, costliest first.
__global__ __launch_bounds__(1024) void k_dispatch_order(const uint32_t* __restrict__ cost, uint32_t n_items,
                                                         const WorkItem* __restrict__ items, WorkItem* __restrict__ ordered) {
    constexpr uint32_t kBuckets = 2048;
    constexpr int kPerThread = (int)(kMaxPlannedItems / 1024u);      // every thread keeps its items' costs in registers
    __shared__ uint32_t bucket[kBuckets];
    __shared__ uint32_t scan[1024];
    static_assert(kMaxPlannedItems <= 65536u, "item indices are kept as 16-bit words");
    __shared__ uint16_t order_lds[kMaxPlannedItems];                  // the order, before the die-affinity pass
    __shared__ uint32_t largest;
    const uint32_t tid = threadIdx.x;
    uint32_t my_cost[kPerThread];
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
        const uint32_t i = tid + (uint32_t)k * 1024u;
        my_cost[k] = i < n_items ? cost[i] : 0u;
    }
    for (uint32_t b = tid; b < kBuckets; b += 1024u) bucket[b] = 0u;
    if (tid == 0) largest = 0u;
    __syncthreads();
    {
        uint32_t mx = 0;
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) mx = max(mx, my_cost[k]);
#pragma unroll
        for (int sh = 32; sh >= 1; sh >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, sh, 64));
        if ((tid & 63u) == 0u) atomicMax(&largest, mx);
    }
    __syncthreads();
    const float scale = largest ? (float)(kBuckets - 1) / (float)largest : 0.0f;
    auto bucket_of = [&](uint32_t c) -> uint32_t {      // bucket 0 holds the costliest items
        return kBuckets - 1u - min((uint32_t)((float)c * scale), kBuckets - 1u);
    };
    uint32_t my_slot[kPerThread];      // position inside the bucket
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
        const uint32_t i = tid + (uint32_t)k * 1024u;
        my_slot[k] = i < n_items ? atomicAdd(&bucket[bucket_of(my_cost[k])], 1u) : 0u;
    }
    __syncthreads();
    // exclusive prefix sum over the buckets: two per thread, then a scan over the 1024 pair sums
    const uint32_t a0 = bucket[2 * tid], a1 = bucket[2 * tid + 1];
    // inclusive scan of the 1024 pair sums: within each wavefront by shuffles, then over the 16
    // wavefront totals
    uint32_t incl = a0 + a1;
#pragma unroll
    for (int step = 1; step < 64; step <<= 1) {
        const uint32_t up = (uint32_t)__shfl_up((int)incl, step, 64);
        if ((tid & 63u) >= (uint32_t)step) incl += up;
    }
    if ((tid & 63u) == 63u) scan[tid >> 6] = incl;
    __syncthreads();
    uint32_t offset = 0;
    for (uint32_t wv = 0; wv < (tid >> 6); ++wv) offset += scan[wv];
    const uint32_t before = offset + incl - (a0 + a1);
    __syncthreads();       // scan[] is reused below, bucket[] is overwritten now
    bucket[2 * tid] = before;
    bucket[2 * tid + 1] = before + a0;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
        const uint32_t i = tid + (uint32_t)k * 1024u;
        if (i < n_items) order_lds[bucket[bucket_of(my_cost[k])] + my_slot[k]] = (uint16_t)i;
    }
    __syncthreads();
    // Die affinity.  Position p of the order runs on die p % 8, and the host lays the items out so
    // that item i's scene is mostly used by items with the same i % 8.  Within every run of 64
    // consecutive positions (items of nearly equal cost, eight positions per die) the items are
    // rearranged so that as many as possible land on their own die; each die still gets eight
    // items of every cost class, but now finds its scenes in its own L2.
    uint32_t* slot_item = scan;                       // [16 waves][64]: the window being rebuilt
    const uint32_t lane = tid & 63u, wave = tid >> 6;
    for (uint32_t base = wave * 64u; base + 64u <= n_items; base += 1024u) {
        const uint32_t item = (uint32_t)order_lds[base + lane];
        const uint32_t home = item & 7u;
        uint32_t* mine = slot_item + wave * 64u;
        mine[lane] = 0xFFFFFFFFu;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        bool placed = false;
        for (uint32_t d = 0; d < 8u; ++d) {
            const unsigned long long want = __builtin_amdgcn_ballot_w64(home == d);
            const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(want >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)want, 0u));
            if (home == d && rank < 8u) {
                mine[rank * 8u + d] = item;
                placed = true;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // the rest take the free positions in order
        const unsigned long long free_mask = __builtin_amdgcn_ballot_w64(mine[lane] == 0xFFFFFFFFu);
        const unsigned long long left_mask = __builtin_amdgcn_ballot_w64(!placed);
        if (!placed) {
            uint32_t r = __builtin_amdgcn_mbcnt_hi((uint32_t)(left_mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)left_mask, 0u));
            unsigned long long m = free_mask;
            for (uint32_t k = 0; k < r; ++k) m &= m - 1ull;      // drop the r lowest free positions
            mine[__builtin_ctzll(m)] = item;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // the raster kernel reads its item at its own work-group index: one dependent load fewer
        // than going through the order
        ordered[base + lane] = items[mine[lane]];
    }
    for (uint32_t i = (n_items & ~63u) + tid; i < n_items; i += 1024u) ordered[i] = items[order_lds[i]];
}

void launch_plan(hipStream_t stream, const SceneDev* scenes, const WorkItem* items, const float* view_proj,
                 const FrameParams& fp, uint32_t n_items, uint32_t* cost, WorkItem* ordered) {
    hipLaunchKernelGGL(k_item_cost, dim3(n_items), dim3(64), 0, stream, scenes, items, view_proj, fp, n_items, cost);
    hipLaunchKernelGGL(k_dispatch_order, dim3(1), dim3(1024), 0, stream, cost, n_items, items, ordered);
}

__global__ __launch_bounds__(64) void k_unpack_items(PackedItems packed, uint32_t first, uint32_t count,
                                                     WorkItem* __restrict__ items) {
    const uint32_t k = blockIdx.x * 64u + threadIdx.x;
    if (k >= count) return;
    const uint32_t w = packed.word[k];
    WorkItem it;
    it.env = w & 0xFFFFu;
    it.scene = (w >> 16) & 0xFFFu;
    it.split_of = 1u << 16;
    it.tile = w >> 28;
    items[first + k] = it;
}

void launch_unpack_items(hipStream_t stream, const PackedItems& packed, uint32_t first, uint32_t count, WorkItem* items) {
    hipLaunchKernelGGL(k_unpack_items, dim3((count + 63u) / 64u), dim3(64), 0, stream, packed, first, count, items);
}

__global__ void k_zero_words(unsigned long long* __restrict__ p, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

__global__ void k_fill_keys(unsigned long long* __restrict__ gvis, size_t n) {
    size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n) gvis[p] = kEmptyKey;
}

namespace {
template <bool DIAG, int CULL>
const void* raster_entry(int threads) {
    return threads == 256   ? reinterpret_cast<const void*>(&k_raster<256, DIAG, CULL, 0>)
           : threads == 384 ? reinterpret_cast<const void*>(&k_raster<384, DIAG, CULL, 0>)
           : threads == 512 ? reinterpret_cast<const void*>(&k_raster<512, DIAG, CULL, 0>)
                            : reinterpret_cast<const void*>(&k_raster<1024, DIAG, CULL, 0>);
}
}  // namespace

hipError_t prepare_raster(int threads, size_t lds) {
    const void* entries[6] = {raster_entry<false, 0>(threads), raster_entry<false, 1>(threads), raster_entry<false, 2>(threads),
                              raster_entry<true, 0>(threads),  raster_entry<true, 1>(threads),  raster_entry<true, 2>(threads)};
    for (const void* f : entries) {
        hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_raster<512, false, 2, 64>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_raster<512, false, 2, 128>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
}

void launch_raster(int threads, dim3 grid, size_t lds, hipStream_t stream, const SceneDev* scenes, const WorkItem* items,
                   const float* view_proj, const FrameParams& fp, unsigned long long* gvis, float* out_depth,
                   uint32_t* out_id, unsigned long long* stats) {
    // 64x64 and 128x128 frames in the default configuration have instances of their own
    if (threads == 512 && !stats && fp.cull == 2 && fp.tile_w == 64 && fp.tile_h == 64 && fp.list_cap == (int)kListCap64) {
        if (fp.W == 64 && fp.H == 64) {
            hipLaunchKernelGGL((k_raster<512, false, 2, 64>), grid, dim3(512), lds, stream, scenes, items, view_proj, fp, gvis,
                               out_depth, out_id, stats);
            return;
        }
        if (fp.W == 128 && fp.H == 128) {
            hipLaunchKernelGGL((k_raster<512, false, 2, 128>), grid, dim3(512), lds, stream, scenes, items, view_proj, fp, gvis,
                               out_depth, out_id, stats);
            return;
        }
    }
#define BPS_LAUNCH3(NT, DIAG, CULL)                                                                                    \
    hipLaunchKernelGGL((k_raster<NT, DIAG, CULL, 0>), grid, dim3(NT), lds, stream, scenes, items, view_proj, fp, gvis,          \
                       out_depth, out_id, stats)
#define BPS_LAUNCH2(NT, DIAG)                                                                                          \
    do {                                                                                                               \
        if (fp.cull == 0) BPS_LAUNCH3(NT, DIAG, 0);                                                                    \
        else if (fp.cull == 1) BPS_LAUNCH3(NT, DIAG, 1);                                                               \
        else BPS_LAUNCH3(NT, DIAG, 2);                                                                                 \
    } while (0)
#define BPS_LAUNCH(NT)                                                                                                 \
    do {                                                                                                               \
        if (stats) BPS_LAUNCH2(NT, true);                                                                              \
        else BPS_LAUNCH2(NT, false);                                                                                   \
    } while (0)
    if (threads == 256) BPS_LAUNCH(256);
    else if (threads == 384) BPS_LAUNCH(384);
    else if (threads == 512) BPS_LAUNCH(512);
    else BPS_LAUNCH(1024);
#undef BPS_LAUNCH
#undef BPS_LAUNCH2
#undef BPS_LAUNCH3
}

}  // namespace bps
