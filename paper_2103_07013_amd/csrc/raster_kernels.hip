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
    uint32_t* clipq;    // [192] cluster << 7 | slot
};

// One lane per queued small triangle: at most kSmallMax pixel centres each.
__device__ __forceinline__ void drain_small(const WaveLds& L, int n, int lane, u64* vis, int W) {
    bool have = lane < n;
    uint32_t xy0 = L.smallq[0 * 64 + lane], xy1 = L.smallq[1 * 64 + lane], xy2 = L.smallq[2 * 64 + lane];
    float iw0 = __uint_as_float(L.smallq[3 * 64 + lane]), iw1 = __uint_as_float(L.smallq[4 * 64 + lane]),
          iw2 = __uint_as_float(L.smallq[5 * 64 + lane]);
    uint32_t id = L.smallq[6 * 64 + lane], box = L.smallq[7 * 64 + lane];
    Setup s = make_setup(xy0, xy1, xy2, iw0, iw1, iw2);
    int i_lo = (int)(box & 0xFFu), j_lo = (int)((box >> 8) & 0xFFu);
    int nx = (int)((box >> 16) & 0xFFu), ny = (int)(box >> 24);
    int cnt = have ? nx * ny : 0;
    int i = i_lo, j = j_lo;
    for (int k = 0; k < kSmallMax; ++k) {
        bool act = k < cnt;
        if (ballot64(act) == 0) break;
        shade_pixel(s, i, j, act, id, vis, W);
        ++i;
        if (i >= i_lo + nx) { i = i_lo; ++j; }
    }
}

// Append small triangles to the wave's queue; whenever it reaches 64 entries, drain them.
__device__ __forceinline__ void push_small(const WaveLds& L, int& count, bool want, uint32_t xy0, uint32_t xy1,
                                           uint32_t xy2, float iw0, float iw1, float iw2, uint32_t id, uint32_t box,
                                           int lane, u64* vis, int W) {
    u64 mask = ballot64(want);
    if (mask == 0) return;
    int n = __popcll(mask);
    int rank = (int)rank_below(mask);
    int room = 64 - count;
    int pos = count + rank;            // position if the queue were unbounded
    bool first = want && rank < room;
    bool later = want && !first;
    if (first) {
        L.smallq[0 * 64 + pos] = xy0; L.smallq[1 * 64 + pos] = xy1; L.smallq[2 * 64 + pos] = xy2;
        L.smallq[3 * 64 + pos] = __float_as_uint(iw0); L.smallq[4 * 64 + pos] = __float_as_uint(iw1);
        L.smallq[5 * 64 + pos] = __float_as_uint(iw2);
        L.smallq[6 * 64 + pos] = id; L.smallq[7 * 64 + pos] = box;
    }
    if (n >= room) {
        wave_lds_sync();
        drain_small(L, 64, lane, vis, W);
        wave_lds_sync();
        pos -= 64;
        if (later) {
            L.smallq[0 * 64 + pos] = xy0; L.smallq[1 * 64 + pos] = xy1; L.smallq[2 * 64 + pos] = xy2;
            L.smallq[3 * 64 + pos] = __float_as_uint(iw0); L.smallq[4 * 64 + pos] = __float_as_uint(iw1);
            L.smallq[5 * 64 + pos] = __float_as_uint(iw2);
            L.smallq[6 * 64 + pos] = id; L.smallq[7 * 64 + pos] = box;
        }
        count = n - room;
    } else {
        count += n;
    }
}

// Whole wavefront on one large triangle: 8x8 pixel blocks over its bounding box.
__device__ __forceinline__ void raster_large(uint32_t xy0, uint32_t xy1, uint32_t xy2, float iw0, float iw1, float iw2,
                                             uint32_t id, int i_lo, int i_hi, int j_lo, int j_hi, int lane, u64* vis,
                                             int W) {
    Setup s = make_setup(xy0, xy1, xy2, iw0, iw1, iw2);
    int li = lane & 7, lj = lane >> 3;
    for (int by = j_lo >> 3; by <= (j_hi >> 3); ++by) {
        int j = (by << 3) + lj;
        bool jok = j >= j_lo && j <= j_hi;
        for (int bx = i_lo >> 3; bx <= (i_hi >> 3); ++bx) {
            int i = (bx << 3) + li;
            bool act = jok && i >= i_lo && i <= i_hi;
            shade_pixel(s, i, j, act, id, vis, W);
        }
    }
}

typedef short short2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ short2v as_s2(uint32_t v) { return __builtin_bit_cast(short2v, v); }
__device__ __forceinline__ uint32_t as_u32(short2v v) { return __builtin_bit_cast(uint32_t, v); }

// Bounding-box cull, classification and hand-off of one candidate triangle per lane.
// Works on both axes at once with packed 16-bit arithmetic.  Pixel i has its centre at
// 256 (i - 64) + 128 in packed coordinates, so the first centre at or right of x is
// (x + 127) >> 8 and the last centre at or left of x is (x - 128) >> 8 (both minus 64).
// id_ptr is only dereferenced by lanes whose triangle can touch a pixel centre.
__device__ __forceinline__ void emit(const WaveLds& L, int& small_count, bool valid, uint32_t xy0, uint32_t xy1,
                                     uint32_t xy2, float iw0, float iw1, float iw2, const BPS_GLOBAL uint32_t* id_ptr,
                                     int lane, u64* vis, int H, int W) {
    short2v a = as_s2(xy0), b = as_s2(xy1), c = as_s2(xy2);
    short2v mn = __builtin_elementwise_min(a, __builtin_elementwise_min(b, c));
    short2v mx = __builtin_elementwise_max(a, __builtin_elementwise_max(b, c));
    short2v lo = (mn + (short)127) >> (short)8;
    short2v hi = (mx - (short)128) >> (short)8;
    short2v lo_clamp = {(short)-64, (short)-64};
    short2v hi_clamp = {(short)(W - 65), (short)(H - 65)};
    lo = __builtin_elementwise_max(lo, lo_clamp);
    hi = __builtin_elementwise_min(hi, hi_clamp);
    short2v ext = hi - lo;                              // both halves >= 0: some pixel centre is inside
    valid = valid && (as_u32(ext) & 0x80008000u) == 0;
    u64 vmask = ballot64(valid);
    if (vmask == 0) return;
    uint32_t id = valid ? *id_ptr : 0u;
    int nx = (int)ext.x + 1, ny = (int)ext.y + 1;
    int i_lo = (int)lo.x + 64, j_lo = (int)lo.y + 64;
    bool small = valid && nx * ny <= kSmallMax;
    uint32_t box = (uint32_t)i_lo | ((uint32_t)j_lo << 8) | ((uint32_t)nx << 16) | ((uint32_t)ny << 24);
    push_small(L, small_count, small, xy0, xy1, xy2, iw0, iw1, iw2, id, box, lane, vis, W);
    u64 big = ballot64(valid && !small);
    while (big) {
        int src = __builtin_ctzll(big);
        big &= big - 1;
        int bi = bcast_i(i_lo, src), bj = bcast_i(j_lo, src);
        raster_large((uint32_t)bcast_i((int)xy0, src), (uint32_t)bcast_i((int)xy1, src), (uint32_t)bcast_i((int)xy2, src),
                     bcast_f(iw0, src), bcast_f(iw1, src), bcast_f(iw2, src), (uint32_t)bcast_i((int)id, src), bi,
                     bi + bcast_i(nx, src) - 1, bj, bj + bcast_i(ny, src) - 1, lane, vis, W);
    }
}

// Conservative test of an axis-aligned box against the six frustum planes of M, in world
// space.  For plane (row3 +- rowk) . (v, 1) >= 0 the largest value over the box is compared
// with a negative margin proportional to the magnitude of the terms, so that rounding in this
// test and in the per-vertex transform can never cull a box holding a vertex the exact rule
// keeps.  NaNs compare false and therefore never cull.
__device__ __forceinline__ bool box_outside_frustum(const float (&M)[16], float lx, float ly, float lz, float hx,
                                                    float hy, float hz) {
    const float eps = 1.52587890625e-05f;   // 2^-16
    float ax = fmaxf(fabsf(lx), fabsf(hx)), ay = fmaxf(fabsf(ly), fabsf(hy)), az = fmaxf(fabsf(lz), fabsf(hz));
    bool outside = false;
#pragma unroll
    for (int k = 0; k < 6; ++k) {
        const int r = (k < 2) ? 0 : (k < 4) ? 1 : 2;
        float px, py, pz, pw, qx, qy, qz, qw;   // plane coefficients and their magnitudes
        if (k == 4) {
            px = M[8]; py = M[9]; pz = M[10]; pw = M[11];
            qx = fabsf(px); qy = fabsf(py); qz = fabsf(pz); qw = fabsf(pw);
        } else {
            const float sg = (k == 0 || k == 2) ? 1.0f : -1.0f;
            px = M[12] + sg * M[4 * r + 0]; py = M[13] + sg * M[4 * r + 1];
            pz = M[14] + sg * M[4 * r + 2]; pw = M[15] + sg * M[4 * r + 3];
            qx = fabsf(M[12]) + fabsf(M[4 * r + 0]); qy = fabsf(M[13]) + fabsf(M[4 * r + 1]);
            qz = fabsf(M[14]) + fabsf(M[4 * r + 2]); qw = fabsf(M[15]) + fabsf(M[4 * r + 3]);
        }
        float dmax = pw + fmaxf(px * lx, px * hx) + fmaxf(py * ly, py * hy) + fmaxf(pz * lz, pz * hz);
        float mag = fmaf(qx, ax, fmaf(qy, ay, fmaf(qz, az, qw)));
        outside = outside || (dmax < -eps * mag);
    }
    return outside;
}

// One lane per queued straddling triangle: clip, project, fan, hand the pieces to emit().
__device__ __forceinline__ void drain_clip(const WaveLds& L, int first, int n, int& small_count, const SceneDev& sc,
                                           const float (&M)[16], const FrameParams& fp, int lane, u64* vis) {
    bool have = lane < n;
    uint32_t ref = have ? L.clipq[first + lane] : 0u;
    uint32_t c = ref >> 7, slot = ref & 127u;
    uint32_t t = gptr(sc.ctris)[(size_t)c * 128 + slot] & 0x00FFFFFFu;
    const BPS_GLOBAL float* cv = gptr(sc.cverts) + (size_t)c * 192;
    Clip4 px[2][kMaxPoly];
    uint32_t oc_or = 0;
    for (int k = 0; k < 3; ++k) {
        uint32_t vi = (t >> (8 * k)) & 0xFFu;
        px[0][k] = to_clip(M, cv[vi], cv[64 + vi], cv[128 + vi]);
        oc_or |= outcode(px[0][k]);
    }
    int cnt = have ? 3 : 0;
    int cur = 0;
    const int order[6] = {4, 5, 0, 1, 2, 3};
    for (int oi = 0; oi < 6; ++oi) {
        int k = order[oi];
        if (!((oc_or >> k) & 1u) || cnt < 3) continue;
        int m = 0;
        Clip4 prev = px[cur][cnt - 1];
        float dprev = plane_dist(prev, k);
        for (int i = 0; i < cnt; ++i) {
            Clip4 v = px[cur][i];
            float dv = plane_dist(v, k);
            bool cin = dv >= 0.0f, pin = dprev >= 0.0f;
            if (cin != pin && m < kMaxPoly) {
                // always from the inside vertex a to the outside vertex b
                Clip4 a = cin ? v : prev, b = cin ? prev : v;
                float da = cin ? dv : dprev, db = cin ? dprev : dv;
                float tt = da / (da - db);
                Clip4 o;
                o.x = fmaf(tt, b.x - a.x, a.x);
                o.y = fmaf(tt, b.y - a.y, a.y);
                o.z = fmaf(tt, b.z - a.z, a.z);
                o.w = fmaf(tt, b.w - a.w, a.w);
                px[cur ^ 1][m++] = o;
            }
            if (cin && m < kMaxPoly) px[cur ^ 1][m++] = v;
            prev = v;
            dprev = dv;
        }
        cnt = m;
        cur ^= 1;
    }
    if (cnt < 3) cnt = 0;
    // project every polygon vertex; one failure drops the triangle
    uint32_t pxy[kMaxPoly];
    float piw[kMaxPoly];
    bool ok = true;
    for (int i = 0; i < cnt; ++i) ok = project(px[cur][i], fp, pxy[i], piw[i]) && ok;
    if (!ok) cnt = 0;
    const BPS_GLOBAL uint32_t* id_ptr = gptr(sc.ctri_id) + (size_t)c * 128 + slot;
    for (int i = 1; ; ++i) {
        bool v = i + 1 < cnt;
        if (ballot64(v) == 0) break;
        uint32_t a = v ? pxy[0] : 0u, b = v ? pxy[i] : 0u, d = v ? pxy[i + 1] : 0u;
        float wa = v ? piw[0] : 0.0f, wb = v ? piw[i] : 0.0f, wd = v ? piw[i + 1] : 0.0f;
        emit(L, small_count, v, a, b, d, wa, wb, wd, id_ptr, lane, vis, fp.H, fp.W);
    }
}

// Append straddling triangles to the wave's clip queue (drained by the caller once per cluster,
// so at most 63 + 128 entries are ever pending).
__device__ __forceinline__ void push_clip(const WaveLds& L, int& count, bool want, uint32_t ref) {
    u64 mask = ballot64(want);
    if (mask == 0) return;
    if (want) L.clipq[count + (int)rank_below(mask)] = ref;
    count += __popcll(mask);
}

}  // namespace

// =============================================================================================
template <int NT>
__global__ __launch_bounds__(NT) void k_raster(const SceneDev* __restrict__ scenes, const WorkItem* __restrict__ items,
                                               const float* __restrict__ view_proj, FrameParams fp,
                                               unsigned long long* __restrict__ gvis, float* __restrict__ out_depth,
                                               uint32_t* __restrict__ out_id, unsigned long long* __restrict__ stats) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int NW = NT / 64;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int HW = fp.H * fp.W;

    u64* vis = reinterpret_cast<u64*>(smem);
    unsigned char* wbase = smem + (size_t)HW * 8 + (size_t)wave * kWaveLdsBytes;
    WaveLds L;
    L.stage = reinterpret_cast<float2*>(wbase);
    L.stage_oc = reinterpret_cast<uint32_t*>(wbase + 64 * 8);
    L.smallq = reinterpret_cast<uint32_t*>(wbase + 64 * 12);
    L.clipq = reinterpret_cast<uint32_t*>(wbase + 64 * 12 + 8 * 64 * 4);

    uint16_t* list = reinterpret_cast<uint16_t*>(smem + (size_t)HW * 8 + (size_t)NW * kWaveLdsBytes);
    uint32_t* counters = reinterpret_cast<uint32_t*>(smem + (size_t)HW * 8 + (size_t)NW * kWaveLdsBytes +
                                                     (size_t)fp.round_blocks * 128);
    uint32_t* list_count = counters;       // survivors appended in this round
    uint32_t* pop_count = counters + 1;    // survivors handed out in this round

    const WorkItem item = items[blockIdx.x];
    const SceneDev sc = scenes[item.scene];
    float M[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) M[k] = view_proj[(size_t)item.env * 16 + k];

    for (int p = tid; p < HW; p += NT) vis[p] = kEmptyKey;

    int small_count = 0, clip_count = 0;
    // diagnostics (only when the host passes a counter block): per-wave tallies, one atomic each at the end
    uint32_t st_tested = 0, st_boxed = 0, st_drawn = 0, st_straddle = 0;
    const unsigned long long t_start = stats ? wall_clock64() : 0ull;
    const uint32_t full_tri_mask = 0x00FFFFFFu;
    const BPS_GLOBAL float* g_cverts = gptr(sc.cverts);
    const BPS_GLOBAL uint32_t* g_ctris = gptr(sc.ctris);
    const BPS_GLOBAL uint32_t* g_ctri_id = gptr(sc.ctri_id);
    const BPS_GLOBAL float* g_bounds = gptr(sc.cbounds);
    const uint32_t S = item.n_splits;
    const uint32_t nblocks_total = (sc.n_clusters + 63u) / 64u;
    const uint32_t nb_item = nblocks_total > item.split ? (nblocks_total - item.split + S - 1u) / S : 0u;
    const uint32_t RB = (uint32_t)fp.round_blocks;

    // The item's clusters are the 64-cluster blocks split, split + S, ... of its scene.  They are
    // handled in rounds of RB blocks:
    //   phase A  every lane tests one cluster's bounds against the frustum; survivors are appended
    //            (ballot + prefix count, one LDS atomic per wavefront) to the work-group's list
    //   phase B  wavefronts pop clusters from the list one at a time until it is empty
    for (uint32_t rb = 0; rb < nb_item; rb += RB) {
        if (tid == 0) { *list_count = 0u; *pop_count = 0u; }
        __syncthreads();
        const uint32_t rb_end = min(rb + RB, nb_item);
        for (uint32_t jb = rb + (uint32_t)wave; jb < rb_end; jb += NW) {
            const uint32_t cl = (jb * S + item.split) * 64u + (uint32_t)lane;
            bool visible = cl < sc.n_clusters;
            st_tested += (uint32_t)__popcll(ballot64(visible));
            if (fp.cull) {
                const uint32_t cc = visible ? cl : 0u;
                float lx = g_bounds[cc], ly = g_bounds[sc.c_stride + cc], lz = g_bounds[2 * sc.c_stride + cc];
                float hx = g_bounds[3 * sc.c_stride + cc], hy = g_bounds[4 * sc.c_stride + cc],
                      hz = g_bounds[5 * sc.c_stride + cc];
                visible = visible && !box_outside_frustum(M, lx, ly, lz, hx, hy, hz);
            }
            const u64 keep = ballot64(visible);
            if (keep) {
                uint32_t base = 0;
                if (lane == 0) base = atomicAdd(list_count, (uint32_t)__popcll(keep));
                base = __builtin_amdgcn_readfirstlane(base);
                if (visible) list[base + rank_below(keep)] = (uint16_t)(((jb - rb) << 6) | (uint32_t)lane);
            }
        }
        __syncthreads();
        const uint32_t n_list = *list_count;
        st_boxed += wave == 0 ? n_list : 0u;

        // pop one ahead so that the next cluster's words are in flight while this one is processed
        uint32_t pop = 0;
        if (lane == 0) pop = atomicAdd(pop_count, 1u);
        pop = __builtin_amdgcn_readfirstlane(pop);
        float nx_ = 0, ny_ = 0, nz_ = 0;
        uint32_t nt0 = 0, nt1 = 0, c_next = 0;
        if (pop < n_list) {
            const uint32_t e = list[pop];
            c_next = ((rb + (e >> 6)) * S + item.split) * 64u + (e & 63u);
            const BPS_GLOBAL float* cv = g_cverts + (size_t)c_next * 192;
            nx_ = cv[lane]; ny_ = cv[64 + lane]; nz_ = cv[128 + lane];
            const BPS_GLOBAL uint32_t* ct = g_ctris + (size_t)c_next * 128;
            nt0 = ct[lane]; nt1 = ct[64 + lane];
        }
        while (pop < n_list) {
            const uint32_t c = c_next;
            float x = nx_, y = ny_, z = nz_;
            uint32_t t0 = nt0, t1 = nt1;
            if (lane == 0) pop = atomicAdd(pop_count, 1u);
            pop = __builtin_amdgcn_readfirstlane(pop);
            if (pop < n_list) {
                const uint32_t e = list[pop];
                c_next = ((rb + (e >> 6)) * S + item.split) * 64u + (e & 63u);
                const BPS_GLOBAL float* cv = g_cverts + (size_t)c_next * 192;
                nx_ = cv[lane]; ny_ = cv[64 + lane]; nz_ = cv[128 + lane];
                const BPS_GLOBAL uint32_t* ct = g_ctris + (size_t)c_next * 128;
                nt0 = ct[lane]; nt1 = ct[64 + lane];
            }

            // ---- vertex phase
            Clip4 cp = to_clip(M, x, y, z);
            bool o0 = !(cp.w + cp.x >= 0.0f), o1 = !(cp.w - cp.x >= 0.0f);
            bool o2 = !(cp.w + cp.y >= 0.0f), o3 = !(cp.w - cp.y >= 0.0f);
            bool o4 = !(cp.z >= 0.0f), o5 = !(cp.w - cp.z >= 0.0f);
            bool culled = ballot64(o0) == ~0ull || ballot64(o1) == ~0ull || ballot64(o2) == ~0ull ||
                          ballot64(o3) == ~0ull || ballot64(o4) == ~0ull || ballot64(o5) == ~0ull;
            if (culled) continue;
            ++st_drawn;
            uint32_t oc = (o0 ? 1u : 0u) | (o1 ? 2u : 0u) | (o2 ? 4u : 0u) | (o3 ? 8u : 0u) | (o4 ? 16u : 0u) |
                          (o5 ? 32u : 0u);
            if (!all_finite(cp)) oc |= kInvalid;
            uint32_t xy;
            float iw;
            bool ok = project(cp, fp, xy, iw);
            if (oc == 0 && !ok) oc = kInvalid;
            const bool all_inside = ballot64(oc != 0) == 0;
            wave_lds_sync();   // earlier reads of the stage are done
            L.stage[lane] = make_float2(__uint_as_float(xy), iw);
            if (!all_inside) L.stage_oc[lane] = oc;
            wave_lds_sync();

            // ---- triangle phase: two slots per lane
            const int ntri = __builtin_amdgcn_readfirstlane((int)(t0 >> 24));
#pragma unroll 1
            for (int slot = 0; slot < 2; ++slot) {
                if (slot == 1 && ntri <= 64) break;
                uint32_t t = (slot == 0 ? t0 : t1) & full_tri_mask;
                const uint32_t i0 = t & 0xFFu, i1 = (t >> 8) & 0xFFu, i2 = t >> 16;
                float2 a = L.stage[i0], b = L.stage[i1], d = L.stage[i2];
                bool fast = slot * 64 + lane < ntri;
                if (!all_inside) {
                    uint32_t oa = L.stage_oc[i0], ob = L.stage_oc[i1], od = L.stage_oc[i2];
                    uint32_t o_or = oa | ob | od, o_and = oa & ob & od;
                    bool live = fast && ((o_or & kInvalid) == 0) && (o_and == 0);
                    fast = live && o_or == 0;
                    st_straddle += (uint32_t)__popcll(ballot64(live && o_or != 0));
                    push_clip(L, clip_count, live && o_or != 0, (c << 7) | (uint32_t)(slot * 64 + lane));
                }
                emit(L, small_count, fast, __float_as_uint(a.x), __float_as_uint(b.x), __float_as_uint(d.x), a.y, b.y,
                     d.y, g_ctri_id + (size_t)c * 128 + slot * 64 + lane, lane, vis, fp.H, fp.W);
            }
            // ---- clip queue: full wavefronts only while streaming
            while (clip_count >= 64) {
                wave_lds_sync();
                drain_clip(L, clip_count - 64, 64, small_count, sc, M, fp, lane, vis);
                clip_count -= 64;
            }
        }
        __syncthreads();
    }
    if (clip_count > 0) {
        wave_lds_sync();
        drain_clip(L, 0, clip_count, small_count, sc, M, fp, lane, vis);
    }
    if (small_count > 0) {
        wave_lds_sync();
        drain_small(L, small_count, lane, vis, fp.W);
    }
    if (stats && lane == 0) {
        atomicAdd(&stats[0], (unsigned long long)st_tested);
        atomicAdd(&stats[1], (unsigned long long)st_boxed);
        atomicAdd(&stats[2], (unsigned long long)st_drawn);
        atomicAdd(&stats[3], (unsigned long long)st_straddle);
        unsigned long long dt = wall_clock64() - t_start;
        atomicAdd(&stats[4], dt);
        atomicMax(&stats[5], dt);
        if (wave == 0) stats[8 + blockIdx.x] = dt;      // duration of this work-group's first wave
    }
    __syncthreads();

    // ---- resolve this work-group's frame
    const size_t base = (size_t)item.env * HW;
    if (fp.merge) {
        for (int p = tid; p < HW; p += NT) {
            u64 key = vis[p];
            if (key != kEmptyKey) atomicMin(&gvis[base + p], key);
        }
    } else {
        for (int p = tid; p < HW; p += NT) {
            u64 key = vis[p];
            bool hit = key != kEmptyKey;
            out_depth[base + p] = hit ? __uint_as_float((uint32_t)(key >> 32)) : fp.background;
            if (out_id) out_id[base + p] = hit ? (uint32_t)key : 0xFFFFFFFFu;
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

__global__ void k_zero_words(unsigned long long* __restrict__ p, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

__global__ void k_fill_keys(unsigned long long* __restrict__ gvis, size_t n) {
    size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n) gvis[p] = kEmptyKey;
}

hipError_t prepare_raster(int threads, size_t lds) {
    const void* f = threads == 256   ? reinterpret_cast<const void*>(&k_raster<256>)
                    : threads == 512 ? reinterpret_cast<const void*>(&k_raster<512>)
                                     : reinterpret_cast<const void*>(&k_raster<1024>);
    return hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
}

void launch_raster(int threads, dim3 grid, size_t lds, hipStream_t stream, const SceneDev* scenes, const WorkItem* items,
                   const float* view_proj, const FrameParams& fp, unsigned long long* gvis, float* out_depth,
                   uint32_t* out_id, unsigned long long* stats) {
    if (threads == 256)
        hipLaunchKernelGGL(k_raster<256>, grid, dim3(256), lds, stream, scenes, items, view_proj, fp, gvis, out_depth, out_id, stats);
    else if (threads == 512)
        hipLaunchKernelGGL(k_raster<512>, grid, dim3(512), lds, stream, scenes, items, view_proj, fp, gvis, out_depth, out_id, stats);
    else
        hipLaunchKernelGGL(k_raster<1024>, grid, dim3(1024), lds, stream, scenes, items, view_proj, fp, gvis, out_depth, out_id, stats);
}

}  // namespace bps
