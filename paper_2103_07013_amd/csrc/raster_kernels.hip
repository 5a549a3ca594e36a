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
    float4* stage;      // [64] staged vertices of the current cluster: (xy bits, 1/w, outcode bits, -)
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

// Bounding-box cull, classification and hand-off of one candidate triangle per lane.
// id_ptr is only dereferenced by lanes whose triangle can touch a pixel centre.
__device__ __forceinline__ void emit(const WaveLds& L, int& small_count, bool valid, uint32_t xy0, uint32_t xy1,
                                     uint32_t xy2, float iw0, float iw1, float iw2, const uint32_t* id_ptr, int lane,
                                     u64* vis, int H, int W) {
    int X0 = (int)(xy0 & 0xFFFFu), Y0 = (int)(xy0 >> 16);
    int X1 = (int)(xy1 & 0xFFFFu), Y1 = (int)(xy1 >> 16);
    int X2 = (int)(xy2 & 0xFFFFu), Y2 = (int)(xy2 >> 16);
    int minX = min(X0, min(X1, X2)), maxX = max(X0, max(X1, X2));
    int minY = min(Y0, min(Y1, Y2)), maxY = max(Y0, max(Y1, Y2));
    // pixel centres 256 i + 128 (+ bias) inside the closed box
    int i_lo = max((minX - kBias + 127) >> 8, 0), i_hi = min((maxX - kBias - 128) >> 8, W - 1);
    int j_lo = max((minY - kBias + 127) >> 8, 0), j_hi = min((maxY - kBias - 128) >> 8, H - 1);
    int a2 = __mul24(X1 - X0, Y2 - Y0) - __mul24(X2 - X0, Y1 - Y0);
    valid = valid && i_lo <= i_hi && j_lo <= j_hi && a2 != 0;
    u64 vmask = ballot64(valid);
    if (vmask == 0) return;
    uint32_t id = valid ? *id_ptr : 0u;
    int nx = i_hi - i_lo + 1, ny = j_hi - j_lo + 1;
    bool small = valid && nx * ny <= kSmallMax;
    uint32_t box = (uint32_t)i_lo | ((uint32_t)j_lo << 8) | ((uint32_t)nx << 16) | ((uint32_t)ny << 24);
    push_small(L, small_count, small, xy0, xy1, xy2, iw0, iw1, iw2, id, box, lane, vis, W);
    u64 big = ballot64(valid && !small);
    while (big) {
        int src = __builtin_ctzll(big);
        big &= big - 1;
        raster_large((uint32_t)bcast_i((int)xy0, src), (uint32_t)bcast_i((int)xy1, src), (uint32_t)bcast_i((int)xy2, src),
                     bcast_f(iw0, src), bcast_f(iw1, src), bcast_f(iw2, src), (uint32_t)bcast_i((int)id, src),
                     bcast_i(i_lo, src), bcast_i(i_hi, src), bcast_i(j_lo, src), bcast_i(j_hi, src), lane, vis, W);
    }
}


// One lane per queued straddling triangle: clip, project, fan, hand the pieces to emit().
__device__ __forceinline__ void drain_clip(const WaveLds& L, int first, int n, int& small_count, const SceneDev& sc,
                                           const float (&M)[16], const FrameParams& fp, int lane, u64* vis) {
    bool have = lane < n;
    uint32_t ref = have ? L.clipq[first + lane] : 0u;
    uint32_t c = ref >> 7, slot = ref & 127u;
    uint32_t t = sc.ctris[(size_t)c * 128 + slot] & 0x00FFFFFFu;
    const float* cv = sc.cverts + (size_t)c * 192;
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
    const uint32_t* id_ptr = sc.ctri_id + (size_t)c * 128 + slot;
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
                                               uint32_t* __restrict__ out_id) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int NW = NT / 64;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int HW = fp.H * fp.W;

    u64* vis = reinterpret_cast<u64*>(smem);
    unsigned char* wbase = smem + (size_t)HW * 8 + (size_t)wave * kWaveLdsBytes;
    WaveLds L;
    L.stage = reinterpret_cast<float4*>(wbase);
    L.smallq = reinterpret_cast<uint32_t*>(wbase + 64 * 16);
    L.clipq = reinterpret_cast<uint32_t*>(wbase + 64 * 16 + 8 * 64 * 4);

    const WorkItem item = items[blockIdx.x];
    const SceneDev sc = scenes[item.scene];
    float M[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) M[k] = view_proj[(size_t)item.env * 16 + k];

    for (int p = tid; p < HW; p += NT) vis[p] = kEmptyKey;
    __syncthreads();

    int small_count = 0, clip_count = 0;
    const uint32_t full_tri_mask = 0x00FFFFFFu;

    uint32_t c = item.c_begin + (uint32_t)wave;
    // software prefetch of the next cluster's vertex and index words
    float nx_ = 0, ny_ = 0, nz_ = 0;
    uint32_t nt0 = 0, nt1 = 0;
    if (c < item.c_end) {
        const float* cv = sc.cverts + (size_t)c * 192;
        nx_ = cv[lane]; ny_ = cv[64 + lane]; nz_ = cv[128 + lane];
        const uint32_t* ct = sc.ctris + (size_t)c * 128;
        nt0 = ct[lane]; nt1 = ct[64 + lane];
    }
    for (;;) {
        const bool have = c < item.c_end;
        if (have) {
            float x = nx_, y = ny_, z = nz_;
            uint32_t t0 = nt0, t1 = nt1;
            uint32_t cn = c + NW;
            if (cn < item.c_end) {
                const float* cv = sc.cverts + (size_t)cn * 192;
                nx_ = cv[lane]; ny_ = cv[64 + lane]; nz_ = cv[128 + lane];
                const uint32_t* ct = sc.ctris + (size_t)cn * 128;
                nt0 = ct[lane]; nt1 = ct[64 + lane];
            }

            // ---- vertex phase
            Clip4 cl = to_clip(M, x, y, z);
            uint32_t oc = outcode(cl);
            bool culled = false;
#pragma unroll
            for (int k = 0; k < 6; ++k) culled = culled || (ballot64((oc >> k) & 1u) == ~0ull);
            if (!culled) {
                uint32_t xy;
                float iw;
                bool ok = project(cl, fp, xy, iw);
                if (oc == 0 && !ok) oc = kInvalid;
                wave_lds_sync();   // earlier reads of the stage are done
                L.stage[lane] = make_float4(__uint_as_float(xy), iw, __uint_as_float(oc), 0.0f);
                wave_lds_sync();

                // ---- triangle phase: two slots per lane
                const int ntri = __builtin_amdgcn_readfirstlane((int)(t0 >> 24));
#pragma unroll 1
                for (int slot = 0; slot < 2; ++slot) {
                    if (slot == 1 && ntri <= 64) break;
                    uint32_t t = (slot == 0 ? t0 : t1) & full_tri_mask;
                    float4 a = L.stage[t & 0xFFu], b = L.stage[(t >> 8) & 0xFFu], d = L.stage[t >> 16];
                    uint32_t oa = __float_as_uint(a.z), ob = __float_as_uint(b.z), od = __float_as_uint(d.z);
                    uint32_t o_or = oa | ob | od, o_and = oa & ob & od;
                    bool live = ((o_or & kInvalid) == 0) && (o_and == 0) && (slot * 64 + lane < ntri);
                    bool fast = live && o_or == 0;
                    bool straddle = live && o_or != 0;
                    push_clip(L, clip_count, straddle, (c << 7) | (uint32_t)(slot * 64 + lane));
                    emit(L, small_count, fast, __float_as_uint(a.x), __float_as_uint(b.x), __float_as_uint(d.x), a.y, b.y,
                         d.y, sc.ctri_id + (size_t)c * 128 + slot * 64 + lane, lane, vis, fp.H, fp.W);
                }
            }
            c += NW;
        }
        // ---- clip queue: full wavefronts while streaming, the remainder at the end
        while (clip_count >= 64 || (!have && clip_count > 0)) {
            int n = clip_count < 64 ? clip_count : 64;
            wave_lds_sync();
            drain_clip(L, clip_count - n, n, small_count, sc, M, fp, lane, vis);
            clip_count -= n;
        }
        if (!have) break;
    }
    if (small_count > 0) {
        wave_lds_sync();
        drain_small(L, small_count, lane, vis, fp.W);
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
                   uint32_t* out_id) {
    if (threads == 256)
        hipLaunchKernelGGL(k_raster<256>, grid, dim3(256), lds, stream, scenes, items, view_proj, fp, gvis, out_depth, out_id);
    else if (threads == 512)
        hipLaunchKernelGGL(k_raster<512>, grid, dim3(512), lds, stream, scenes, items, view_proj, fp, gvis, out_depth, out_id);
    else
        hipLaunchKernelGGL(k_raster<1024>, grid, dim3(1024), lds, stream, scenes, items, view_proj, fp, gvis, out_depth, out_id);
}

}  // namespace bps
