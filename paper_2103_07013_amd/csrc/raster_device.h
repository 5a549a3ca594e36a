// Device helpers shared by the raster and shading kernels: wave intrinsics, the vertex transform,
// outcodes, projection / snapping and the integer triangle set-up.  Both kernels must evaluate
// exactly the same IEEE operation sequence, so the code lives in one place.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "raster_kernels.h"

namespace bps {
namespace dev {

typedef unsigned long long u64;

__device__ __forceinline__ u64 ballot64(bool p) { return __builtin_amdgcn_ballot_w64(p); }

__device__ __forceinline__ uint32_t rank_below(u64 mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Orders this wavefront's LDS writes before its later LDS reads by other lanes.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ int bcast_i(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ float bcast_f(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// ---------------------------------------------------------------------------------------------
// Triangle in snapped screen space, oriented so that A2 > 0, with its edge set-up.
struct Setup {
    int X0, Y0, X1, Y1, X2, Y2;   // biased 1/256-px coordinates
    float iw0, iw1, iw2;
    int A2;
    int dx0, dy0, dx1, dy1, dx2, dy2;   // edge k is opposite vertex k
    int b0, b1, b2;                     // 0 on a top-left edge, -1 otherwise
    bool swapped;                       // vertices 1 and 2 were exchanged to make A2 positive
};

__device__ __forceinline__ int tl_bias(int dx, int dy) { return (dy < 0 || (dy == 0 && dx > 0)) ? 0 : -1; }

__device__ __forceinline__ Setup make_setup(uint32_t xy0, uint32_t xy1, uint32_t xy2, float iw0, float iw1, float iw2) {
    Setup s;
    s.X0 = (int)(xy0 & 0xFFFFu); s.Y0 = (int)(xy0 >> 16);
    s.X1 = (int)(xy1 & 0xFFFFu); s.Y1 = (int)(xy1 >> 16);
    s.X2 = (int)(xy2 & 0xFFFFu); s.Y2 = (int)(xy2 >> 16);
    s.iw0 = iw0; s.iw1 = iw1; s.iw2 = iw2;
    int a2 = __mul24(s.X1 - s.X0, s.Y2 - s.Y0) - __mul24(s.X2 - s.X0, s.Y1 - s.Y0);
    s.swapped = a2 < 0;
    if (a2 < 0) {   // two-sided: swap vertices 1 and 2
        int t;
        t = s.X1; s.X1 = s.X2; s.X2 = t;
        t = s.Y1; s.Y1 = s.Y2; s.Y2 = t;
        float f = s.iw1; s.iw1 = s.iw2; s.iw2 = f;
        a2 = -a2;
    }
    s.A2 = a2;
    s.dx0 = s.X2 - s.X1; s.dy0 = s.Y2 - s.Y1;
    s.dx1 = s.X0 - s.X2; s.dy1 = s.Y0 - s.Y2;
    s.dx2 = s.X1 - s.X0; s.dy2 = s.Y1 - s.Y0;
    s.b0 = tl_bias(s.dx0, s.dy0);
    s.b1 = tl_bias(s.dx1, s.dy1);
    s.b2 = tl_bias(s.dx2, s.dy2);
    return s;
}

// Coverage test and z-test of pixel (i, j) against one set-up triangle.
__device__ __forceinline__ void shade_pixel(const Setup& s, int i, int j, bool active, uint32_t id, u64* vis, int W) {
    int px = (i << 8) + 128 + kBias, py = (j << 8) + 128 + kBias;
    int E0 = __mul24(s.dx0, py - s.Y1) - __mul24(s.dy0, px - s.X1);
    int E1 = __mul24(s.dx1, py - s.Y2) - __mul24(s.dy1, px - s.X2);
    int E2 = __mul24(s.dx2, py - s.Y0) - __mul24(s.dy2, px - s.X0);
    bool in = active && (((E0 + s.b0) | (E1 + s.b1) | (E2 + s.b2)) >= 0);
    if (in) {
        float e0 = (float)E0, e1 = (float)E1, e2 = (float)E2;
        float num = fmaf(e2, s.iw2, fmaf(e1, s.iw1, e0 * s.iw0));
        float depth = (float)s.A2 / num;
        u64 key = ((u64)__float_as_uint(depth) << 32) | (u64)id;
        atomicMin(&vis[j * W + i], key);
    }
}

// ---------------------------------------------------------------------------------------------
// Vertex transform, shared by the vertex phase and the clip path so both see identical bits.
struct Clip4 { float x, y, z, w; };

__device__ __forceinline__ Clip4 to_clip(const float (&M)[16], float x, float y, float z) {
    Clip4 c;
    c.x = fmaf(M[2], z, fmaf(M[1], y, fmaf(M[0], x, M[3])));
    c.y = fmaf(M[6], z, fmaf(M[5], y, fmaf(M[4], x, M[7])));
    c.z = fmaf(M[10], z, fmaf(M[9], y, fmaf(M[8], x, M[11])));
    c.w = fmaf(M[14], z, fmaf(M[13], y, fmaf(M[12], x, M[15])));
    return c;
}

__device__ __forceinline__ float plane_dist(const Clip4& v, int k) {
    switch (k) {
    case 0: return v.w + v.x;
    case 1: return v.w - v.x;
    case 2: return v.w + v.y;
    case 3: return v.w - v.y;
    case 4: return v.z;
    default: return v.w - v.z;
    }
}

__device__ __forceinline__ uint32_t outcode(const Clip4& c) {
    uint32_t oc = 0;
    oc |= !(c.w + c.x >= 0.0f) ? 1u : 0u;
    oc |= !(c.w - c.x >= 0.0f) ? 2u : 0u;
    oc |= !(c.w + c.y >= 0.0f) ? 4u : 0u;
    oc |= !(c.w - c.y >= 0.0f) ? 8u : 0u;
    oc |= !(c.z >= 0.0f) ? 16u : 0u;
    oc |= !(c.w - c.z >= 0.0f) ? 32u : 0u;
    bool fin = __builtin_isfinite(c.x) && __builtin_isfinite(c.y) && __builtin_isfinite(c.z) && __builtin_isfinite(c.w);
    if (!fin) oc |= kInvalid;
    return oc;
}

// Perspective divide + snap.  Returns false when the vertex cannot be placed on the sub-pixel grid.
__device__ __forceinline__ bool project(const Clip4& c, const FrameParams& fp, uint32_t& xy, float& iw) {
    iw = 1.0f / c.w;
    float xn = c.x * iw, yn = c.y * iw;
    float fx = fmaf(xn, fp.sx, fp.sx), fy = fmaf(yn, fp.sy, fp.sy);
    bool ok = (c.w > 0.0f) && fx >= -64.0f && fx <= fp.xmax && fy >= -64.0f && fy <= fp.ymax;
    int X = __float2int_rn(fx) + kBias, Y = __float2int_rn(fy) + kBias;
    xy = ((uint32_t)X & 0xFFFFu) | ((uint32_t)Y << 16);
    return ok;
}

constexpr int kMaxPoly = 16;   // a triangle cut by six planes has at most 9 corners; rounding can add a few

}  // namespace dev
}  // namespace bps
