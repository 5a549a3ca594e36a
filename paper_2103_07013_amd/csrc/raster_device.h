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

// Loads through pointers that arrive inside structs would otherwise be generic ("flat") accesses.
#define BPS_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ const BPS_GLOBAL T* gptr(const T* p) {
    return (const BPS_GLOBAL T*)p;
}

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

// Snapped screen coordinates travel as two signed 16-bit halves, x low and y high, relative to
// kOrigin = 64 pixels, so that the whole range [-64, 256*128 + 64] of a 128-pixel axis fits and
// bounding boxes can be computed with packed 16-bit instructions.
__device__ __forceinline__ uint32_t pack_xy(int X, int Y) {
    return ((uint32_t)(X - kOrigin) & 0xFFFFu) | ((uint32_t)(Y - kOrigin) << 16);
}
__device__ __forceinline__ int unpack_x(uint32_t xy) { return (int)(short)(xy & 0xFFFFu); }
__device__ __forceinline__ int unpack_y(uint32_t xy) { return (int)xy >> 16; }

// ---------------------------------------------------------------------------------------------
// Triangle in snapped screen space, oriented so that A2 > 0, with its edge set-up.
struct Setup {
    int X0, Y0, X1, Y1, X2, Y2;   // 1/256-px coordinates relative to kOrigin
    float iw0, iw1, iw2;
    int A2;
    int dx0, dy0, dx1, dy1, dx2, dy2;   // edge k is opposite vertex k
    int b0, b1, b2;                     // 0 on a top-left edge, -1 otherwise
    bool swapped;                       // vertices 1 and 2 were exchanged to make A2 positive
};

__device__ __forceinline__ int tl_bias(int dx, int dy) { return (dy < 0 || (dy == 0 && dx > 0)) ? 0 : -1; }

__device__ __forceinline__ Setup make_setup(uint32_t xy0, uint32_t xy1, uint32_t xy2, float iw0, float iw1, float iw2) {
    Setup s;
    s.X0 = unpack_x(xy0); s.Y0 = unpack_y(xy0);
    s.X1 = unpack_x(xy1); s.Y1 = unpack_y(xy1);
    s.X2 = unpack_x(xy2); s.Y2 = unpack_y(xy2);
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

// The part of the frame one work-group owns: pixels [x0, x0 + w) x [y0, y0 + h), and the same
// rectangle in normalised device coordinates (aL <= x/w <= aR, aT <= y/w <= aB).
struct Window {
    int x0, y0, w, h;
    float aL, aR, aT, aB;
};

// Coverage test and z-test of pixel (i, j) against one set-up triangle; vis holds the window's pixels.
__device__ __forceinline__ void shade_pixel(const Setup& s, int i, int j, bool active, uint32_t id, u64* vis,
                                            const Window& win) {
    int px = (i << 8) + 128 - kOrigin, py = (j << 8) + 128 - kOrigin;
    int E0 = __mul24(s.dx0, py - s.Y1) - __mul24(s.dy0, px - s.X1);
    int E1 = __mul24(s.dx1, py - s.Y2) - __mul24(s.dy1, px - s.X2);
    int E2 = __mul24(s.dx2, py - s.Y0) - __mul24(s.dy2, px - s.X0);
    bool in = active && s.A2 != 0 && (((E0 + s.b0) | (E1 + s.b1) | (E2 + s.b2)) >= 0);
    if (in) {
        float e0 = (float)E0, e1 = (float)E1, e2 = (float)E2;
        float num = fmaf(e2, s.iw2, fmaf(e1, s.iw1, e0 * s.iw0));
        float depth = (float)s.A2 / num;
        u64 key = ((u64)__float_as_uint(depth) << 32) | (u64)id;
        atomicMin(&vis[__mul24(j - win.y0, win.w) + (i - win.x0)], key);   // 24-bit multiply: full rate
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

// x*0 is 0 for every finite x and NaN otherwise, so one fma chain tests all four coordinates.
__device__ __forceinline__ bool all_finite(const Clip4& c) {
    float t = fmaf(c.x, 0.0f, fmaf(c.y, 0.0f, fmaf(c.z, 0.0f, c.w * 0.0f)));
    return t == t;
}

__device__ __forceinline__ uint32_t outcode(const Clip4& c) {
    uint32_t oc = 0;
    oc |= !(c.w + c.x >= 0.0f) ? 1u : 0u;
    oc |= !(c.w - c.x >= 0.0f) ? 2u : 0u;
    oc |= !(c.w + c.y >= 0.0f) ? 4u : 0u;
    oc |= !(c.w - c.y >= 0.0f) ? 8u : 0u;
    oc |= !(c.z >= 0.0f) ? 16u : 0u;
    oc |= !(c.w - c.z >= 0.0f) ? 32u : 0u;
    if (!all_finite(c)) oc |= kInvalid;
    return oc;
}

// Perspective divide + snap.  Returns false when the vertex cannot be placed on the sub-pixel grid
// of the frame (the numeric rule then drops its triangle).  can_project tells whether the vertex is
// in front of the eye with finite screen coordinates; such a vertex outside the frame is packed
// with its coordinates clamped to the 16-bit range, which keeps it on its side of the frame.
__device__ __forceinline__ bool project(const Clip4& c, const FrameParams& fp, uint32_t& xy, float& iw,
                                        bool& can_project) {
    iw = 1.0f / c.w;
    float xn = c.x * iw, yn = c.y * iw;
    float fx = fmaf(xn, fp.sx, fp.sx), fy = fmaf(yn, fp.sy, fp.sy);
    bool ok = (c.w > 0.0f) && fx >= -64.0f && fx <= fp.xmax && fy >= -64.0f && fy <= fp.ymax;
    can_project = (c.w > 0.0f) && fabsf(fx) < 3.0e38f && fabsf(fy) < 3.0e38f;
    int X = min(max(__float2int_rn(fx), kOrigin - 32768), kOrigin + 32767);
    int Y = min(max(__float2int_rn(fy), kOrigin - 32768), kOrigin + 32767);
    xy = pack_xy(X, Y);
    return ok;
}

constexpr int kMaxPoly = 16;   // a triangle cut by six planes has at most 9 corners; rounding can add a few

}  // namespace dev
}  // namespace bps
