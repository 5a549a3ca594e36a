// Colour resolve for RGB-D frames (stand-in for the paper's textured RGB sensor, Sec. 4.1):
// per-vertex uint8 colours, perspective-correct interpolation at the pixel centre of the
// triangle that won the z-test.  Runs after k_raster, one thread per pixel: the winner's
// three vertices are transformed, clipped and set up again with exactly the arithmetic of
// the raster kernel, so the barycentric weights are the ones the z-test used.
//   cn = fma(e2/w2, c2, fma(e1/w1, c1, (e0/w0) c0)),  out = clamp(rint(cn / num), 0, 255)
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

// Colour of pixel (i, j) from one snapped fan triangle; returns false when it does not cover the pixel.
__device__ __forceinline__ bool piece_colour(const SVert& v0, const SVert& v1, const SVert& v2, int i, int j,
                                             float& depth, float (&rgb)[3], float& uv_area2, int& area2) {
    Setup s = make_setup(v0.xy, v1.xy, v2.xy, v0.iw, v1.iw, v2.iw);
    if (s.A2 == 0) return false;
    const SVert& a = v0;
    const SVert& b = s.swapped ? v2 : v1;
    const SVert& c = s.swapped ? v1 : v2;
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

}  // namespace

__global__ __launch_bounds__(256) void k_shade(const SceneDev* __restrict__ scenes, const uint32_t* __restrict__ env_scene,
                                               const float* __restrict__ view_proj, FrameParams fp, uint32_t B,
                                               const uint32_t* __restrict__ tri_id, uint8_t* __restrict__ out_rgb) {
    const int HW = fp.H * fp.W;
    size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // HW is a multiple of 64: one env per wave
    if (p >= (size_t)B * HW) return;
    const uint32_t env = __builtin_amdgcn_readfirstlane((uint32_t)(p / HW));
    const int pix = (int)(p - (size_t)env * HW);
    const int i = pix % fp.W, j = pix / fp.W;
    uint8_t out[3] = {0, 0, 0};
    const uint32_t id = tri_id[p];
    const SceneDev sc = scenes[env_scene[env]];
    const bool textured = sc.texels != nullptr;
    if (id != 0xFFFFFFFFu && (sc.colors != nullptr || textured) && id < sc.n_tris) {
        float M[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) M[k] = view_proj[(size_t)env * 16 + k];
        CVert poly[2][kMaxPoly];
        uint32_t oc_or = 0;
        for (int k = 0; k < 3; ++k) {
            uint32_t vi = sc.indices[3 * (size_t)id + k];
            const float* v = sc.verts + 3 * (size_t)vi;
            poly[0][k].c = to_clip(M, v[0], v[1], v[2]);
            if (textured) {
                poly[0][k].r = sc.uvs[2 * (size_t)vi + 0];
                poly[0][k].g = sc.uvs[2 * (size_t)vi + 1];
                poly[0][k].b = 0.0f;
            } else {
                const uint8_t* col = sc.colors + 3 * (size_t)vi;
                poly[0][k].r = (float)col[0];
                poly[0][k].g = (float)col[1];
                poly[0][k].b = (float)col[2];
            }
            oc_or |= outcode(poly[0][k].c);
        }
        int cnt = 3, cur = 0;
        const int order[6] = {4, 5, 0, 1, 2, 3};
        for (int oi = 0; oi < 6; ++oi) {
            int k = order[oi];
            if (!((oc_or >> k) & 1u) || cnt < 3) continue;
            int m = 0;
            CVert prev = poly[cur][cnt - 1];
            float dprev = plane_dist(prev.c, k);
            for (int q = 0; q < cnt; ++q) {
                CVert v = poly[cur][q];
                float dv = plane_dist(v.c, k);
                bool cin = dv >= 0.0f, pin = dprev >= 0.0f;
                if (cin != pin && m < kMaxPoly) {
                    const CVert& a = cin ? v : prev;      // inside
                    const CVert& b = cin ? prev : v;      // outside
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
                    poly[cur ^ 1][m++] = o;
                }
                if (cin && m < kMaxPoly) poly[cur ^ 1][m++] = v;
                prev = v;
                dprev = dv;
            }
            cnt = m;
            cur ^= 1;
        }
        if (cnt >= 3) {
            SVert sv[kMaxPoly];
            bool ok = true;
            for (int q = 0; q < cnt; ++q) {
                bool unused;
                ok = project(poly[cur][q].c, fp, sv[q].xy, sv[q].iw, unused) && ok;
                sv[q].r = poly[cur][q].r;
                sv[q].g = poly[cur][q].g;
                sv[q].b = poly[cur][q].b;
            }
            if (ok) {
                // the fan pieces of one triangle tile it; should rounding ever make two of them
                // cover this pixel, the nearer one is the one the z-test kept (first one on a tie)
                float best = 0.0f;
                bool found = false;
                for (int q = 1; q + 1 < cnt; ++q) {
                    float d, rgb[3], uv_area2;
                    int area2;
                    if (piece_colour(sv[0], sv[q], sv[q + 1], i, j, d, rgb, uv_area2, area2) && (!found || d < best)) {
                        found = true;
                        best = d;
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
                }
            }
        }
    }
    out_rgb[3 * p + 0] = out[0];
    out_rgb[3 * p + 1] = out[1];
    out_rgb[3 * p + 2] = out[2];
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

void launch_shade(hipStream_t stream, const SceneDev* scenes, const uint32_t* env_scene, const float* view_proj,
                  const FrameParams& fp, uint32_t B, const uint32_t* tri_id, uint8_t* out_rgb) {
    size_t n = (size_t)B * fp.H * fp.W;
    hipLaunchKernelGGL(k_shade, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, scenes, env_scene, view_proj, fp, B,
                       tri_id, out_rgb);
}

}  // namespace bps
