/*
 * CPU oracle for the batch renderer  --  TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this.  It shares no code with the GPU library and is never a fallback for it.
 *
 * What it computes (paper Sec. 3, Sec. 3.2: one request per environment, N frames
 * out; K scenes shared by reference): for every environment b and every pixel
 * centre of its H x W frame, the nearest triangle of scene s_b as seen through
 * view_proj[b].  The paper delegates rasterisation to the graphics API and states
 * no rule, so the rule below is this build's numeric contract:
 *
 *   N0  binary32, round-to-nearest-even, no contraction, fmaf exactly where written.
 *   N1  clip = M (x,y,z,1): c_r = fma(M[r][2],z, fma(M[r][1],y, fma(M[r][0],x, M[r][3]))).
 *   N2  six planes d0=w+x d1=w-x d2=w+y d3=w-y d4=z d5=w-z, inside iff d >= 0.
 *       Any non-finite clip coordinate drops the triangle; all three vertices outside
 *       one plane drops it; all inside every plane leaves it whole; otherwise N3.
 *   N3  Sutherland-Hodgman, planes in order near, far, left, right, top, bottom
 *       (4,5,0,1,2,3), skipping planes no original vertex is outside of.  A crossing
 *       is always interpolated from the inside vertex a to the outside vertex b:
 *       t = d(a) / (d(a) - d(b)), p = fma(t, b - a, a) per attribute.
 *   N4  w > 0 required; iw = 1/w; xn = x*iw; yn = y*iw;
 *       X = lrint(fma(xn, 128 W, 128 W)), Y likewise with H: 1/256-pixel units,
 *       origin at the top-left corner of pixel (0,0), y down.  A vertex whose
 *       un-rounded coordinate leaves [-64, 256 W + 64] (or is NaN) drops the triangle.
 *   N5  fan (q0, qi, qi+1); A2 = (X1-X0)(Y2-Y0) - (X2-X0)(Y1-Y0); A2 = 0 skipped;
 *       A2 < 0: swap vertices 1 and 2 (two-sided).  Edge i is opposite vertex i,
 *       E(p) = dx (py - Yj) - dy (px - Xj) for edge j -> k.
 *   N6  covered iff every E_i > 0, or E_i = 0 on a top-left edge
 *       (dy < 0, or dy = 0 and dx > 0), at pixel centre (256 i + 128, 256 j + 128).
 *   N7  depth = (float)A2 / fma(e2,iw2, fma(e1,iw1, e0*iw0)), e_i = (float)E_i:
 *       perspective-correct clip w.  key = depth bits << 32 | original triangle id;
 *       the pixel keeps the minimum key.
 *   N8  uncovered pixel: depth = background, id = 0xFFFFFFFF, rgb = 0.
 *   N9  colour: cn = fma(e2*iw2,c2, fma(e1*iw1,c1, (e0*iw0)*c0)); out = clamp(lrint(cn/num)).
 *   N10 texture (stand-in for the paper's textured RGB sensor, Sec. 4.1): per-vertex (u,v) are
 *       interpolated like colours, u = un/num.  Texture w x h (powers of two), RGB8, with a mip
 *       pyramid: each level halves both sides (not below 1) and a texel is (a+b+c+d+2)>>2 of its
 *       2x2 parents (parents clamped at the border).  One level per fan triangle, from the
 *       oriented vertices: auv = |fma(du1,dv2, -(du2*dv1))|, r = auv*w*h*65536 / A2 (texels per
 *       pixel), level = number of times r can be quartered while r >= 4 (at most the last level).
 *       Sample: fu = u - floor(u) (0 if that is not in [0,1)), x = min((int)(fu*lw), lw-1), likewise y;
 *       the pixel takes that texel, no filtering.
 *   N11 bilinear filtering (optional; same level L and fractions fu, fv as N10): x = fu*lw - 0.5,
 *       x0 = floor(x), tx = x - x0, x1 = x0 + 1, both wrapped into [0, lw) (the texture repeats;
 *       sides are powers of two); likewise y.  Per channel, with the four texels as floats:
 *       top = fma(tx, c01 - c00, c00), bot = fma(tx, c11 - c10, c10), v = fma(ty, bot - top, top),
 *       out = clamp(lrint(v), 0, 255).  At a texel centre the result is that texel.
 *
 * Everything after N4 is exact integer arithmetic in int64.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define MAXPOLY 16

typedef struct {
    float c[4];   /* clip x, y, z, w */
    float col[3]; /* r, g, b as floats */
} overt;

typedef struct {
    int w, h, levels;
    uint8_t **level; /* level[l] = RGB8 texels of size max(w>>l,1) x max(h>>l,1) */
    int bilinear;    /* 0: N10 nearest texel, 1: N11 */
} otexture;

/* N10 / N11: the colour at fractions (fu, fv) in [0,1) of level L (lw x lh texels). */
static void fetch_texel(const otexture *tx, int L, int lw, int lh, float fu, float fv, uint8_t *out)
{
    if (!tx->bilinear) {
        int x = (int)(fu * (float)lw), y = (int)(fv * (float)lh);
        if (x > lw - 1) x = lw - 1;
        if (y > lh - 1) y = lh - 1;
        memcpy(out, tx->level[L] + 3 * ((size_t)y * (size_t)lw + (size_t)x), 3);
        return;
    }
    float x = fu * (float)lw - 0.5f, y = fv * (float)lh - 0.5f;
    float fx0 = floorf(x), fy0 = floorf(y);
    float tx_ = x - fx0, ty_ = y - fy0;
    int x0 = (int)fx0 & (lw - 1), x1 = ((int)fx0 + 1) & (lw - 1); /* two's complement: -1 wraps to lw - 1 */
    int y0 = (int)fy0 & (lh - 1), y1 = ((int)fy0 + 1) & (lh - 1);
    const uint8_t *t = tx->level[L];
    for (int c = 0; c < 3; ++c) {
        float c00 = (float)t[3 * ((size_t)y0 * lw + x0) + c], c01 = (float)t[3 * ((size_t)y0 * lw + x1) + c];
        float c10 = (float)t[3 * ((size_t)y1 * lw + x0) + c], c11 = (float)t[3 * ((size_t)y1 * lw + x1) + c];
        float top = fmaf(tx_, c01 - c00, c00), bot = fmaf(tx_, c11 - c10, c10);
        float v = fmaf(ty_, bot - top, top);
        long q = lrintf(v);
        if (q < 0) q = 0;
        if (q > 255) q = 255;
        out[c] = (uint8_t)q;
    }
}

typedef struct {
    int H, W;
    uint64_t *key;   /* [H*W] */
    uint32_t *cover; /* [H*W] or NULL: number of covering sub-triangles */
    uint8_t *rgb;    /* [H*W*3] or NULL */
    const otexture *tex; /* when set, attribute slots 0,1 hold (u,v) and colour comes from the texture */
} oframe;

static float plane_dist(const overt *v, int k)
{
    switch (k) {
    case 0: return v->c[3] + v->c[0];
    case 1: return v->c[3] - v->c[0];
    case 2: return v->c[3] + v->c[1];
    case 3: return v->c[3] - v->c[1];
    case 4: return v->c[2];
    default: return v->c[3] - v->c[2];
    }
}

/* N1 */
static void transform(const float *M, const float *p, overt *o)
{
    for (int r = 0; r < 4; ++r)
        o->c[r] = fmaf(M[r * 4 + 2], p[2], fmaf(M[r * 4 + 1], p[1], fmaf(M[r * 4 + 0], p[0], M[r * 4 + 3])));
}

/* N3: crossing point, always from the inside vertex a towards the outside vertex b */
static void intersect(const overt *a, const overt *b, int k, overt *o)
{
    float da = plane_dist(a, k), db = plane_dist(b, k);
    float t = da / (da - db);
    for (int i = 0; i < 4; ++i) o->c[i] = fmaf(t, b->c[i] - a->c[i], a->c[i]);
    for (int i = 0; i < 3; ++i) o->col[i] = fmaf(t, b->col[i] - a->col[i], a->col[i]);
}

/* The clipper's polygons hold MAXPOLY corners.  A triangle cut by six planes has at most nine in
 * exact arithmetic; rounding can make a polygon slightly non-convex, which bounds the growth per
 * plane by 4/3 (3, 4, 5, 6, 8, 10, 13).  Should a polygon ever need more, the oracle does not guess:
 * it counts the event, drops the triangle, and the render call reports failure. */
static int g_poly_overflow = 0; /* polygons that did not fit, since the last oracle_clip_stats(…, reset) */
static int g_poly_max = 0;      /* largest corner count any clipped polygon reached */

void oracle_clip_stats(int *overflows, int *max_corners, int reset)
{
    if (overflows) *overflows = g_poly_overflow;
    if (max_corners) *max_corners = g_poly_max;
    if (reset) { g_poly_overflow = 0; g_poly_max = 0; }
}

/* N2 + N3.  Returns the polygon's vertex count (0 = dropped). */
static int clip_triangle(const overt tri[3], overt *poly)
{
    int out_any[6] = {0, 0, 0, 0, 0, 0};
    for (int v = 0; v < 3; ++v)
        for (int i = 0; i < 4; ++i)
            if (!isfinite(tri[v].c[i])) return 0;
    for (int k = 0; k < 6; ++k) {
        int nout = 0;
        for (int v = 0; v < 3; ++v)
            if (!(plane_dist(&tri[v], k) >= 0.0f)) ++nout;
        if (nout == 3) return 0;
        out_any[k] = nout > 0;
    }
    overt bufa[MAXPOLY], bufb[MAXPOLY];
    overt *cur = bufa, *nxt = bufb;
    int n = 3;
    memcpy(cur, tri, 3 * sizeof(overt));
    static const int order[6] = {4, 5, 0, 1, 2, 3};
    for (int oi = 0; oi < 6; ++oi) {
        int k = order[oi];
        if (!out_any[k]) continue;
        int m = 0;
        for (int i = 0; i < n; ++i) {
            const overt *c = &cur[i];
            const overt *p = &cur[(i + n - 1) % n];
            int cin = plane_dist(c, k) >= 0.0f;
            int pin = plane_dist(p, k) >= 0.0f;
            if (m + 2 > MAXPOLY && (cin || pin)) { /* no room for what this corner may add */
#pragma omp atomic
                g_poly_overflow += 1;
                return 0;
            }
            if (cin) {
                if (!pin) intersect(c, p, k, &nxt[m++]);
                nxt[m++] = *c;
            } else if (pin) {
                intersect(p, c, k, &nxt[m++]);
            }
        }
        n = m;
        if (n > g_poly_max) {
#pragma omp critical(oracle_poly_max)
            if (n > g_poly_max) g_poly_max = n;
        }
        overt *t = cur; cur = nxt; nxt = t;
        if (n < 3) return 0;
    }
    memcpy(poly, cur, (size_t)n * sizeof(overt));
    return n;
}

static int64_t floor_div(int64_t a, int64_t b) /* b > 0 */
{
    int64_t q = a / b;
    if ((a % b) != 0 && a < 0) --q;
    return q;
}

/* N5-N9 on one fan triangle with snapped vertices */
static void raster_subtri(oframe *f, const int64_t Xi[3], const int64_t Yi[3], const float iwi[3],
                          float coli[3][3], uint32_t id)
{
    int64_t X[3] = {Xi[0], Xi[1], Xi[2]}, Y[3] = {Yi[0], Yi[1], Yi[2]};
    float iw[3] = {iwi[0], iwi[1], iwi[2]};
    float col[3][3];
    memcpy(col, coli, sizeof(col));
    int64_t A2 = (X[1] - X[0]) * (Y[2] - Y[0]) - (X[2] - X[0]) * (Y[1] - Y[0]);
    if (A2 == 0) return;
    if (A2 < 0) {
        int64_t t;
        float ft;
        t = X[1]; X[1] = X[2]; X[2] = t;
        t = Y[1]; Y[1] = Y[2]; Y[2] = t;
        ft = iw[1]; iw[1] = iw[2]; iw[2] = ft;
        for (int c = 0; c < 3; ++c) { ft = col[1][c]; col[1][c] = col[2][c]; col[2][c] = ft; }
        A2 = -A2;
    }
    int64_t minX = X[0], maxX = X[0], minY = Y[0], maxY = Y[0];
    for (int v = 1; v < 3; ++v) {
        if (X[v] < minX) minX = X[v];
        if (X[v] > maxX) maxX = X[v];
        if (Y[v] < minY) minY = Y[v];
        if (Y[v] > maxY) maxY = Y[v];
    }
    /* pixel centres 256 i + 128 inside the closed bounding box, clamped to the frame */
    int64_t i0 = -floor_div(-(minX - 128), 256), i1 = floor_div(maxX - 128, 256);
    int64_t j0 = -floor_div(-(minY - 128), 256), j1 = floor_div(maxY - 128, 256);
    if (i0 < 0) i0 = 0;
    if (j0 < 0) j0 = 0;
    if (i1 > f->W - 1) i1 = f->W - 1;
    if (j1 > f->H - 1) j1 = f->H - 1;
    for (int64_t j = j0; j <= j1; ++j) {
        for (int64_t i = i0; i <= i1; ++i) {
            int64_t px = 256 * i + 128, py = 256 * j + 128;
            int64_t E[3];
            int in = 1;
            for (int e = 0; e < 3; ++e) {
                int a = (e + 1) % 3, b = (e + 2) % 3; /* edge e runs a -> b, opposite vertex e */
                int64_t dx = X[b] - X[a], dy = Y[b] - Y[a];
                E[e] = dx * (py - Y[a]) - dy * (px - X[a]);
                int topleft = (dy < 0) || (dy == 0 && dx > 0);
                if (!(E[e] > 0 || (E[e] == 0 && topleft))) in = 0;
            }
            if (!in) continue;
            size_t p = (size_t)j * (size_t)f->W + (size_t)i;
            if (f->cover) f->cover[p]++;
            float e0 = (float)E[0], e1 = (float)E[1], e2 = (float)E[2];
            float num = fmaf(e2, iw[2], fmaf(e1, iw[1], e0 * iw[0]));
            float depth = (float)A2 / num;
            uint32_t dbits;
            memcpy(&dbits, &depth, 4);
            uint64_t k = ((uint64_t)dbits << 32) | (uint64_t)id;
            if (k < f->key[p]) {
                f->key[p] = k;
                if (f->rgb && f->tex) {
                    const otexture *tx = f->tex;
                    /* one mip level per fan triangle, from its oriented vertices */
                    float du1 = col[1][0] - col[0][0], dv1 = col[1][1] - col[0][1];
                    float du2 = col[2][0] - col[0][0], dv2 = col[2][1] - col[0][1];
                    float auv = fabsf(fmaf(du1, dv2, -(du2 * dv1)));
                    float r = ((auv * (float)tx->w) * (float)tx->h) * 65536.0f / (float)A2;
                    int L = 0;
                    while (L < tx->levels - 1 && r >= 4.0f) { r *= 0.25f; ++L; }
                    int lw = tx->w >> L, lh = tx->h >> L;
                    if (lw < 1) lw = 1;
                    if (lh < 1) lh = 1;
                    float uv[2];
                    for (int c = 0; c < 2; ++c) {
                        float cn = fmaf(e2 * iw[2], col[2][c], fmaf(e1 * iw[1], col[1][c], (e0 * iw[0]) * col[0][c]));
                        float v = cn / num;
                        float fr = v - floorf(v);
                        if (!(fr >= 0.0f && fr < 1.0f)) fr = 0.0f;
                        uv[c] = fr;
                    }
                    fetch_texel(tx, L, lw, lh, uv[0], uv[1], f->rgb + p * 3);
                } else if (f->rgb) {
                    for (int c = 0; c < 3; ++c) {
                        float cn = fmaf(e2 * iw[2], col[2][c], fmaf(e1 * iw[1], col[1][c], (e0 * iw[0]) * col[0][c]));
                        float v = cn / num;
                        long q = lrintf(v);
                        if (!(v == v)) q = 0;
                        if (q < 0) q = 0;
                        if (q > 255) q = 255;
                        f->rgb[p * 3 + c] = (uint8_t)q;
                    }
                }
            }
        }
    }
}

/* N2-N7 for one scene triangle already transformed to clip space */
static void raster_clip_tri(oframe *f, const overt tri[3], uint32_t id)
{
    overt poly[MAXPOLY];
    int n = clip_triangle(tri, poly);
    if (n < 3) return;
    int64_t X[MAXPOLY], Y[MAXPOLY];
    float iw[MAXPOLY];
    const float sx = 128.0f * (float)f->W, sy = 128.0f * (float)f->H;
    for (int v = 0; v < n; ++v) {
        float w = poly[v].c[3];
        if (!(w > 0.0f)) return;
        iw[v] = 1.0f / w;
        float xn = poly[v].c[0] * iw[v], yn = poly[v].c[1] * iw[v];
        float fx = fmaf(xn, sx, sx), fy = fmaf(yn, sy, sy);
        if (!(fx >= -64.0f && fx <= 2.0f * sx + 64.0f && fy >= -64.0f && fy <= 2.0f * sy + 64.0f)) return;
        X[v] = (int64_t)lrintf(fx);
        Y[v] = (int64_t)lrintf(fy);
    }
    for (int i = 1; i + 1 < n; ++i) {
        int64_t tx[3] = {X[0], X[i], X[i + 1]}, ty[3] = {Y[0], Y[i], Y[i + 1]};
        float tw[3] = {iw[0], iw[i], iw[i + 1]};
        float tc[3][3];
        for (int c = 0; c < 3; ++c) { tc[0][c] = poly[0].col[c]; tc[1][c] = poly[i].col[c]; tc[2][c] = poly[i + 1].col[c]; }
        raster_subtri(f, tx, ty, tw, tc, id);
    }
}

static void render_env(oframe *f, const float *verts, const uint32_t *idx, uint32_t T, const uint8_t *colors,
                       const float *uvs, const float *M)
{
    for (uint32_t t = 0; t < T; ++t) {
        overt tri[3];
        for (int v = 0; v < 3; ++v) {
            uint32_t vi = idx[3 * (size_t)t + v];
            transform(M, verts + 3 * (size_t)vi, &tri[v]);
            for (int c = 0; c < 3; ++c) tri[v].col[c] = colors ? (float)colors[3 * (size_t)vi + c] : 0.0f;
            if (uvs) {
                tri[v].col[0] = uvs[2 * (size_t)vi + 0];
                tri[v].col[1] = uvs[2 * (size_t)vi + 1];
                tri[v].col[2] = 0.0f;
            }
        }
        raster_clip_tri(f, tri, t);
    }
}

/* ------------------------------------------------------------------ exported */

/* Render B environments of ONE scene.  All pointers are host memory.
 * depth [B][H][W] float, tri_id [B][H][W] uint32 (may be NULL), rgb [B][H][W][3] uint8
 * (NULL unless colors given), cover [B][H][W] uint32 (may be NULL).
 * nthreads <= 0 uses every core.  Returns the number of threads used. */
/* N10: build the mip pyramid of an RGB8 texture (w, h powers of two). */
static otexture *build_pyramid(const uint8_t *texels, int w, int h)
{
    otexture *t = (otexture *)malloc(sizeof(otexture));
    t->w = w;
    t->h = h;
    t->bilinear = 0;
    int levels = 1;
    for (int a = w, b = h; a > 1 || b > 1; a = a > 1 ? a / 2 : 1, b = b > 1 ? b / 2 : 1) ++levels;
    t->levels = levels;
    t->level = (uint8_t **)malloc((size_t)levels * sizeof(uint8_t *));
    t->level[0] = (uint8_t *)malloc((size_t)w * h * 3);
    memcpy(t->level[0], texels, (size_t)w * h * 3);
    int pw = w, ph = h;
    for (int l = 1; l < levels; ++l) {
        int lw = pw > 1 ? pw / 2 : 1, lh = ph > 1 ? ph / 2 : 1;
        t->level[l] = (uint8_t *)malloc((size_t)lw * lh * 3);
        for (int y = 0; y < lh; ++y)
            for (int x = 0; x < lw; ++x) {
                int x0 = 2 * x, y0 = 2 * y, x1 = 2 * x + 1, y1 = 2 * y + 1;
                if (x0 > pw - 1) x0 = pw - 1;
                if (x1 > pw - 1) x1 = pw - 1;
                if (y0 > ph - 1) y0 = ph - 1;
                if (y1 > ph - 1) y1 = ph - 1;
                for (int c = 0; c < 3; ++c) {
                    int s = t->level[l - 1][3 * (y0 * pw + x0) + c] + t->level[l - 1][3 * (y0 * pw + x1) + c] +
                            t->level[l - 1][3 * (y1 * pw + x0) + c] + t->level[l - 1][3 * (y1 * pw + x1) + c];
                    t->level[l][3 * (y * lw + x) + c] = (uint8_t)((s + 2) >> 2);
                }
            }
        pw = lw;
        ph = lh;
    }
    return t;
}

static void free_pyramid(otexture *t)
{
    if (!t) return;
    for (int l = 0; l < t->levels; ++l) free(t->level[l]);
    free(t->level);
    free(t);
}

int oracle_render_textured(const float *verts, uint32_t V, const uint32_t *idx, uint32_t T, const uint8_t *colors,
                           const float *uvs, const uint8_t *texels, int tex_w, int tex_h, const float *view_proj,
                           uint32_t B, int H, int W, float background, float *depth, uint32_t *tri_id, uint8_t *rgb,
                           uint32_t *cover, int nthreads);
int oracle_render_filtered(const float *verts, uint32_t V, const uint32_t *idx, uint32_t T, const uint8_t *colors,
                           const float *uvs, const uint8_t *texels, int tex_w, int tex_h, int bilinear,
                           const float *view_proj, uint32_t B, int H, int W, float background, float *depth,
                           uint32_t *tri_id, uint8_t *rgb, uint32_t *cover, int nthreads);

int oracle_render(const float *verts, uint32_t V, const uint32_t *idx, uint32_t T, const uint8_t *colors,
                  const float *view_proj, uint32_t B, int H, int W, float background, float *depth,
                  uint32_t *tri_id, uint8_t *rgb, uint32_t *cover, int nthreads)
{
    return oracle_render_textured(verts, V, idx, T, colors, NULL, NULL, 0, 0, view_proj, B, H, W, background, depth, tri_id,
                                  rgb, cover, nthreads);
}

/* As oracle_render, with optional texturing: uvs [V][2] float and texels [tex_h][tex_w][3] uint8
 * (both NULL for per-vertex colours). */
int oracle_render_textured(const float *verts, uint32_t V, const uint32_t *idx, uint32_t T, const uint8_t *colors,
                           const float *uvs, const uint8_t *texels, int tex_w, int tex_h, const float *view_proj,
                           uint32_t B, int H, int W, float background, float *depth, uint32_t *tri_id, uint8_t *rgb,
                           uint32_t *cover, int nthreads)
{
    return oracle_render_filtered(verts, V, idx, T, colors, uvs, texels, tex_w, tex_h, 0, view_proj, B, H, W, background, depth,
                                  tri_id, rgb, cover, nthreads);
}

/* As oracle_render_textured; bilinear = 1 samples the texture by rule N11 instead of N10. */
int oracle_render_filtered(const float *verts, uint32_t V, const uint32_t *idx, uint32_t T, const uint8_t *colors,
                           const float *uvs, const uint8_t *texels, int tex_w, int tex_h, int bilinear,
                           const float *view_proj, uint32_t B, int H, int W, float background, float *depth,
                           uint32_t *tri_id, uint8_t *rgb, uint32_t *cover, int nthreads)
{
    (void)V;
    otexture *tex = (uvs && texels) ? build_pyramid(texels, tex_w, tex_h) : NULL;
    if (tex) tex->bilinear = bilinear != 0;
    int used = 1;
    const int overflow_before = g_poly_overflow;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_num_procs();
    used = nthreads;
#else
    nthreads = 1;
#endif
    size_t npix = (size_t)H * (size_t)W;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int64_t b = 0; b < (int64_t)B; ++b) {
        oframe f;
        f.H = H;
        f.W = W;
        f.key = (uint64_t *)malloc(npix * sizeof(uint64_t));
        for (size_t p = 0; p < npix; ++p) f.key[p] = ~(uint64_t)0;
        f.cover = cover ? cover + (size_t)b * npix : NULL;
        if (f.cover) memset(f.cover, 0, npix * sizeof(uint32_t));
        f.rgb = (rgb && (colors || tex)) ? rgb + (size_t)b * npix * 3 : NULL;
        f.tex = tex;
        if (f.rgb) memset(f.rgb, 0, npix * 3);
        render_env(&f, verts, idx, T, colors, tex ? uvs : NULL, view_proj + 16 * (size_t)b);
        for (size_t p = 0; p < npix; ++p) {
            uint64_t k = f.key[p];
            float d = background;
            uint32_t id = 0xFFFFFFFFu;
            if (k != ~(uint64_t)0) {
                uint32_t bits = (uint32_t)(k >> 32);
                memcpy(&d, &bits, 4);
                id = (uint32_t)(k & 0xFFFFFFFFu);
            }
            depth[(size_t)b * npix + p] = d;
            if (tri_id) tri_id[(size_t)b * npix + p] = id;
        }
        free(f.key);
    }
    free_pyramid(tex);
    if (g_poly_overflow != overflow_before) return -1; /* a clipped polygon outgrew MAXPOLY: the frames are not to be trusted */
    return used;
}

/* Supersampled output (the paper renders at a higher resolution and downsamples, Sec. 4.1 and
 * appendix): the 2H x 2W frame `depth` (and optionally `rgb`) is averaged over 2x2 blocks.
 * Depth: ((d00 + d01) + (d10 + d11)) * 0.25 in float32, in that order, background samples counting
 * with the value the frame holds for them.  Colour: (a + b + c + d + 2) >> 2 per channel.
 *   depth [B][2H][2W] float32 -> out_depth [B][H][W];  rgb [B][2H][2W][3] uint8 -> out_rgb [B][H][W][3] (both or neither) */
void oracle_downsample2(const float *depth, const uint8_t *rgb, uint32_t B, int H, int W, float *out_depth, uint8_t *out_rgb)
{
    const size_t W2 = 2 * (size_t)W, H2 = 2 * (size_t)H;
    for (uint32_t b = 0; b < B; ++b)
        for (int y = 0; y < H; ++y)
            for (int x = 0; x < W; ++x) {
                const size_t s = (size_t)b * H2 * W2 + (size_t)(2 * y) * W2 + (size_t)(2 * x);
                const float top = depth[s] + depth[s + 1];
                const float bottom = depth[s + W2] + depth[s + W2 + 1];
                out_depth[((size_t)b * H + y) * W + x] = (top + bottom) * 0.25f;
                if (rgb && out_rgb)
                    for (int c = 0; c < 3; ++c) {
                        const int sum = rgb[3 * s + c] + rgb[3 * (s + 1) + c] + rgb[3 * (s + W2) + c] + rgb[3 * (s + W2 + 1) + c];
                        out_rgb[(((size_t)b * H + y) * W + x) * 3 + c] = (uint8_t)((sum + 2) >> 2);
                    }
            }
}

/* N10 / N11 alone: the colour the sampling rule gives for (u, v) at mip level L. */
void oracle_sample_filtered(const uint8_t *texels, int tex_w, int tex_h, int L, float u, float v, int bilinear, uint8_t *rgb_out)
{
    otexture *tx = build_pyramid(texels, tex_w, tex_h);
    tx->bilinear = bilinear != 0;
    if (L > tx->levels - 1) L = tx->levels - 1;
    int lw = tx->w >> L, lh = tx->h >> L;
    if (lw < 1) lw = 1;
    if (lh < 1) lh = 1;
    float fu = u - floorf(u), fv = v - floorf(v);
    if (!(fu >= 0.0f && fu < 1.0f)) fu = 0.0f;
    if (!(fv >= 0.0f && fv < 1.0f)) fv = 0.0f;
    fetch_texel(tx, L, lw, lh, fu, fv, rgb_out);
    free_pyramid(tx);
}

void oracle_sample(const uint8_t *texels, int tex_w, int tex_h, int L, float u, float v, uint8_t *rgb_out)
{
    oracle_sample_filtered(texels, tex_w, tex_h, L, u, v, 0, rgb_out);
}

/* N5-N6 alone: coverage counts of triangles given directly in 1/256-pixel integer
 * coordinates xy[n][3][2]; cover[H][W] is incremented.  For pinning the fill rule. */
void oracle_cover_fixed(const int32_t *xy, uint32_t n, int H, int W, uint32_t *cover)
{
    size_t npix = (size_t)H * (size_t)W;
    uint64_t *key = (uint64_t *)malloc(npix * sizeof(uint64_t));
    for (size_t p = 0; p < npix; ++p) key[p] = ~(uint64_t)0;
    oframe f = {H, W, key, cover, NULL, NULL};
    for (uint32_t t = 0; t < n; ++t) {
        int64_t X[3], Y[3];
        float iw[3] = {1.0f, 1.0f, 1.0f};
        float col[3][3] = {{0}};
        for (int v = 0; v < 3; ++v) { X[v] = xy[6 * t + 2 * v]; Y[v] = xy[6 * t + 2 * v + 1]; }
        raster_subtri(&f, X, Y, iw, col, t);
    }
    free(key);
}

/* N1-N3 alone: transform + clip one triangle; poly_out[MAXPOLY][4] receives clip coords.
 * Returns the vertex count.  For pinning the clipper. */
int oracle_clip(const float *M, const float *tri_xyz, float *poly_out)
{
    overt tri[3], poly[MAXPOLY];
    for (int v = 0; v < 3; ++v) {
        transform(M, tri_xyz + 3 * v, &tri[v]);
        tri[v].col[0] = tri[v].col[1] = tri[v].col[2] = 0.0f;
    }
    int n = clip_triangle(tri, poly);
    for (int v = 0; v < n; ++v)
        for (int i = 0; i < 4; ++i) poly_out[4 * v + i] = poly[v].c[i];
    return n;
}
