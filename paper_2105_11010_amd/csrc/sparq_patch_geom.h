// Index arithmetic of the input-patch convolution kernel, shared by device and host code.
//
// A tile is PatchGeom::tm (128 or 256) consecutive output pixels in (b, oy, ox) order.  All input pixels that any
// filter tap of any of those outputs touches form a rectangle of "virtual rows" x columns:
//
//   virtual row  v = b * Hv + (iy + pad_h),  Hv = H + 2 * pad_h     (padding rows included)
//   column       ix in [xlo, xlo + pwt)                             (padding columns included)
//
// The rectangle (the tile's patch) is staged once in LDS, trimmed, and every tap reads its
// operands from it at a shifted position, so an activation is loaded and trimmed once per tile
// instead of once per tap.  Patch pixel index: (v - v0) * pwt + (ix - xlo).
//
// Divisions use a float reciprocal plus a one-step correction; all dividends stay below 2^22,
// which the host checks, so the result is exact.  The file compiles for the host as well, where a
// test walks every tile of many shapes and compares against plain integer arithmetic.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define SPARQ_GEOM_HD __host__ __device__ __forceinline__
#else
#define SPARQ_GEOM_HD inline
#endif

namespace sparq {

constexpr int kPatchTM = 128;              // output pixels per tile (default; PatchGeom::tm is what counts)
constexpr int kPatchMaxDividend = 1 << 22;

struct PatchGeom {                          // per launch
    int M;                                  // B * Ho * Wo
    int tm;                                 // output pixels per tile
    int B, H, W, Ho, Wo, KH, KW, sh, sw, ph, pw;
    int Hv;                                 // H + 2 * ph
    float rcp_wo, rcp_ho, rcp_hv;
    // 1x1 filters without padding are run as one long row of M pixels (B = H = 1, W = M).  With a
    // stride the m-th pixel of that row is pixel (oy * rm_sh, ox * rm_sw) of image b in the real
    // tensor, m = (b * rm_ho + oy) * rm_wo + ox; rm_wo == 0: no stride, the row is the tensor itself.
    int rm_wo, rm_ho, rm_h, rm_w, rm_sh, rm_sw;
    float rm_rcp_wo, rm_rcp_ho;
};

// Pixel index of the m-th pixel of the long row in the real tensor (see PatchGeom::rm_wo).
SPARQ_GEOM_HD int remap_pixel(const PatchGeom& g, int m);

struct TilePatch {                          // per tile, uniform over the workgroup
    int m0;                                 // first output pixel
    int v0;                                 // first virtual row
    int xlo;                                // first column (may be negative: padding)
    int pwt;                                // columns
    int npix;                               // rows * columns
    float rcp_pwt;
};

// a / d for 0 <= a < 2^22, d > 0, rcp = 1.0f / d
SPARQ_GEOM_HD int div_rcp(int a, int d, float rcp, int* rem) {
    int q = (int)((float)a * rcp);
    int r = a - q * d;
    const int lo = r < 0 ? 1 : 0;
    q -= lo;
    r += lo ? d : 0;
    const int hi = r >= d ? 1 : 0;
    q += hi;
    r -= hi ? d : 0;
    *rem = r;
    return q;
}

SPARQ_GEOM_HD int remap_pixel(const PatchGeom& g, int m) {
    int ox, oy;
    const int r = div_rcp(m, g.rm_wo, g.rm_rcp_wo, &ox);
    const int b = div_rcp(r, g.rm_ho, g.rm_rcp_ho, &oy);
    return (b * g.rm_h + oy * g.rm_sh) * g.rm_w + ox * g.rm_sw;
}

// The geometry the patch kernel runs a convolution with (set-up shared by the library and its host test).
// 1x1 filters without padding become one long row (with a pixel remap when strided).
inline PatchGeom make_patch_geom(int B, int H, int W, int KH, int KW, int sh, int sw, int ph, int pw, int tm = kPatchTM) {
    PatchGeom q{};
    q.tm = tm;
    const int Ho = (H + 2 * ph - KH) / sh + 1, Wo = (W + 2 * pw - KW) / sw + 1;
    const int M = B * Ho * Wo;
    if (KH == 1 && KW == 1 && ph == 0 && pw == 0) {
        q.B = 1; q.H = 1; q.W = M; q.Ho = 1; q.Wo = M; q.KH = q.KW = 1; q.sh = q.sw = 1;
        if (sh != 1 || sw != 1) {
            q.rm_wo = Wo; q.rm_ho = Ho; q.rm_h = H; q.rm_w = W; q.rm_sh = sh; q.rm_sw = sw;
            q.rm_rcp_wo = 1.0f / (float)Wo; q.rm_rcp_ho = 1.0f / (float)Ho;
        }
    } else {
        q.B = B; q.H = H; q.W = W; q.Ho = Ho; q.Wo = Wo; q.KH = KH; q.KW = KW;
        q.sh = sh; q.sw = sw; q.ph = ph; q.pw = pw;
    }
    q.M = M;
    q.Hv = q.H + 2 * q.ph;
    q.rcp_wo = 1.0f / (float)q.Wo; q.rcp_ho = 1.0f / (float)q.Ho; q.rcp_hv = 1.0f / (float)q.Hv;
    return q;
}

// virtual row of tap row 0 and first column of tap column 0 for output pixel m
SPARQ_GEOM_HD void out_pixel_origin(const PatchGeom& g, int m, int* v, int* x) {
    int ox, oy;
    const int r = div_rcp(m, g.Wo, g.rcp_wo, &ox);
    const int b = div_rcp(r, g.Ho, g.rcp_ho, &oy);
    *v = b * g.Hv + oy * g.sh;
    *x = ox * g.sw - g.pw;
}

SPARQ_GEOM_HD TilePatch tile_patch(const PatchGeom& g, int m0) {
    TilePatch t;
    t.m0 = m0;
    const int m1 = (m0 + g.tm - 1 < g.M - 1) ? m0 + g.tm - 1 : g.M - 1;
    int va, xa, vb, xb;
    out_pixel_origin(g, m0, &va, &xa);
    out_pixel_origin(g, m1, &vb, &xb);
    int ox0, ox1;
    const int r0 = div_rcp(m0, g.Wo, g.rcp_wo, &ox0);
    const int r1 = div_rcp(m1, g.Wo, g.rcp_wo, &ox1);
    t.v0 = va;
    const int nrows = vb - va + g.KH;
    if (r0 == r1) {                         // one output row: only the columns it needs
        t.xlo = xa;
        t.pwt = xb - xa + g.KW;
    } else {                                // several rows: full width
        t.xlo = -g.pw;
        t.pwt = (g.Wo - 1) * g.sw + g.KW;
    }
    t.npix = nrows * t.pwt;
    t.rcp_pwt = 1.0f / (float)t.pwt;
    return t;
}

// Upper bound of TilePatch::npix over all tiles of a launch (closed form, no tile walk).
inline int64_t patch_npix_bound(const PatchGeom& g) {
    const int64_t rows_total = (int64_t)g.B * g.Ho;
    int64_t d = (g.tm - 2) / g.Wo + 1;                           // largest r1 - r0 of a tile
    if (g.M <= 1 || g.tm == 1) d = 0;
    if (d > rows_total - 1) d = rows_total - 1;
    if (g.Wo >= g.M) d = 0;
    const int64_t gap = g.Hv - (int64_t)g.Ho * g.sh > 0 ? g.Hv - (int64_t)g.Ho * g.sh : 0;   // unused virtual rows between images
    const int64_t crossings = (d + g.Ho - 1) / g.Ho;
    const int64_t nrows = d * g.sh + g.KH + crossings * gap;
    int64_t single = (int64_t)(g.tm - 1) * g.sw + g.KW;          // widest one-row tile
    const int64_t full = (int64_t)(g.Wo - 1) * g.sw + g.KW;
    if (single > full) single = full;
    const int64_t pwt = d > 0 ? full : single;
    return nrows * pwt;
}

// Patch pixel -> byte offset of its channel 0 in the NHWC tensor with C channels per pixel,
// or -1 for padding (outside the image) and for pixels past the patch.  Branch-free.
SPARQ_GEOM_HD int64_t patch_pixel_offset(const PatchGeom& g, const TilePatch& t, int pix, int C) {
    int px, iyp;
    const int row = div_rcp(pix, t.pwt, t.rcp_pwt, &px);
    const int b = div_rcp(t.v0 + row, g.Hv, g.rcp_hv, &iyp);
    const int iy = iyp - g.ph, ix = t.xlo + px;
    const bool ok = (pix < t.npix) & (b < g.B) & ((unsigned)iy < (unsigned)g.H) & ((unsigned)ix < (unsigned)g.W);
    int64_t off = (((int64_t)b * g.H + iy) * g.W + ix) * C;
    if (g.rm_wo) off = (int64_t)remap_pixel(g, ok ? ix : 0) * C;
    return ok ? off : -1;
}

// The same in 32-bit arithmetic for tensors below 2 GiB; `invalid` is returned in place of -1.
// REMAP = false compiles the pixel remap of strided 1x1 layers out (callers that never see one).
template <bool REMAP = true>
SPARQ_GEOM_HD uint32_t patch_pixel_offset_u32(const PatchGeom& g, const TilePatch& t, int pix, int C, uint32_t invalid) {
    int px, iyp;
    const int row = div_rcp(pix, t.pwt, t.rcp_pwt, &px);
    const int b = div_rcp(t.v0 + row, g.Hv, g.rcp_hv, &iyp);
    const int iy = iyp - g.ph, ix = t.xlo + px;
    const bool ok = (pix < t.npix) & (b < g.B) & ((unsigned)iy < (unsigned)g.H) & ((unsigned)ix < (unsigned)g.W);
    uint32_t off = (uint32_t)(((b * g.H + iy) * g.W + ix) * C);
    if (REMAP && g.rm_wo) off = (uint32_t)(remap_pixel(g, ok ? ix : 0) * C);
    return ok ? off : invalid;
}

// Patch pixel index of output pixel m's tap (0, 0); tap (kh, kw) sits kh * pwt + kw further.
SPARQ_GEOM_HD int patch_pixel_of_output(const PatchGeom& g, const TilePatch& t, int m) {
    int v, x;
    out_pixel_origin(g, m, &v, &x);
    return (v - t.v0) * t.pwt + (x - t.xlo);
}

}  // namespace sparq
