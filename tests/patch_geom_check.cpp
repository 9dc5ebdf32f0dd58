// Host check of the input-patch index arithmetic (sparq_patch_geom.h): for every tile of a
// convolution shape, every output pixel and every filter tap, the patch pixel the kernel would
// read must hold exactly the input pixel the convolution's definition names (or padding), lie
// inside the patch, and the patch must not exceed the closed-form size bound.
// Both tile heights the kernels use (128 and 256 output pixels) are walked.
//   usage: patch_geom_check B H W KH KW stride_h stride_w pad_h pad_w   -> prints "ok <tiles> <max npix> <bound>" (of the 128-pixel walk)
#include <stdio.h>
#include <stdlib.h>

#include "../paper_2105_11010_amd/csrc/sparq_patch_geom.h"

using namespace sparq;

static int walk(int B, int H, int W, int KH, int KW, int sh, int sw, int ph, int pw, int tm, bool report) {
    const PatchGeom g = make_patch_geom(B, H, W, KH, KW, sh, sw, ph, pw, tm);      // as the library sets it up
    const int Ho = (H + 2 * ph - KH) / sh + 1, Wo = (W + 2 * pw - KW) / sw + 1;
    const int C = 16;
    const long long bound = patch_npix_bound(g);
    long long maxpix = 0;
    int tiles = 0;
    for (int m0 = 0; m0 < g.M; m0 += tm, ++tiles) {
        const TilePatch t = tile_patch(g, m0);
        if (t.npix > maxpix) maxpix = t.npix;
        if (t.npix > bound) { printf("FAIL bound: tile %d npix %d > %lld\n", tiles, t.npix, bound); return 1; }
        for (int m = m0; m < m0 + tm && m < g.M; ++m) {
            const int ox = m % Wo, oy = (m / Wo) % Ho, b = m / (Wo * Ho);
            const int base = patch_pixel_of_output(g, t, m);
            for (int kh = 0; kh < KH; ++kh)
                for (int kw = 0; kw < KW; ++kw) {
                    const int pix = base + kh * t.pwt + kw;
                    if (pix < 0 || pix >= t.npix) { printf("FAIL range: m %d tap %d,%d pix %d npix %d\n", m, kh, kw, pix, t.npix); return 1; }
                    const int iy = oy * sh - ph + kh, ix = ox * sw - pw + kw;
                    const long long want = (iy < 0 || iy >= H || ix < 0 || ix >= W) ? -1 : (((long long)b * H + iy) * W + ix) * C;
                    const long long got = patch_pixel_offset(g, t, pix, C);
                    if (got != want) { printf("FAIL map: m %d tap %d,%d got %lld want %lld\n", m, kh, kw, got, want); return 1; }
                    const uint32_t got32 = patch_pixel_offset_u32(g, t, pix, C, 0x80000000u);
                    if (got32 != (want < 0 ? 0x80000000u : (uint32_t)want)) { printf("FAIL map32: m %d tap %d,%d\n", m, kh, kw); return 1; }
                }
        }
        // pixels past the patch must decode as "nothing"
        if (patch_pixel_offset(g, t, t.npix, C) != -1) { printf("FAIL tail\n"); return 1; }
    }
    if (report) printf("ok %d %lld %lld\n", tiles, maxpix, bound);
    return 0;
}

int main(int argc, char** argv) {
    if (argc < 10) return 2;
    const int B = atoi(argv[1]), H = atoi(argv[2]), W = atoi(argv[3]), KH = atoi(argv[4]), KW = atoi(argv[5]);
    const int sh = atoi(argv[6]), sw = atoi(argv[7]), ph = atoi(argv[8]), pw = atoi(argv[9]);
    if (int rc = walk(B, H, W, KH, KW, sh, sw, ph, pw, 256, false)) return rc;
    return walk(B, H, W, KH, KW, sh, sw, ph, pw, 128, true);
}
