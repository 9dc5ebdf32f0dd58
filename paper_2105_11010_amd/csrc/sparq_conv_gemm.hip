// Host entry point of the fused SPARQ convolution: validation, the channel-padding
// pre-pass for channel counts that are not a multiple of 16, and the choice of tile shape.
#include "sparq_conv_gemm_kernel.h"

#include <string.h>


using namespace sparq;

#include <stdlib.h>

namespace {

struct TileEntry { const char* name; int tm, tn; TileLauncher fn; };
const TileEntry kTiles[] = {
    {"128x128", 128, 128, launch_tile_128x128_w2x2_a1b2},
    {"128x256", 128, 256, launch_tile_128x256_w1x4_a2b3},
    {"128x512", 128, 512, launch_tile_128x512_w1x4_a1b3},
};

// Tile choice: the widest output-channel tile the layer fills, so that an activation
// is gathered and trimmed as few times as possible.  SPARQ_TILE=<name> (a tuning knob,
// not part of the interface) forces one.
TileLauncher pick_tile(const ConvGeom& g) {
    if (const char* e = getenv("SPARQ_TILE"))
        for (const TileEntry& t : kTiles)
            if (!strcmp(e, t.name) && t.tn <= g.Np) return t.fn;   // weight loads must stay inside the padded buffer
    if (g.N > 256) return kTiles[2].fn;
    if (g.N > 128) return kTiles[1].fn;
    return kTiles[0].fn;
}

}  // namespace

extern "C" size_t sparq_workspace_bytes(const sparq_conv_desc* desc, const sparq_mode* mode) {
    ConvGeom g;
    if (!conv_geom(desc, &g) || !mode_valid(mode)) return 0;
    if (g.Cp == g.C) return 0;
    return (size_t)round_up((int64_t)g.B * g.H * g.W * g.Cp, 256);
}

extern "C" sparq_status sparq_conv_gemm(const uint8_t* x, const void* packed_w, const sparq_conv_desc* desc,
                                        const sparq_mode* mode, int32_t* acc, const float* scale, float* out,
                                        void* workspace, size_t workspace_bytes, void* stream) {
    ConvGeom g;
    if (!x || !packed_w || !conv_geom(desc, &g) || !mode_valid(mode)) return SPARQ_EINVAL;
    if (!acc && !out) return SPARQ_EINVAL;
    if (out && !scale) return SPARQ_EINVAL;
    if (!aligned(x, 16) || !aligned(packed_w, 256) || (acc && !aligned(acc, 16)) || (out && !aligned(out, 16)) ||
        (scale && !aligned(scale, 16)))
        return SPARQ_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);

    const uint8_t* xin = x;
    TrimKind kind = trim_kind(mode);
    size_t x_bytes = g.x_bytes;
    if (g.Cp != g.C) {
        // Channel counts that are not a multiple of 16: trim into a channel-padded copy
        // first (pairs stay inside the row; padded channels are zeros with zero weights),
        // then contract the copy without further trimming.
        const size_t need = sparq_workspace_bytes(desc, mode);
        if (!workspace || !aligned(workspace, 256)) return SPARQ_EINVAL;
        if (workspace_bytes < need) return SPARQ_EWORKSPACE;
        x_bytes = (size_t)g.B * g.H * g.W * g.Cp;
        if (x_bytes >= kInvalidOffset) return SPARQ_EUNSUPPORTED;
        const sparq_status st = launch_trim_pad(x, static_cast<uint8_t*>(workspace), (int64_t)g.B * g.H * g.W, g.C,
                                                g.Cp, mode, s);
        if (st != SPARQ_OK) return st;
        xin = static_cast<const uint8_t*>(workspace);
        kind = kTrimNone;
    }
    if (x_bytes >= kInvalidOffset) return SPARQ_EUNSUPPORTED;

    GemmParams p{};
    p.x = xin;
    p.wpk = static_cast<const uint8_t*>(packed_w) + g.w_off;
    p.colsum = static_cast<const int32_t*>(packed_w);
    p.acc = acc;
    p.scale = scale;
    p.out = out;
    p.M = g.M;
    p.x_bytes = (uint32_t)x_bytes;
    p.N = g.N; p.Np = g.Np; p.Kk = g.Kk; p.nkb = g.Kp / kStepK;
    p.H = g.H; p.W = g.W; p.C = g.Cp; p.Ho = g.Ho; p.Wo = g.Wo; p.KH = g.KH; p.KW = g.KW;
    p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw;
    p.rcp_c = 1.0f / (float)g.Cp;
    p.rcp_kw = 1.0f / (float)g.KW;
    p.luts = make_luts(mode->window_bits, mode->shift_mask);

    return pick_tile(g)(kind, p, s);
}
