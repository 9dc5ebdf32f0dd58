// Host entry point of the fused SPARQ convolution: validation, the channel-padding
// pre-pass for channel counts that are not a multiple of 16, and the choice of tile shape.
#include "sparq_conv_gemm_kernel.h"
#include "sparq_conv_patch_kernel.h"

#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>

using namespace sparq;

namespace {

// ---- the one test / tuning hook (sparq_set_tuning): process-wide overrides of the kernel choice ----
struct Tuning {
    int path = 0;             // 0: rules decide, 1: gather kernel, 2: input-patch kernel
    char tile[16] = "";       // gather kernel tile "128x128" | "128x256" | "128x512"
    int patch_tn = 0;         // input-patch kernel: output channels per tile (64 / 128 / 256), 0: rules decide
    int patch_ws = -1;        // 1 / 0: wave-specialised / plain form, -1: rules decide
};
Tuning g_tuning;
std::mutex g_tuning_mu;
Tuning current_tuning() {
    std::lock_guard<std::mutex> lock(g_tuning_mu);
    return g_tuning;
}

struct TileEntry { const char* name; int tm, tn; TileLauncher fn; };
const TileEntry kTiles[] = {
    {"128x128", 128, 128, launch_tile_128x128_w2x2_a4b2},
    {"128x256", 128, 256, launch_tile_128x256_w1x4_a2b3},
    {"128x512", 128, 512, launch_tile_128x512_w1x4_half},
};

// Tile choice: the widest output-channel tile the layer fills, so that an activation
// is gathered and trimmed as few times as possible; the tuning hook forces one.
// A tile shape is usable only if all its weight loads stay inside the padded buffer; the 512-wide tile's
// main loop also needs every 64-byte reduction step to lie inside one filter tap (more than 32 channels).
bool tile_fits(int tn, const ConvGeom& g) { return round_up(g.N, tn) <= g.Np && (tn != 512 || g.Cq % kStepK == 0); }

// byte_output: the requantised uint8 output, which the 128x512 tile does not have.
TileLauncher pick_tile(const ConvGeom& g, const Tuning& tune, bool byte_output = false) {
    if (tune.tile[0])
        for (const TileEntry& t : kTiles)
            if (!strcmp(tune.tile, t.name) && tile_fits(t.tn, g) && !(byte_output && t.tn == 512)) return t.fn;
    if (g.N > 256 && tile_fits(512, g) && !byte_output) return kTiles[2].fn;
    if (g.N > 128) return kTiles[1].fn;
    return kTiles[0].fn;
}

// ---- input-patch kernel: eligibility and variant choice --------------------------------------
struct PatchVariant { int tn, ac, cbs; PatchLauncher fn; PatchLauncher fn_ws; PatchLauncher fn_sp; };   // plain, wave-specialised, sparse weights
const PatchVariant kPatchVariants[] = {
    {64, 2, 1, launch_patch_n64_a2c1, launch_patch_ws_n64_a2c1, launch_patch_sp_n64_a2c1},
    {64, 4, 1, launch_patch_n64_a4c1, launch_patch_ws_n64_a4c1, launch_patch_sp_n64_a4c1},
    {64, 8, 1, launch_patch_n64_a8c1, launch_patch_ws_n64_a8c1, launch_patch_sp_n64_a8c1},
    {64, 12, 1, launch_patch_n64_a12c1, launch_patch_ws_n64_a12c1, launch_patch_sp_n64_a12c1},
    {64, 4, 2, launch_patch_n64_a4c2, launch_patch_ws_n64_a4c2, launch_patch_sp_n64_a4c2},
    {64, 8, 4, launch_patch_n64_a8c4, launch_patch_ws_n64_a8c4, launch_patch_sp_n64_a8c4},
    {128, 2, 1, launch_patch_n128_a2c1, launch_patch_ws_n128_a2c1, launch_patch_sp_n128_a2c1},
    {128, 4, 1, launch_patch_n128_a4c1, launch_patch_ws_n128_a4c1, launch_patch_sp_n128_a4c1},
    {128, 8, 1, launch_patch_n128_a8c1, launch_patch_ws_n128_a8c1, launch_patch_sp_n128_a8c1},
    {128, 12, 1, launch_patch_n128_a12c1, launch_patch_ws_n128_a12c1, launch_patch_sp_n128_a12c1},
    {128, 4, 2, launch_patch_n128_a4c2, launch_patch_ws_n128_a4c2, launch_patch_sp_n128_a4c2},
    {128, 8, 4, launch_patch_n128_a8c4, launch_patch_ws_n128_a8c4, launch_patch_sp_n128_a8c4},
    {256, 2, 1, launch_patch_n256_a2c1, launch_patch_ws_n256_a2c1, launch_patch_sp_n256_a2c1},
    {256, 4, 1, launch_patch_n256_a4c1, launch_patch_ws_n256_a4c1, launch_patch_sp_n256_a4c1},
    {256, 8, 1, launch_patch_n256_a8c1, launch_patch_ws_n256_a8c1, launch_patch_sp_n256_a8c1},
    {256, 12, 1, launch_patch_n256_a12c1, launch_patch_ws_n256_a12c1, launch_patch_sp_n256_a12c1},
    {256, 4, 2, launch_patch_n256_a4c2, launch_patch_ws_n256_a4c2, launch_patch_sp_n256_a4c2},
    {256, 8, 4, launch_patch_n256_a8c4, launch_patch_ws_n256_a8c4, launch_patch_sp_n256_a8c4},
};

// Largest patch (in pixels) any tile of this geometry needs.  Tile positions repeat relative to the
// image with period lcm(128, Ho*Wo), so one period plus the last tile is an exact walk; results
// are cached because the same layers are launched over and over.
int patch_npix_max(const PatchGeom& g) {
    struct Key { int v[13]; int npix; };
    static Key cache[64];
    static int used = 0, next = 0;
    static std::mutex mu;
    const int key[13] = {g.tm, g.M, g.B, g.H, g.W, g.KH, g.KW, g.sh, g.sw, g.ph, g.pw, g.Ho, g.Wo};
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < used; ++i)
        if (!memcmp(cache[i].v, key, sizeof(key))) return cache[i].npix;
    const int64_t img = (int64_t)g.Ho * g.Wo;
    int64_t a = g.tm, b = img;
    while (b) { const int64_t t = a % b; a = b; b = t; }
    const int64_t period_tiles = img / a;                       // lcm(TM, img) / TM
    const int64_t tiles = ((int64_t)g.M + g.tm - 1) / g.tm;
    int npix = 0;
    for (int64_t t = 0; t < tiles && t <= period_tiles; ++t) {
        const int n = tile_patch(g, (int)(t * g.tm)).npix;
        npix = n > npix ? n : npix;
    }
    const int n_last = tile_patch(g, (int)((tiles - 1) * g.tm)).npix;
    npix = n_last > npix ? n_last : npix;
    Key& slot = cache[used < 64 ? used++ : (next++ & 63)];
    memcpy(slot.v, key, sizeof(key));
    slot.npix = npix;
    return npix;
}

// The patch geometry of `g` for tiles of `tm` output pixels and the largest patch; false: outside what the
// index arithmetic of the input-patch kernels covers.
bool patch_geom_for(const ConvGeom& g, int tm, PatchGeom* pg, int* npix) {
    if (g.Cq % kStepK != 0) return false;                        // fewer than 33 channels: taps are not step-aligned
    if (g.M >= kPatchMaxDividend || (size_t)g.Kp * g.Np >= kPatchInvalidOffset) return false;
    if ((int64_t)g.B * g.H * g.W >= kPatchMaxDividend) return false;     // the pixel remap of strided 1x1 layers
    PatchGeom q = make_patch_geom(g.B, g.H, g.W, g.KH, g.KW, g.sh, g.sw, g.ph, g.pw, tm);
    if ((int64_t)q.B * q.Hv + q.KH >= kPatchMaxDividend) return false;
    if (patch_npix_bound(q) > 4096) return false;               // far too large: skip the exact walk
    *npix = patch_npix_max(q);
    *pg = q;
    return true;
}

// Fills `pg`, `npix`, and picks staging (chunks per lane, channel block); false: not eligible.
bool plan_patch(const ConvGeom& g, PatchGeom* pg, int* npix, int* ac, int* cbs) {
    PatchGeom q;
    int n;
    if (!patch_geom_for(g, kPatchTM, &q, &n)) return false;
    const int taps = q.KH * q.KW;
    const int ksteps = g.Cq / kStepK;
    // candidates (chunks per lane, channel block / 64): larger channel blocks first for 1x1 layers,
    // the smallest staging that holds the patch otherwise
    static const int cand[6][2] = {{8, 4}, {4, 2}, {2, 1}, {4, 1}, {8, 1}, {12, 1}};
    for (const auto& c : cand) {
        const int a = c[0], cb = c[1];
        if (ksteps % cb) continue;
        if (n * 4 * cb > a * 256) continue;                      // patch does not fit the staging registers
        if (cb > 1 && taps > 1) continue;                        // multi-tap layers: 64-channel units
        const int as = a / 2, steps = taps * cb;
        const int unrolled = as + (((as ^ steps) & 1) ? 1 : 0);  // as the kernel lays out a unit
        if (cb == 1 && !(taps & 1)) continue;                    // 64-channel units need an odd tap count
        if (steps < unrolled) continue;                          // unit too short to stage all chunks
        *pg = q; *npix = n; *ac = a; *cbs = cb;
        return true;
    }
    return false;
}

// Output-channel tile and form of the patch kernel (rules fitted to per-layer measurements of the workload tables).
//   64 for narrow layers (wave-specialised, two workgroups of 8 wavefronts per CU: the accumulators are small
//   enough for 128 registers per lane), and for layers so small that 128-wide tiles would leave half the chip idle.
//   256 (wave-specialised: 4 matrix + 4 staging wavefronts, one workgroup per CU) when it pads N to no more columns
//   than 128-wide tiles would and either fills three quarters of the chip or the layer is small anyway (then one
//   larger tile per CU beats a split reduction with its two extra launches); also for patches so large that LDS
//   holds one workgroup per CU anyway (strided 3x3 layers on large images) when the layer is wide and fills the chip.
//   128 otherwise: two plain workgroups per CU that hide each other's latencies for 1x1 layers with many tiles,
//   wave-specialised for multi-tap layers and for layers with no more tiles than CUs.
// The tuning hook forces tile width and form.
const PatchVariant* pick_patch(const ConvGeom& g, const Tuning& tune, int ac, int cbs, int npix, bool forced, bool* ws) {
    const int64_t tiles_m = (g.M + kPatchTM - 1) / kPatchTM;
    const int64_t t128 = tiles_m * ((g.N + 127) / 128), t256 = tiles_m * ((g.N + 255) / 256);
    const int cus = device_cu_count();
    int tn = g.N <= 64 ? 64 : 128;
    const bool same_columns = round_up(g.N, 256) == round_up(g.N, 128);
    if (g.N > 128 && same_columns && (t256 * 4 >= (int64_t)cus * 3 || (t128 <= cus && t256 * 8 >= cus))) tn = 256;
    if (g.N > 64 && t128 * 2 <= cus) tn = 64;      // a small layer: more, narrower tiles fill more CUs, and need no split reduction
    if (2 * 4 * cbs * patch_plane_stride(npix, 4 * cbs) > kLdsPerCu / 2) {
        if (g.N >= 256 && t256 >= cus) tn = 256;
        else if (g.N < 256 && t128 >= cus && !forced) return nullptr;   // narrow: gather kernel
    }
    *ws = tn != 128 || g.KH * g.KW > 1 || t128 <= cus;
    if ((tune.patch_tn == 64 || tune.patch_tn == 128 || tune.patch_tn == 256) && tile_fits(tune.patch_tn, g)) tn = tune.patch_tn;
    if (tune.patch_ws >= 0) *ws = tune.patch_ws != 0;
    const bool strided_1x1 = g.KH == 1 && g.KW == 1 && (g.sh > 1 || g.sw > 1);    // pixel remap: staging wavefronts only
    if (strided_1x1) *ws = true;
    for (const PatchVariant& v : kPatchVariants)
        if (v.tn == tn && v.ac == ac && v.cbs == cbs) {
            if (!v.fn_ws) *ws = false;
            if (strided_1x1 && !*ws) return nullptr;
            return &v;
        }
    return nullptr;
}

// 1x1 layers with a long reduction have nothing to reuse between taps; when they also
// fill the chip with wide tiles and waste little on channel padding, the gather kernel's wider
// tiles (each activation trimmed once for up to 512 output channels) are faster.
bool prefer_gather(const ConvGeom& g) {
    const bool gemm = g.KH == 1 && g.KW == 1 && g.ph == 0 && g.pw == 0;      // any stride
    if (!gemm || g.K < 768) return false;
    const int tn = (g.N > 256 && tile_fits(512, g)) ? 512 : g.N > 128 ? 256 : 128;
    const int64_t tiles = (g.M + 127) / 128 * ((g.N + tn - 1) / tn);
    return tiles >= device_cu_count() && round_up(g.N, tn) * 100 <= (int64_t)g.N * 115;
}

// Everything the entry points decide before launching.
struct ConvPlan {
    bool patch = false;
    const PatchVariant* variant = nullptr;
    PatchGeom pg{};
    int npix = 0, ac = 0, cbs = 0;
    bool ws = false;            // wave-specialised form of the patch kernel
    size_t pad_bytes = 0;       // channel-padded copy of x (channel counts that are not a multiple of 16)
};

ConvPlan make_plan(const ConvGeom& g, const Tuning& tune) {
    ConvPlan pl;
    if (g.fold) {               // at most 4 channels: 4-channel padded copy, pixel-folded, gather kernel
        pl.pad_bytes = (size_t)round_up((int64_t)g.B * g.H * g.W * 4, 256);
        return pl;
    }
    if (g.Cp != g.C) pl.pad_bytes = (size_t)round_up((int64_t)g.B * g.H * g.W * g.Cp, 256);
    const bool force_gather = tune.path == 1, force_patch = tune.path == 2;
    ConvGeom gk = g;
    gk.C = gk.Cp;                                                // what the kernel sees after the padding pre-pass
    if (!force_gather && (force_patch || !prefer_gather(g)) && plan_patch(gk, &pl.pg, &pl.npix, &pl.ac, &pl.cbs)) {
        pl.variant = pick_patch(g, tune, pl.ac, pl.cbs, pl.npix, force_patch, &pl.ws);
        pl.patch = pl.variant != nullptr;
    }
    return pl;
}

// 2:4 pruned weights run on the sparse matrix instruction when the layer's plan is the wave-specialised
// input-patch kernel and the trim looks at one activation at a time (with pairing on, the caller expands the
// problem and `kind` is the plain one; with it off the staging wavefronts trim as in the dense form).
bool sparse_plan(const ConvPlan& pl, TrimKind kind) {
    const bool single = kind == kTrimNone || kind == kTrimFloor || kind == kTrimRound || kind == kTrimRound4;
    return pl.patch && pl.ws && pl.variant->fn_sp && single;
}

}  // namespace

extern "C" sparq_status sparq_set_tuning(const char* spec) {
    Tuning t;
    const char* p = spec ? spec : "";
    while (*p) {
        const char* end = strchr(p, ',');
        const size_t len = end ? (size_t)(end - p) : strlen(p);
        char item[48];
        if (len == 0 || len >= sizeof(item)) return SPARQ_EINVAL;
        memcpy(item, p, len);
        item[len] = 0;
        char* eq = strchr(item, '=');
        if (!eq) return SPARQ_EINVAL;
        *eq = 0;
        const char* key = item;
        const char* val = eq + 1;
        if (!strcmp(key, "path")) {
            if (!strcmp(val, "gather")) t.path = 1;
            else if (!strcmp(val, "patch")) t.path = 2;
            else return SPARQ_EINVAL;
        } else if (!strcmp(key, "tile")) {
            if (strcmp(val, "128x128") && strcmp(val, "128x256") && strcmp(val, "128x512")) return SPARQ_EINVAL;
            strcpy(t.tile, val);
        } else if (!strcmp(key, "patch_tn")) {
            t.patch_tn = atoi(val);
            if (t.patch_tn != 64 && t.patch_tn != 128 && t.patch_tn != 256) return SPARQ_EINVAL;
        } else if (!strcmp(key, "patch_ws")) {
            if (strcmp(val, "0") && strcmp(val, "1")) return SPARQ_EINVAL;
            t.patch_ws = val[0] - '0';
        } else {
            return SPARQ_EINVAL;
        }
        p += len + (end ? 1 : 0);
    }
    std::lock_guard<std::mutex> lock(g_tuning_mu);
    g_tuning = t;
    return SPARQ_OK;
}

extern "C" size_t sparq_workspace_bytes(const sparq_conv_desc* desc, const sparq_mode* mode) {
    ConvGeom g;
    if (!conv_geom(desc, &g) || !mode_valid(mode)) return 0;
    return make_plan(g, current_tuning()).pad_bytes;
}

extern "C" sparq_status sparq_conv_plan(const sparq_conv_desc* desc, const sparq_mode* mode, char* text, size_t text_bytes) {
    ConvGeom g;
    if (!text || text_bytes == 0 || !conv_geom(desc, &g) || !mode_valid(mode)) return SPARQ_EINVAL;
    const Tuning tune = current_tuning();
    const ConvPlan pl = make_plan(g, tune);
    if (pl.patch) {
        snprintf(text, text_bytes, "conv_patch_kernel tile=128x%d chunks=%d unit_channels=%d patch_pixels=%d%s%s",
                 pl.variant->tn, pl.ac, 64 * pl.cbs, pl.npix, pl.ws ? " wave_specialised" : "",
                 pl.pad_bytes ? " padded_copy" : "");
    } else {
        const char* name = "?";
        ConvGeom gt = g.fold ? folded_view(g) : g;
        gt.Np = g.Np;
        const TileLauncher fn = pick_tile(gt, tune);
        for (const TileEntry& t : kTiles)
            if (t.fn == fn) name = t.name;
        snprintf(text, text_bytes, "conv_gemm_kernel tile=%s%s%s", name, pl.pad_bytes ? " padded_copy" : "",
                 g.fold ? " pixel_folded" : "");
    }
    return SPARQ_OK;
}

namespace {

// The gather kernel splits an output row number into (image, oy, ox) once per lane and tile with two divisions by
// numbers fixed per launch.
void set_row_division(GemmParams& p) {
    p.div_wo = make_fastdiv((uint32_t)p.Wo);
    p.div_ho = make_fastdiv((uint32_t)p.Ho);
    p.rows_fit_31 = p.M < (1ll << 31) ? 1 : 0;
}

// Both convolution entry points: acc / out (with scale) as in sparq_conv_gemm, or y (with scale holding the
// requantisation factors) as in sparq_conv_gemm_u8.
// sp: the weights as operands of the sparse matrix instruction as well (2:4 pruned layers); used when the plan is
// the wave-specialised input-patch kernel, ignored otherwise.
struct SparseOperand { const uint8_t* vals; const uint32_t* pos; };
sparq_status conv_launch(const uint8_t* x, const void* packed_w, const sparq_conv_desc* desc, const sparq_mode* mode,
                         int32_t* acc, const float* scale, float* out, uint8_t* y, const sparq_mode* out_mode,
                         void* workspace, size_t workspace_bytes, void* stream, const SparseOperand* sp = nullptr) {
    ConvGeom g;
    if (!x || !packed_w || !conv_geom(desc, &g) || !mode_valid(mode)) return SPARQ_EINVAL;
    if (!acc && !out && !y) return SPARQ_EINVAL;
    if ((out || y) && !scale) return SPARQ_EINVAL;
    // y trimmed for the next layer: in the epilogue when that layer's mode is this layer's own and the kernel
    // packs the bytes (N a multiple of 4, no split reduction, not a plain 8-bit layer); otherwise one in-place
    // pass of the standalone trim over y afterwards.  Either way y = trim(requantised result), pairs (2j, 2j+1) of a row.
    const bool trim_y = y && out_mode && out_mode->window_bits != 8;
    if (trim_y && !mode_valid(out_mode)) return SPARQ_EINVAL;
    const bool same_mode = trim_y && out_mode->window_bits == mode->window_bits && out_mode->shift_mask == mode->shift_mask &&
                           out_mode->round_nearest == mode->round_nearest && out_mode->pair == mode->pair;
    bool fused_trim = same_mode && g.N % 4 == 0;
    if (!aligned(x, 16) || !aligned(packed_w, 256) || (acc && !aligned(acc, 16)) || (out && !aligned(out, 16)) ||
        (y && !aligned(y, 16)) || (scale && !aligned(scale, 4)))
        return SPARQ_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Tuning tune = current_tuning();
    const ConvPlan pl = make_plan(g, tune);
    const size_t need = pl.pad_bytes;
    if (need) {
        if (!workspace || !aligned(workspace, 256)) return SPARQ_EINVAL;
        if (workspace_bytes < need) return SPARQ_EWORKSPACE;
    }

    const uint8_t* xin = x;
    TrimKind kind = trim_kind(mode);
    size_t x_bytes = g.x_bytes;
    if (g.fold) {
        // A first-layer shape (C <= 4): trim into a copy with 4 channels per pixel, then contract the
        // pixel-folded problem (16-channel super-pixels, fold_p * N output channels) with trimming off.
        const ConvGeom f = folded_view(g);
        if (f.x_bytes >= kInvalidOffset) return SPARQ_EUNSUPPORTED;
        const sparq_status st = launch_trim_pad(x, static_cast<uint8_t*>(workspace), (int64_t)g.B * g.H * g.W, g.C, 4, mode, s);
        if (st != SPARQ_OK) return st;
        GemmParams p{};
        p.x = static_cast<const uint8_t*>(workspace);
        p.wpk = static_cast<const uint8_t*>(packed_w) + g.w_off;
        p.colsum = static_cast<const int32_t*>(packed_w);
        p.acc = acc; p.scale = scale; p.out = out; p.out_u8 = y;
        p.M = f.M;
        p.x_bytes = (uint32_t)f.x_bytes;
        p.N = f.N; p.Np = g.Np; p.Kk = f.Kk; p.nkb = g.Kp / kStepK; p.scale_n = g.N;
        p.H = f.H; p.W = f.W; p.C = 16; p.Cq = 16; p.Ho = f.Ho; p.Wo = f.Wo; p.KH = f.KH; p.KW = f.KW;
        p.sh = f.sh; p.sw = 1; p.ph = f.ph; p.pw = f.pw;
        p.rcp_c = 1.0f / 16.0f;
        p.rcp_kw = 1.0f / (float)f.KW;
        set_row_division(p);
        p.luts = make_luts(8, 1);
        ConvGeom ft = f;
        ft.Np = g.Np;
        const sparq_status stf = pick_tile(ft, tune, y != nullptr)(kTrimNone, p, s);
        if (stf != SPARQ_OK || !trim_y) return stf;
        return sparq_trim(y, y, g.M, g.N, out_mode, stream);
    }
    if (g.Cp != g.C) {
        // Channel counts that are not a multiple of 16: trim into a channel-padded copy
        // first (pairs stay inside the row; padded channels are zeros with zero weights),
        // then contract the copy without further trimming.
        x_bytes = (size_t)g.B * g.H * g.W * g.Cp;
        if (x_bytes >= kInvalidOffset) return SPARQ_EUNSUPPORTED;
        const sparq_status st = launch_trim_pad(x, static_cast<uint8_t*>(workspace), (int64_t)g.B * g.H * g.W, g.C,
                                                g.Cp, mode, s);
        if (st != SPARQ_OK) return st;
        xin = static_cast<const uint8_t*>(workspace);
        kind = kTrimNone;
        fused_trim = false;                     // the kernel runs with trimming off
    }
    if (x_bytes >= kInvalidOffset) return SPARQ_EUNSUPPORTED;
    const auto finish = [&](sparq_status st, bool fused) {
        if (st != SPARQ_OK || !trim_y || fused) return st;
        return sparq_trim(y, y, g.M, g.N, out_mode, stream);
    };

    // Preferred: the input-patch kernel (activations loaded and trimmed once per tile and channel block).
    if (pl.patch) {
        PatchParams q{};
        q.x = xin;
        q.wpk = static_cast<const uint8_t*>(packed_w) + g.w_off;
        q.colsum = static_cast<const int32_t*>(packed_w);
        q.acc = acc; q.scale = scale; q.out = out; q.out_u8 = y; q.trim_out = fused_trim ? 1 : 0;
        q.x_bytes = (uint32_t)x_bytes;
        q.w_bytes = (uint32_t)((size_t)g.Kp * g.Np);
        q.N = g.N; q.Np = g.Np; q.C = g.Cp;
        q.ksteps_tap = g.Cq / kStepK;
        q.ncb = q.ksteps_tap / pl.cbs;
        q.nsteps = g.KH * g.KW * pl.cbs;
        q.g = pl.pg;
        q.luts = make_luts(mode->window_bits, mode->shift_mask);
        q.trim_in = 1;
        TrimKind pkind = kind;
        bool pfused = fused_trim;
        // An input that arrives trimmed (mode: plain 8 bits) with an output to be trimmed for the next layer:
        // the wave-specialised kernel of the OUTPUT mode, told not to trim its input, trims y in its epilogue.
        // (A layer that would take the plain form takes the wave-specialised one here: that costs a few per cent,
        // the separate trim pass over y it avoids costs more.)
        bool use_ws = pl.ws;
        if (trim_y && !fused_trim && kind == kTrimNone && mode->window_bits == 8 && g.N % 4 == 0 &&
            g.Cp == g.C && pl.variant->fn_ws) {
            use_ws = true;
            pkind = trim_kind(out_mode);
            q.luts = make_luts(out_mode->window_bits, out_mode->shift_mask);
            q.trim_in = 0;
            pfused = true;
        }
        q.trim_out = pfused ? 1 : 0;
        if (sp && sparse_plan(pl, kind) && !y) {
            PatchParams qs = q;
            qs.wpk = sp->vals;
            qs.widx = sp->pos;
            qs.w_bytes = (uint32_t)((size_t)g.Kp * g.Np / 2);
            const sparq_status st = pl.variant->fn_sp(kind, qs, pl.npix, s);
            if (st != SPARQ_EUNSUPPORTED) return st;
        }
        {
            const PatchLauncher fn = use_ws ? pl.variant->fn_ws : pl.variant->fn;
            const sparq_status st = fn(pkind, q, pl.npix, s);
            if (st != SPARQ_EUNSUPPORTED) return finish(st, pfused);
        }
    }

    GemmParams p{};
    p.x = xin;
    p.wpk = static_cast<const uint8_t*>(packed_w) + g.w_off;
    p.colsum = static_cast<const int32_t*>(packed_w);
    p.acc = acc;
    p.scale = scale;
    p.out = out;
    p.out_u8 = y;
    p.trim_out = fused_trim ? 1 : 0;
    p.M = g.M;
    p.x_bytes = (uint32_t)x_bytes;
    p.N = g.N; p.Np = g.Np; p.Kk = g.Kk; p.nkb = g.Kp / kStepK; p.scale_n = g.N;
    p.H = g.H; p.W = g.W; p.C = g.Cp; p.Cq = g.Cq; p.Ho = g.Ho; p.Wo = g.Wo; p.KH = g.KH; p.KW = g.KW;
    p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw;
    p.rcp_c = 1.0f / (float)g.Cq;
    p.rcp_kw = 1.0f / (float)g.KW;
    set_row_division(p);
    p.luts = make_luts(mode->window_bits, mode->shift_mask);

    return finish(pick_tile(g, tune, y != nullptr)(kind, p, s), fused_trim);
}

}  // namespace

extern "C" sparq_status sparq_conv_gemm(const uint8_t* x, const void* packed_w, const sparq_conv_desc* desc,
                                        const sparq_mode* mode, int32_t* acc, const float* scale, float* out,
                                        void* workspace, size_t workspace_bytes, void* stream) {
    if (!acc && !out) return SPARQ_EINVAL;
    return conv_launch(x, packed_w, desc, mode, acc, scale, out, nullptr, nullptr, workspace, workspace_bytes, stream);
}

// ---- the same convolution for callers that cannot allocate: the scratch lives in the library's own image ----
// One array per device (every GPU the library's code object is loaded on holds its own copy at its own
// address, until the process ends).  In host code the array's name is only a handle for the symbol lookup:
// the device address comes from hipGetSymbolAddress, once per device, and is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[SPARQ_STATIC_WORKSPACE_BYTES];

namespace {
sparq_status static_scratch_address(void** ptr) {
    static void* addr[kMaxDevices] = {};
    static std::mutex mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return SPARQ_ELAUNCH;
    std::lock_guard<std::mutex> lock(mu);
    if (dev < kMaxDevices && addr[dev]) {
        *ptr = addr[dev];
        return SPARQ_OK;
    }
    void* a = nullptr;
    if (hipGetSymbolAddress(&a, HIP_SYMBOL(scratch)) != hipSuccess || !a) {
        (void)hipGetLastError();
        return SPARQ_ELAUNCH;
    }
    if (dev < kMaxDevices) addr[dev] = a;       // ordinals past the table look the address up on every call
    *ptr = a;
    return SPARQ_OK;
}
}  // namespace

extern "C" sparq_status sparq_conv_gemm_static_ws(const uint8_t* x, const void* packed_w, const sparq_conv_desc* desc,
                                                  const sparq_mode* mode, int32_t* acc, const float* scale, float* out,
                                                  void* stream) {
    if (!acc && !out) return SPARQ_EINVAL;
    ConvGeom g;
    if (!conv_geom(desc, &g) || !mode_valid(mode)) return SPARQ_EINVAL;
    const size_t need = make_plan(g, current_tuning()).pad_bytes;
    if (need > (size_t)SPARQ_STATIC_WORKSPACE_BYTES) return SPARQ_EWORKSPACE;
    void* ws = nullptr;
    if (need) {
        const sparq_status st = static_scratch_address(&ws);
        if (st != SPARQ_OK) return st;
    }
    // Every byte of the scratch a call reads it has written itself first (the padded copy is written whole by the
    // trim pass), so the last call's contents never show.
    return conv_launch(x, packed_w, desc, mode, acc, scale, out, nullptr, nullptr, ws, need, stream);
}

// ---- input in packed storage (Sections 3.1, 5.1, 6): records expanded into the workspace, contracted at 8 bits ----
namespace {
const sparq_mode kPlainMode = {8, 1, 0, 0};
}

extern "C" size_t sparq_conv_packed_workspace_bytes(const sparq_conv_desc* desc, const sparq_mode* mode) {
    ConvGeom g;
    if (!conv_geom(desc, &g) || !mode_valid(mode)) return 0;
    return (size_t)round_up((int64_t)g.x_bytes, 256) + sparq_workspace_bytes(desc, &kPlainMode);
}

extern "C" sparq_status sparq_conv_gemm_packed(const void* packed_x, size_t packed_x_bytes, int32_t group,
                                               const void* packed_w, const sparq_conv_desc* desc, const sparq_mode* mode,
                                               int32_t* acc, const float* scale, float* out, void* workspace,
                                               size_t workspace_bytes, void* stream) {
    ConvGeom g;
    if (!packed_x || !conv_geom(desc, &g) || !mode_valid(mode) || (!acc && !out)) return SPARQ_EINVAL;
    const int64_t pixels = (int64_t)g.B * g.H * g.W;
    const size_t need_packed = sparq_packed_act_bytes(pixels, g.C, mode, group);
    if (need_packed == 0 || !aligned(packed_x, 4)) return SPARQ_EINVAL;
    if (packed_x_bytes < need_packed) return SPARQ_EWORKSPACE;
    if (!workspace || !aligned(workspace, 256)) return SPARQ_EINVAL;
    if (workspace_bytes < sparq_conv_packed_workspace_bytes(desc, mode)) return SPARQ_EWORKSPACE;
    uint8_t* xu = static_cast<uint8_t*>(workspace);
    const size_t x_room = (size_t)round_up((int64_t)g.x_bytes, 256);
    const sparq_status st = launch_unpack_act(packed_x, xu, pixels, g.C, mode, group, static_cast<hipStream_t>(stream));
    if (st != SPARQ_OK) return st;
    return conv_launch(xu, packed_w, desc, &kPlainMode, acc, scale, out, nullptr, nullptr, xu + x_room,
                       workspace_bytes - x_room, stream);
}

// ---- 2:4 pruned weights (Section 4, sparse tensor core; Section 5.3): see sparq_sparse24.hip ----
namespace {
// The dense problem that is actually contracted: with vSPARQ on, 16 expanded channels per group of four.
bool sparse24_geometry(const sparq_conv_desc* desc, const sparq_mode* mode, sparq_conv_desc* eff, bool* expand) {
    ConvGeom g;
    if (!desc || desc->C % 4 != 0 || !conv_geom(desc, &g) || !mode_valid(mode)) return false;
    *expand = mode->pair && mode->window_bits != 8;
    *eff = *desc;
    if (*expand) {
        if ((int64_t)desc->C * 4 > 0x7FFFFFFF) return false;
        eff->C = desc->C * 4;
    }
    return conv_geom(eff, &g);
}
const sparq_mode kNoPairPlain = {8, 1, 0, 0};

// Layout of the buffer sparq_pack_weights_sparse24 fills: the dense packed tiles of the contracted problem, room
// to decompress into, then the same weights as operands of the sparse matrix instruction (kept bytes, positions)
// when the contracted problem's taps are 64-byte aligned (otherwise those two parts are empty).
struct Sparse24Layout { size_t tiles, dense, vals, pos; bool sparse; };
Sparse24Layout sparse24_layout(const sparq_conv_desc& eff) {
    ConvGeom g;
    conv_geom(&eff, &g);
    Sparse24Layout L;
    L.tiles = (size_t)round_up((int64_t)g.packed_bytes, 256);
    L.dense = (size_t)round_up((int64_t)eff.N * eff.KH * eff.KW * eff.C, 256);
    L.sparse = !g.fold && g.Cq % kStepK == 0;
    L.vals = L.sparse ? (size_t)round_up((int64_t)g.Kp * g.Np / 2, 256) : 0;
    L.pos = L.sparse ? (size_t)round_up((int64_t)g.Kp * g.Np / 8, 256) : 0;
    return L;
}
}  // namespace

extern "C" size_t sparq_sparse24_packed_bytes(const sparq_conv_desc* desc, const sparq_mode* mode) {
    sparq_conv_desc eff;
    bool expand;
    if (!sparse24_geometry(desc, mode, &eff, &expand)) return 0;
    const Sparse24Layout L = sparse24_layout(eff);
    return L.tiles + L.dense + L.vals + L.pos;
}

extern "C" sparq_status sparq_pack_weights_sparse24(const int8_t* w_vals, const uint8_t* w_idx, const sparq_conv_desc* desc,
                                                    const sparq_mode* mode, void* packed, size_t packed_bytes, void* stream) {
    sparq_conv_desc eff;
    bool expand;
    if (!w_vals || !w_idx || !packed || !sparse24_geometry(desc, mode, &eff, &expand) || !aligned(packed, 256)) return SPARQ_EINVAL;
    if (packed_bytes < sparq_sparse24_packed_bytes(desc, mode)) return SPARQ_EWORKSPACE;
    const Sparse24Layout L = sparse24_layout(eff);
    int8_t* dense = static_cast<int8_t*>(packed) + L.tiles;
    const int64_t groups = (int64_t)desc->N * desc->KH * desc->KW * (desc->C / 4);
    sparq_status st = launch_sparse24_expand_weights(w_vals, w_idx, dense, groups, expand, static_cast<hipStream_t>(stream));
    if (st != SPARQ_OK) return st;
    st = sparq_pack_weights(dense, &eff, packed, L.tiles, stream);
    if (st != SPARQ_OK || !L.sparse) return st;
    ConvGeom g;
    conv_geom(&eff, &g);
    uint8_t* vals = static_cast<uint8_t*>(packed) + L.tiles + L.dense;
    return launch_sparse24_pack_operand(dense, vals, reinterpret_cast<uint32_t*>(vals + L.vals), eff.N, g.Np, eff.KH * eff.KW,
                                        eff.C, g.Cq, static_cast<hipStream_t>(stream));
}

extern "C" size_t sparq_sparse24_workspace_bytes(const sparq_conv_desc* desc, const sparq_mode* mode) {
    sparq_conv_desc eff;
    bool expand;
    if (!sparse24_geometry(desc, mode, &eff, &expand)) return 0;
    if (!expand) return sparq_workspace_bytes(desc, mode);
    return (size_t)round_up((int64_t)eff.B * eff.H * eff.W * eff.C, 256) + sparq_workspace_bytes(&eff, &kNoPairPlain);
}

extern "C" sparq_status sparq_conv_gemm_sparse24(const uint8_t* x, const void* packed, const sparq_conv_desc* desc,
                                                 const sparq_mode* mode, int32_t* acc, const float* scale, float* out,
                                                 void* workspace, size_t workspace_bytes, void* stream) {
    sparq_conv_desc eff;
    bool expand;
    if (!x || !packed || (!acc && !out) || !sparse24_geometry(desc, mode, &eff, &expand)) return SPARQ_EINVAL;
    const Sparse24Layout L = sparse24_layout(eff);
    const uint8_t* sp_vals = static_cast<const uint8_t*>(packed) + L.tiles + L.dense;
    const SparseOperand sp_op = {sp_vals, reinterpret_cast<const uint32_t*>(sp_vals + L.vals)};
    const SparseOperand* sp = L.sparse ? &sp_op : nullptr;
    if (!expand)      // nothing depends on the partner: the decompressed weights, the ordinary path
        return conv_launch(x, packed, desc, mode, acc, scale, out, nullptr, nullptr, workspace, workspace_bytes, stream, sp);
    if (!aligned(x, 4) || !workspace || !aligned(workspace, 256)) return SPARQ_EINVAL;
    if (workspace_bytes < sparq_sparse24_workspace_bytes(desc, mode)) return SPARQ_EWORKSPACE;
    const int64_t pixels = (int64_t)desc->B * desc->H * desc->W;
    const size_t x_room = (size_t)round_up(pixels * eff.C, 256);
    uint8_t* xe = static_cast<uint8_t*>(workspace);
    const sparq_status st = launch_sparse24_expand_act(x, xe, pixels, desc->C, mode, static_cast<hipStream_t>(stream));
    if (st != SPARQ_OK) return st;
    return conv_launch(xe, packed, &eff, &kNoPairPlain, acc, scale, out, nullptr, nullptr, xe + x_room,
                       workspace_bytes - x_room, stream, sp);
}

extern "C" sparq_status sparq_sparse24_plan(const sparq_conv_desc* desc, const sparq_mode* mode, char* text, size_t text_bytes) {
    sparq_conv_desc eff;
    bool expand;
    if (!text || text_bytes == 0 || !sparse24_geometry(desc, mode, &eff, &expand)) return SPARQ_EINVAL;
    const sparq_mode* m = expand ? &kNoPairPlain : mode;
    char line[200];
    const sparq_status st = sparq_conv_plan(&eff, m, line, sizeof(line));
    if (st != SPARQ_OK) return st;
    ConvGeom g;
    conv_geom(&eff, &g);
    const ConvPlan pl = make_plan(g, current_tuning());
    const TrimKind kind = (g.fold || g.Cp != g.C) ? kTrimNone : trim_kind(m);     // a padded copy is trimmed by its pre-pass
    const bool smfmac = sparse24_layout(eff).sparse && sparse_plan(pl, kind);
    snprintf(text, text_bytes, "%s%s%s", line, expand ? " expanded_x4" : "", smfmac ? " sparse_mfma" : " dense_mfma");
    return SPARQ_OK;
}

extern "C" sparq_status sparq_conv_gemm_u8(const uint8_t* x, const void* packed_w, const sparq_conv_desc* desc,
                                           const sparq_mode* mode, const float* factor, uint8_t* y,
                                           const sparq_mode* out_mode, void* workspace, size_t workspace_bytes,
                                           void* stream) {
    if (!factor || !y) return SPARQ_EINVAL;
    return conv_launch(x, packed_w, desc, mode, nullptr, factor, nullptr, y, out_mode, workspace, workspace_bytes, stream);
}
