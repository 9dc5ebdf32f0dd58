// Fused SPARQ convolution for gfx950, input-patch form.
//
//   acc[m][n] = sum_{kh,kw,c} T(x)[b, oy*sh-ph+kh, ox*sw-pw+kw, c] * w[n][kh][kw][c]     (Eq. 1, trimmed activations)
//
// A workgroup owns tiles of 128 consecutive output pixels x TN output channels.  For one tile and
// one block of CB input channels (a "unit") it stages the rectangle of input pixels the tile's
// filter taps touch (sparq_patch_geom.h) in LDS: loaded with 128-bit reads, trimmed in registers
// (vSPARQ pairs are bytes (2j, 2j+1) of a word, bSPARQ window per byte; sparq_swar.h), flipped to
// signed (x - 128).  Every tap then reads its matrix-instruction operands from that patch at a
// shifted position, so an activation is fetched and trimmed once per unit -- not once per tap as
// an im2col gather would -- and there is one workgroup barrier per unit instead of one per
// 64-byte reduction step.  Weights come pre-packed in fragment order straight from L2 into
// registers, two steps ahead.  The epilogue adds 128 * sum_k w[n][k] (exact in int32) and applies
// the per-channel scale (Section 5).
//
// Units of all tiles a workgroup owns form one continuous software pipeline: while unit u is
// multiplied, the patch of unit u+1 is trimmed and written to the other LDS buffer and the loads
// of unit u+2 are issued; the weight stream runs ahead across unit and tile boundaries as well.
// This keeps short-reduction layers (1x1 convolutions, few channels) from draining the pipeline
// at every tile.
//
// The paper puts its trimming unit in front of the multiplier array and notes that it is shared
// and runs at a much lower rate than the multipliers (Section 5); staging the trimmed patch once
// and reusing it for all taps and all output channels of the tile is that arrangement.
#pragma once
#include <atomic>
#include <type_traits>

#include "sparq_common.h"
#include "sparq_patch_geom.h"

namespace sparq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

struct PatchParams {
    const uint8_t* x;        // activations, NHWC, C a multiple of 16
    const uint8_t* wpk;      // packed weight tiles (taps padded to 64 channels); sparse form: the kept weights
    const int32_t* colsum;   // sum_k w[n][k], Np entries
    int32_t* acc;            // [M][N] or null
    const float* scale;      // [N] or null
    float* out;              // [M][N] or null
    uint8_t* out_u8;         // [M][N] requantised output or null (then it is the only output; scale holds its factors)
    int trim_out;            // out_u8 with N % 4 == 0 only: trim the requantised bytes with this launch's own mode as well
    int trim_in;             // 0: x is taken as it is (wave-specialised form only; elsewhere the instantiation decides)
    uint32_t x_bytes, w_bytes;
    int N, Np, C;
    int ncb;                 // channel blocks (units) per work item
    int ksteps_tap;          // 64-byte steps per filter tap in the packed weights
    int nsteps;              // steps per unit = KH * KW * CBS
    int plane_stride;        // bytes between the 16-channel planes of a patch buffer
    int tiles_m, tiles_n;
    PatchGeom g;
    TrimLuts luts;
    const uint32_t* widx;    // sparse form only: positions of the kept weights, one word per 32 reduction indices
                             // (last, so that the other forms' argument offsets, and with them their code, stay as they were)
};

constexpr int kLdsPerCu = 160 * 1024;
constexpr int kSparseRowPitch = 272;               // LDS row of 64 fp32 results, padded so that the lanes' 16-byte writes spread over the banks
constexpr int kSparseEpilogueLds = 4 * 32 * kSparseRowPitch;
constexpr uint32_t kPatchInvalidOffset = 0x80000000u;   // beyond any buffer this kernel accepts (< 2 GiB)

// TN output channels per workgroup, WGM x WGN wavefronts, AC 16-byte patch chunks per lane and
// unit, CBS * 64 input channels per unit, WPC resident workgroups per CU the register budget allows.
// WS: wave-specialised variant -- wavefronts 4..7 load, trim and stage the patches, wavefronts 0..3 only read
// fragments and weights and multiply.  A wavefront's loads return in order, so in the plain variant a weight wait
// also waits for every older (slow, HBM) activation load; with separate wavefronts it does not, and the trim
// arithmetic issues from other wavefronts while the matrix instructions run.
// SP: 2:4 pruned weights on the sparse matrix instruction (v_smfmac_i32_32x32x64_i8: the weights are its sparse
// operand, two kept values of every four reduction indices plus their positions; the activations its dense
// one), so a 64-byte step is one instruction per fragment pair instead of two and a lane ends up with 16 output
// channels of one output pixel.  Wave-specialised form only, int32 / fp32 outputs only.
template <int TN, int WGM, int WGN, int AC, int CBS, int WPC, bool WS = false, bool SP = false>
struct PatchCfg {
    static constexpr bool kWaveSpecialised = WS;            // four more wavefronts do the loading, trimming and staging
    static constexpr bool kSparse = SP;
    static constexpr int kTM = kPatchTM, kTN = TN, kWGM = WGM, kWGN = WGN, kAC = AC, kCBS = CBS, kWgPerCu = WPC;
    static constexpr int kMathThreads = 64 * WGM * WGN;
    static constexpr int kStageThreads = 256;
    static constexpr int kThreads = kMathThreads + (WS ? kStageThreads : 0);
    static constexpr int kWTM = kTM / WGM, kWTN = TN / WGN;
    static constexpr int kFM = kWTM / 32, kFN = kWTN / 32;
    static constexpr int kPlanes = 4 * CBS;                  // 16-channel planes per patch buffer
    static constexpr int kCB = 64 * CBS;
    static constexpr int kAS = WS ? 0 : (AC + 1) / 2;        // steps of a unit that also stage and load patch chunks
    static constexpr int kMaxPix = AC * kStageThreads / kPlanes;   // patch pixels one unit can stage
    // 64-channel units cover multi-tap filters with an odd number of taps (1x1 included); wider
    // units are for 1x1 filters only, where steps per unit = CBS is even
    static constexpr bool kOddSteps = CBS == 1;
    static constexpr int kUnrolled = kAS + (((kAS & 1) != (kOddSteps ? 1 : 0)) ? 1 : 0);
    static_assert(kMathThreads == 256, "four matrix wavefronts");
    static_assert(kTM % (32 * WGM) == 0 && TN % (32 * WGN) == 0, "tile must split into 32x32 fragments");
    static_assert(CBS == 1 || CBS == 2 || CBS == 4, "channel block");
    static_assert(AC >= 2 && AC % 2 == 0, "chunks per lane");
    static_assert(!SP || (WS && kFN % 2 == 0), "sparse form: wave-specialised, an even number of channel fragments");
};

// bytes between planes: a multiple of 256 plus 256 / planes, so that the lanes that write one
// pixel's chunks (one plane each) and their neighbours (next pixel) hit different LDS banks
inline int patch_plane_stride(int npix_max, int planes) {
    return (int)round_up((int64_t)npix_max * kChunk, 256) + 256 / planes;
}

template <int V> using int_c = std::integral_constant<int, V>;

template <class Cfg, int KIND>
__global__ __launch_bounds__(Cfg::kThreads, Cfg::kWgPerCu * Cfg::kThreads / 256) void conv_patch_kernel(const PatchParams p) {
    constexpr bool WS = Cfg::kWaveSpecialised, SP = Cfg::kSparse;
    constexpr int NT = Cfg::kStageThreads, FM = Cfg::kFM, FN = Cfg::kFN, AC = Cfg::kAC, CBS = Cfg::kCBS, AS = Cfg::kAS;
    constexpr int PL = Cfg::kPlanes, TN = Cfg::kTN;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];     // [2][PL][plane_stride]

    const int lane = threadIdx.x & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const bool producer = WS && wave_all >= 4;            // uniform per wavefront
    const int wave = wave_all & 3;
    const int tid = wave * 64 + lane;                     // index inside the role's 256 lanes
    const int wm = wave % Cfg::kWGM, wn = wave / Cfg::kWGM;
    const int l32 = lane & 31, lhi = lane >> 5;
    const PatchGeom& g = p.g;
    const int ntiles = p.tiles_m * p.tiles_n;
    const int grid = (int)gridDim.x;
    const int buf_bytes = PL * p.plane_stride;
    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(p.x), 0, (int)p.x_bytes, 0x00020000);

    // ---- patch staging: chunk i of this lane is element e = tid + i * 256 of a unit, i.e. plane
    //      e % PL (the same for every i) of patch pixel tid / PL + i * (256 / PL) ----
    const int my_plane = tid % PL;
    const int my_c = my_plane * kChunk;           // channel offset inside the unit's channel block
    const int my_pix = tid / PL;
    const int my_loff = my_plane * p.plane_stride + my_pix * kChunk;
    const int dummy_off = 2 * buf_bytes;          // 16 spare bytes: where chunks outside the patch are written
    v4u a_reg[AC];                                // requested chunks (of the unit after next)

    // load cursor: the unit whose chunks are requested next; its tile's patch, uniform
    int l_tile = (int)blockIdx.x, l_cb = 0;
    TilePatch lt;
    int stage_npix = 0;                           // patch size of the unit whose chunks are staged next
    auto load_tile_patch = [&]() __attribute__((always_inline)) {
        const bool live = l_tile < ntiles;
        const int tm = live ? l_tile / p.tiles_n : 0;
        const TilePatch t = tile_patch(g, tm * kPatchTM);
        lt.v0 = __builtin_amdgcn_readfirstlane(t.v0);
        lt.xlo = __builtin_amdgcn_readfirstlane(t.xlo);
        lt.pwt = __builtin_amdgcn_readfirstlane(t.pwt);
        lt.npix = live ? __builtin_amdgcn_readfirstlane(t.npix) : 0;
        lt.rcp_pwt = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, t.rcp_pwt)));
    };
    auto advance_load_cursor = [&]() __attribute__((always_inline)) {
        if (++l_cb == p.ncb) {
            l_cb = 0;
            l_tile += grid;
            load_tile_patch();
        }
    };
    uint32_t pix_off[AC];                         // staging wavefronts: byte offset of the pixel of chunk i, kept per tile
    auto load_chunk = [&](int i) __attribute__((always_inline)) {
        const int pix = my_pix + i * (NT / PL);
        const int ch = l_cb * Cfg::kCB + my_c;
        uint32_t off;
        if constexpr (WS) {
            // The staging wavefronts' own loop can afford uniform branches around address arithmetic: a pixel's offset
            // is computed for the first channel block of a tile and reused for the others, and not at all for a chunk
            // that lies past the patch altogether.  The request itself stays unconditional (it then reads 0 without
            // touching memory), so that the counts of outstanding requests stay exact.
            // (only these wavefronts handle the pixel remap of strided 1x1 layers)
            if (l_cb == 0)
                pix_off[i] = (i * (NT / PL) < lt.npix) ? patch_pixel_offset_u32<WS>(g, lt, pix, p.C, kPatchInvalidOffset)
                                                       : kPatchInvalidOffset;
            off = pix_off[i];
        } else {
            off = patch_pixel_offset_u32<WS>(g, lt, pix, p.C, kPatchInvalidOffset);
        }
        off = (ch < p.C) ? off : kPatchInvalidOffset;            // a tap's channel padding reads as zero
        off += (off != kPatchInvalidOffset) ? (uint32_t)ch : 0u;
        a_reg[i] = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, (int)off, 0, 0);   // out of range reads 0
    };
    // trim + flip to signed + write into the patch buffer at `buf`
    auto stage_chunk = [&](int i, uint8_t* buf) __attribute__((always_inline)) {
        v4u v = a_reg[i];
        // The staging wavefronts' own loop can afford a (uniform) branch: a layer whose input was trimmed by its
        // producer skips the trim here while the epilogue still trims the output with the same tables.
        if (WS && KIND != kTrimNone && !p.trim_in) {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] ^= 0x80808080u;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = trim4_kind<KIND>(v[j], p.luts) ^ 0x80808080u;
        }
        const int pix = my_pix + i * (NT / PL);
        uint8_t* dst = (pix < stage_npix) ? buf + my_loff + i * (NT / PL) * kChunk : lds + dummy_off;
        *reinterpret_cast<v4u*>(dst) = v;
    };

    // ---- compute cursor ----
    int c_tile = (int)blockIdx.x, c_cb = 0, c_tm = 0, c_tn = 0;
    int c_pwt16 = 0;                              // bytes per patch row inside a plane
    int32_t fbase[FM];                            // patch byte offset of this lane's pixel (tap 0,0) per fragment
    // Per-channel constants of the tile's epilogue (128 * sum_k w[n][k] and the dequantisation / requantisation
    // factor), requested when the tile starts: at its end they have long arrived, where a request placed there
    // exposed a memory latency per tile -- a fifth of the time of layers with one reduction step per tile.
    int32_t corr[FN];
    float sc[FN];
    const float* scale_or_dummy = (p.out || p.out_u8) ? p.scale : reinterpret_cast<const float*>(p.colsum);
    auto setup_compute_tile = [&]() __attribute__((always_inline)) {
        c_tm = c_tile / p.tiles_n;
        c_tn = c_tile - c_tm * p.tiles_n;
#pragma unroll
        for (int j = 0; j < (SP ? 0 : FN); ++j) {
            const int n = c_tn * TN + wn * Cfg::kWTN + j * 32 + l32;
            const int nc = n < p.N ? n : 0;
            // both constants are loaded on every path (a load under a condition makes the compiler put a full
            // memory wait in front of every store of the epilogue)
            corr[j] = p.colsum[nc] * 128;
            sc[j] = scale_or_dummy[nc];
        }
        const TilePatch t = tile_patch(g, c_tm * kPatchTM);
        c_pwt16 = t.pwt * kChunk;
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            int m = c_tm * kPatchTM + wm * Cfg::kWTM + i * 32 + l32;
            m = m < g.M ? m : g.M - 1;
            fbase[i] = patch_pixel_of_output(g, t, m) * kChunk + lhi * p.plane_stride;
        }
    };

    // fragment cursor: which (kh, kw, 64-channel sub-block) the next fragment read is for
    int f_j = 0, f_kw = 0, f_kh = 0, f_off = 0;
    auto advance_frag_cursor = [&]() __attribute__((always_inline)) {
        const int sub = 4 * p.plane_stride;
        ++f_j;
        f_off += sub;
        const bool wj = f_j == CBS;
        f_j = wj ? 0 : f_j;
        f_off += wj ? kChunk - CBS * sub : 0;
        f_kw += wj ? 1 : 0;
        const bool wk = f_kw == g.KW;
        f_kw = wk ? 0 : f_kw;
        f_off += wk ? c_pwt16 - g.KW * kChunk : 0;
        f_kh += wk ? 1 : 0;
        const bool wh = f_kh == g.KH;              // past the unit's last step: wrap (the read is not used)
        f_kh = wh ? 0 : f_kh;
        f_off = wh ? 0 : f_off;
    };
    auto load_frags = [&](v4i (&af)[2][FM], const uint8_t* buf) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int i = 0; i < FM; ++i)
                af[ks][i] = *reinterpret_cast<const v4i*>(buf + fbase[i] + f_off + ks * 2 * p.plane_stride);
    };

    // ---- weight cursor: runs two steps ahead of the multiplications, across units and tiles.
    //      Lane (l32, lhi) of fragment j, half ks holds w[n0 + wn*WTN + j*32 + l32][16 bytes at 16*(2*ks+lhi)];
    //      the lane part of the address is fixed, everything else is uniform ----
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(p.wpk), 0, (int)p.w_bytes, 0x00020000);
    //      Sparse form: lane (l32, lhi) of fragment j holds the 16 kept weights of w[...][32 indices at 32*lhi] and
    //      one word with their positions (two bits each); same addressing with half the bytes per step.
    const __amdgpu_buffer_rsrc_t irsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t*>(p.widx), 0, SP ? (int)(p.w_bytes / 4) : 0, 0x00020000);
    const int wlane = (lhi * p.Np + wn * Cfg::kWTN + l32) * kChunk;
    const int w_half = (SP ? 1 : 2) * p.Np * kChunk;   // bytes between the two 32-index halves of a step
    const int grid_n = grid % p.tiles_n;
    int b_s = 0, b_cb = 0, b_tn = (int)blockIdx.x % p.tiles_n;
    auto next_b_offset = [&]() __attribute__((always_inline)) -> int {
        const int kidx = (b_s / CBS) * p.ksteps_tap + b_cb * CBS + (b_s % CBS);
        const int off = b_tn * TN * kChunk + kidx * 2 * w_half;
        ++b_s;
        const bool ws = b_s == p.nsteps;
        b_s = ws ? 0 : b_s;
        b_cb += ws ? 1 : 0;
        const bool wc = b_cb == p.ncb;
        b_cb = wc ? 0 : b_cb;
        b_tn += wc ? grid_n : 0;
        b_tn -= b_tn >= p.tiles_n ? p.tiles_n : 0;
        return off;
    };
    // dense form: half ks of a step, all FN fragments; sparse form: the whole step of fragments ks*FN/2 .. +FN/2-1
    auto load_b = [&](v4i (&br)[FN], int (&bi)[FN], int wstep, int ks) __attribute__((always_inline)) {
        if constexpr (SP) {
#pragma unroll
            for (int jj = 0; jj < FN / 2; ++jj) {
                const int soff = wstep + (ks * (FN / 2) + jj) * 32 * kChunk;
                br[jj] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wlane, soff, 0));
                bi[jj] = (int)__builtin_amdgcn_raw_buffer_load_b32(irsrc, wlane / 4, soff / 4, 0);
            }
        } else {
#pragma unroll
            for (int j = 0; j < FN; ++j)
                br[j] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wlane, wstep + ks * w_half + j * 32 * kChunk, 0));
        }
    };
    v16i c[FM][FN];
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) c[i][j][v] = 0;
    };
    v4i b_reg[2][2][FN];          // weights of the current and the next step: [step parity][half][fragment]
    int b_idx[2][2][FN];          // sparse form: their position words
    int w_next = 0;               // weight offset of the step two ahead, computed one step early
    v4i a_frag[2][2][FM];         // activation fragments: [step parity][half][fragment]

    // ---- staging wavefronts (wave-specialised form): a loop of their own, so that their registers
    //      and those of the matrix wavefronts do not add up; both loops pass the same barriers ----
    if constexpr (WS) {
        if (producer) {
            load_tile_patch();
#pragma unroll
            for (int i = 0; i < AC; ++i) load_chunk(i);
            stage_npix = lt.npix;
#pragma unroll
            for (int i = 0; i < AC; ++i) stage_chunk(i, lds);
            advance_load_cursor();
            stage_npix = lt.npix;                     // unit 1 is staged while unit 0 is multiplied
#pragma unroll
            for (int i = 0; i < AC; ++i) load_chunk(i);
            advance_load_cursor();
            __syncthreads();
            int p_tile = (int)blockIdx.x, p_cb = 0, p_buf = 0;     // the unit the matrix wavefronts are on
            while (true) {
                uint8_t* sbuf = lds + (p_buf ^ 1) * buf_bytes;
#pragma unroll
                for (int i = 0; i < AC; ++i) {    // trim and write the next unit's chunks, request those of the unit after it
                    // (a chunk whose 256 / PL pixels all lie past the patch holds nothing: skip its trim -- the
                    // staging capacity is sized for the layer's largest patch, most tiles' patches are smaller)
                    if (i * (NT / PL) < stage_npix) stage_chunk(i, sbuf);
                    load_chunk(i);                // unconditional: a request under a condition costs exact wait counts
                }
                p_buf ^= 1;
                const bool tile_done = p_cb == p.ncb - 1;
                __syncthreads();
                if (tile_done) { p_cb = 0; p_tile += grid; } else { ++p_cb; }
                stage_npix = lt.npix;             // the unit requested during the last unit is staged in the next
                advance_load_cursor();
                if (p_tile >= ntiles) break;
            }
            return;
        }
    }

    // ---- prologue: unit 0 staged, unit 1 requested, two weight steps requested ----
    if constexpr (!WS) {
        load_tile_patch();
#pragma unroll
        for (int i = 0; i < AC; ++i) load_chunk(i);
    }
    {
        const int w0 = next_b_offset();
        load_b(b_reg[0][0], b_idx[0][0], w0, 0);
        load_b(b_reg[0][1], b_idx[0][1], w0, 1);
        const int w1 = next_b_offset();
        load_b(b_reg[1][0], b_idx[1][0], w1, 0);
        load_b(b_reg[1][1], b_idx[1][1], w1, 1);
        w_next = next_b_offset();
    }
    if constexpr (!WS) {
        stage_npix = lt.npix;
#pragma unroll
        for (int i = 0; i < AC; ++i) stage_chunk(i, lds);
        advance_load_cursor();
        stage_npix = lt.npix;                         // unit 1 is staged while unit 0 is multiplied
#pragma unroll
        for (int i = 0; i < AC; ++i) load_chunk(i);
        advance_load_cursor();
    }
    setup_compute_tile();
    zero_acc();
    __syncthreads();

    // One reduction step (64 channels of one tap).  A >= 0: the step also trims and stages chunks
    // 2A and 2A+1 of the next unit and requests the same chunks of the unit after it.  The two
    // scheduling regions keep the compiler from sinking the loads next to their uses.
    constexpr int NMF = SP ? FM * FN / 2 : FM * FN;   // matrix instructions per half of a step
    auto step = [&](auto A_, v4i (&cur)[2][FM], v4i (&nxt)[2][FM], v4i (&br)[2][FN], int (&bi)[2][FN], const uint8_t* rbuf, uint8_t* sbuf) __attribute__((always_inline)) {
        constexpr int A = decltype(A_)::value;
        load_frags(nxt, rbuf);                      // f_off already points at the next step
        const int wstep = w_next;
        if constexpr (SP) {
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                const v8i a = __builtin_shufflevector(cur[0][i], cur[1][i], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int j = 0; j < FN / 2; ++j)
                    c[i][j] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(br[0][j], a, c[i][j], bi[0][j], 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    c[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur[0][i], br[0][j], c[i][j], 0, 0, 0);
        }
        load_b(br[0], bi[0], wstep, 0);
        if constexpr (A >= 0) {
            stage_chunk(2 * A, sbuf);
            load_chunk(2 * A);
        } else {
            // plain step: the fragment reads and weight requests of this half are independent of its
            // matrix instructions; issue them in between rather than in front
#pragma unroll
            for (int k = 0; k < NMF; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                            // one matrix instruction
                __builtin_amdgcn_sched_group_barrier(0x100, (2 * FM + NMF - 1) / NMF, 0);     // fragment reads
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);                            // their address adds
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                            // a weight request
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // The cursor arithmetic of the following step (scalar instructions) is issued between this
        // half's matrix instructions, where it is free, instead of in front of the next step's.
        advance_frag_cursor();
        w_next = next_b_offset();
        if constexpr (SP) {
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                const v8i a = __builtin_shufflevector(cur[0][i], cur[1][i], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int j = 0; j < FN / 2; ++j)
                    c[i][FN / 2 + j] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(br[1][j], a, c[i][FN / 2 + j], bi[1][j], 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    c[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur[1][i], br[1][j], c[i][j], 0, 0, 0);
        }
        load_b(br[1], bi[1], wstep, 1);
        if constexpr (A >= 0 && 2 * A + 1 < AC) {
            stage_chunk(2 * A + 1, sbuf);
            load_chunk(2 * A + 1);
        }
#pragma unroll
        for (int k = 0; k < NMF; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                    // one matrix instruction
            __builtin_amdgcn_sched_group_barrier(0x004, (40 + NMF - 1) / NMF, 0); // a slice of the scalar work
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // One unit.  P: parity of the global step count at its start; step s uses fragment and weight
    // slot (P + s) & 1.  The first U0 steps are unrolled (the AS staging steps, plus one plain step if
    // that is what makes the rest an even count); the rest runs as pairs.  Keeping the structure this
    // rigid lets every wait for an outstanding load be exact.
    constexpr bool ODD = Cfg::kOddSteps;
    constexpr int U0 = Cfg::kUnrolled;
    auto run_unit = [&](auto P_, const uint8_t* rbuf, uint8_t* sbuf) __attribute__((always_inline)) {
        constexpr int P = decltype(P_)::value;
        f_j = f_kw = f_kh = f_off = 0;
        load_frags(a_frag[P], rbuf);
        advance_frag_cursor();
        auto head = [&](auto self, auto s_) __attribute__((always_inline)) {
            constexpr int s0 = decltype(s_)::value;
            if constexpr (s0 < U0) {
                step(int_c<(s0 < AS ? s0 : -1)>{}, a_frag[(P + s0) & 1], a_frag[(P + s0 + 1) & 1], b_reg[(P + s0) & 1], b_idx[(P + s0) & 1], rbuf, sbuf);
                self(self, int_c<s0 + 1>{});
            }
        };
        head(head, int_c<0>{});
        constexpr int Q = (P + U0) & 1;
        for (int rem = p.nsteps - U0; rem > 0; rem -= 2) {
            step(int_c<-1>{}, a_frag[Q], a_frag[Q ^ 1], b_reg[Q], b_idx[Q], rbuf, sbuf);
            step(int_c<-1>{}, a_frag[Q ^ 1], a_frag[Q], b_reg[Q ^ 1], b_idx[Q ^ 1], rbuf, sbuf);
        }
    };

    // End of a unit: results out if it was the tile's last channel block, barrier, cursors forward.
    int ubuf = 0;
    auto boundary = [&]() __attribute__((always_inline)) {
        ubuf ^= 1;
        const bool tile_done = c_cb == p.ncb - 1;
        if (tile_done) {
            // ---- epilogue: undo the -128 offset, store int32 and/or dequantised fp32 ----
            // Register v of fragment (i, j) is pixel 8*(v/4) + 4*lhi + v%4, channel l32: each store
            // instruction writes two full 128-byte runs of consecutive channels.
            const int64_t m0 = (int64_t)c_tm * kPatchTM;
            const int n0 = c_tn * TN;
            {
                // Buffer stores relative to the tile's first row: the lane's part of the offset is computed
                // once, every row adds a uniform multiple of the row pitch, and rows past M or channels
                // past N fall outside the buffer's range and are dropped by the hardware (no per-row
                // branches, no 64-bit address arithmetic).  One copy per combination of outputs, chosen per tile.
                const int rows = g.M - (int)m0 < kPatchTM ? g.M - (int)m0 : kPatchTM;
#pragma unroll
                for (int j = 0; j < (SP ? 0 : FN); ++j) asm volatile("" : "+v"(corr[j]), "+v"(sc[j]));   // the tile's constants have landed from here on
                auto store_tile = [&](auto acc_, auto out_, auto u8_) __attribute__((always_inline)) {
                    constexpr bool kAcc = decltype(acc_)::value, kOut = decltype(out_)::value, kU8 = decltype(u8_)::value;
                    constexpr int kElem = kU8 ? 1 : 4;                 // bytes per stored result
                    const int pitch = p.N * kElem;
                    const int tile_bytes = rows * pitch;
                    const __amdgpu_buffer_rsrc_t arsrc = __builtin_amdgcn_make_buffer_rsrc(
                        kAcc ? (void*)(p.acc + m0 * p.N) : nullptr, 0, kAcc ? tile_bytes : 0, 0x00020000);
                    const __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(
                        kOut ? (void*)(p.out + m0 * p.N) : kU8 ? (void*)(p.out_u8 + m0 * p.N) : nullptr, 0,
                        (kOut || kU8) ? tile_bytes : 0, 0x00020000);
                    uint32_t lane_off[FN];
#pragma unroll
                    for (int j = 0; j < FN; ++j) {
                        const int n = n0 + wn * Cfg::kWTN + j * 32 + l32;
                        lane_off[j] = n < p.N ? (uint32_t)((wm * Cfg::kWTM + 4 * lhi) * pitch + n * kElem) : 0x80000000u;
                    }
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int row_bytes = (i * 32 + 8 * (v / 4) + (v % 4)) * pitch;
#pragma unroll
                            for (int j = 0; j < FN; ++j) {
                                const int32_t r = c[i][j][v] + corr[j];
                                const int off = (int)(lane_off[j] + (uint32_t)row_bytes);
                                if constexpr (kAcc) __builtin_amdgcn_raw_buffer_store_b32(r, arsrc, off, 0, kResultStorePolicy);
                                if constexpr (kOut)
                                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, __fmul_rn((float)r, sc[j])), orsrc, off, 0, kResultStorePolicy);
                                if constexpr (kU8)
                                    __builtin_amdgcn_raw_buffer_store_b8((unsigned char)requant_u8(r, sc[j]), orsrc, off, 0, 0);
                            }
                        }
                };
                // Requantised bytes, N a multiple of 4: the four rows a lane holds of one channel are exchanged
                // inside groups of four lanes for four channels of one row: one 32-bit store instead of four
                // byte stores (the byte form is bound by the number of store instructions).
                auto store_tile_u8_packed = [&](auto trim_) __attribute__((always_inline)) {
                    constexpr bool kTrimOut = decltype(trim_)::value;   // the next layer's trim applied here, once per result
                    const int pitch = p.N;
                    const __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(
                        (void*)(p.out_u8 + m0 * p.N), 0, rows * pitch, 0x00020000);
                    const QuadSel qs = quad_transpose_selectors(l32);
                    uint32_t lane_off[FN];
#pragma unroll
                    for (int j = 0; j < FN; ++j) {
                        const int n4 = (n0 + wn * Cfg::kWTN + j * 32 + l32) & ~3;
                        lane_off[j] = n4 < p.N ? (uint32_t)((wm * Cfg::kWTM + 4 * lhi + (l32 & 3)) * pitch + n4) : 0x80000000u;
                    }
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int row_bytes = (i * 32 + 8 * q) * pitch;
#pragma unroll
                            for (int j = 0; j < FN; ++j) {
                                const uint32_t w = requant_u8x4(c[i][j][4 * q] + corr[j], c[i][j][4 * q + 1] + corr[j], c[i][j][4 * q + 2] + corr[j],
                                                            c[i][j][4 * q + 3] + corr[j], sc[j]);
                                // after the transpose the word holds channels n4 .. n4+3 of one pixel: two pairs
                                uint32_t t = quad_transpose_bytes(w, qs);
                                if constexpr (kTrimOut) t = trim4_kind<KIND>(t, p.luts);
                                __builtin_amdgcn_raw_buffer_store_b32((int)t, orsrc, (int)(lane_off[j] + (uint32_t)row_bytes), 0, 0);
                            }
                        }
                };
                // Sparse form: the weights are the matrix instruction's row operand, so register v of fragment
                // (i, j) is channel 8*(v/4) + 4*lhi + v%4 of pixel l32.  Stored straight from the registers that is
                // 16 bytes per lane to 32 different rows per instruction; instead the accumulators go through a
                // wavefront-private LDS area ([32 pixels][64 channels] int32, rows padded to 272 bytes) and leave
                // as whole rows: a lane reads 16 bytes of a row, applies its four channels' constants and every
                // store instruction writes four 256-byte runs.  The LDS queue of a wavefront is in order, so its
                // reads see its writes without a barrier.
                auto store_tile_sp = [&](auto acc_, auto out_, auto vec_) __attribute__((always_inline)) {
                    constexpr bool kAcc = decltype(acc_)::value, kOut = decltype(out_)::value, kVec = decltype(vec_)::value;
                    const int pitch = p.N * 4;
                    const int tile_bytes = rows * pitch;
                    const __amdgpu_buffer_rsrc_t arsrc = __builtin_amdgcn_make_buffer_rsrc(
                        kAcc ? (void*)(p.acc + m0 * p.N) : nullptr, 0, kAcc ? tile_bytes : 0, 0x00020000);
                    const __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(
                        kOut ? (void*)(p.out + m0 * p.N) : nullptr, 0, kOut ? tile_bytes : 0, 0x00020000);
                    // (the lane number made opaque here: otherwise the addresses below are computed once, ahead of
                    // the tile loop, and held in registers the step loop then has to spill)
                    int le = lane;
                    asm volatile("" : "+v"(le));
                    uint8_t* xr = lds + 2 * buf_bytes + kChunk + wave * (32 * kSparseRowPitch);
                    uint8_t* xw = xr + (le & 31) * kSparseRowPitch + 16 * (le >> 5);
                    const uint8_t* xrd = xr + (le >> 4) * kSparseRowPitch + (le & 15) * 16;
                    const int nrun = n0 + wn * Cfg::kWTN + (le & 15) * 4;            // first channel of this lane's 16 bytes
                    const uint32_t run_off = (uint32_t)((wm * Cfg::kWTM + (le >> 4)) * pitch + nrun * 4);
                    // the lane's four channels' constants: requested here, ahead of every store, and not at the
                    // tile's start (the step loop has no registers to spare for them)
                    static_assert(!SP || Cfg::kWTN == 64, "64 channels per wavefront");
                    int32_t corr4[4];
                    float sc4[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int nc = nrun + e < p.N ? nrun + e : 0;
                        corr4[e] = p.colsum[nc] * 128;
                        sc4[e] = scale_or_dummy[nc];
                    }
#pragma unroll
                    for (int i = 0; i < FM; ++i) {
#pragma unroll
                        for (int j = 0; j < FN; ++j)
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const v4i r = {c[i][j][4 * q], c[i][j][4 * q + 1], c[i][j][4 * q + 2], c[i][j][4 * q + 3]};
                                *reinterpret_cast<v4i*>(xw + (j * 32 + 8 * q) * 4) = r;
                            }
#pragma unroll
                        for (int k = 0; k < 8; ++k) {
                            v4i r = *reinterpret_cast<const v4i*>(xrd + 4 * k * kSparseRowPitch);
                            v4i f;
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                r[e] += corr4[e];
                                f[e] = __builtin_bit_cast(int, __fmul_rn((float)r[e], sc4[e]));
                            }
                            const uint32_t off = run_off + (uint32_t)((i * 32 + 4 * k) * pitch);
                            if constexpr (kVec) {      // N % 4 == 0: the four channels are inside N together or not at all
                                const int o = (int)(nrun < p.N ? off : 0x80000000u);
                                if constexpr (kAcc) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, r), arsrc, o, 0, kResultStorePolicy);
                                if constexpr (kOut) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, f), orsrc, o, 0, kResultStorePolicy);
                            } else {
#pragma unroll
                                for (int e = 0; e < 4; ++e) {
                                    const int o = (int)(nrun + e < p.N ? off + 4u * e : 0x80000000u);
                                    if constexpr (kAcc) __builtin_amdgcn_raw_buffer_store_b32(r[e], arsrc, o, 0, kResultStorePolicy);
                                    if constexpr (kOut) __builtin_amdgcn_raw_buffer_store_b32(f[e], orsrc, o, 0, kResultStorePolicy);
                                }
                            }
                        }
                    }
                };
                if constexpr (SP) {
                    const bool vec = (p.N & 3) == 0;
                    if (p.acc && p.out) { if (vec) store_tile_sp(std::true_type{}, std::true_type{}, std::true_type{}); else store_tile_sp(std::true_type{}, std::true_type{}, std::false_type{}); }
                    else if (p.out) { if (vec) store_tile_sp(std::false_type{}, std::true_type{}, std::true_type{}); else store_tile_sp(std::false_type{}, std::true_type{}, std::false_type{}); }
                    else { if (vec) store_tile_sp(std::true_type{}, std::false_type{}, std::true_type{}); else store_tile_sp(std::true_type{}, std::false_type{}, std::false_type{}); }
                } else
                if (p.out_u8 && (p.N & 3) == 0) {
                    if (KIND != kTrimNone && p.trim_out) store_tile_u8_packed(std::true_type{});
                    else store_tile_u8_packed(std::false_type{});
                }
                else if (p.out_u8) store_tile(std::false_type{}, std::false_type{}, std::true_type{});
                else if (p.acc && p.out) store_tile(std::true_type{}, std::true_type{}, std::false_type{});
                else if (p.out) store_tile(std::false_type{}, std::true_type{}, std::false_type{});
                else store_tile(std::true_type{}, std::false_type{}, std::false_type{});
            }
            zero_acc();
        }
        __syncthreads();
        if (++c_cb == p.ncb) {
            c_cb = 0;
            c_tile += grid;
            if (c_tile < ntiles) setup_compute_tile();
        }
        if constexpr (!WS) {
            stage_npix = lt.npix;                 // the unit requested during the last unit is staged in the next
            advance_load_cursor();
        }
    };

    while (true) {
        run_unit(int_c<0>{}, lds + ubuf * buf_bytes, lds + (ubuf ^ 1) * buf_bytes);
        boundary();
        if (c_tile >= ntiles) break;
        if constexpr (ODD) {       // an odd number of steps flips the slot parity: alternate two copies
            run_unit(int_c<1>{}, lds + ubuf * buf_bytes, lds + (ubuf ^ 1) * buf_bytes);
            boundary();
            if (c_tile >= ntiles) break;
        }
    }
}


// `p` carries everything except plane_stride and the tile counts; npix_max bounds TilePatch::npix.
template <class Cfg, int KIND>
sparq_status launch_patch_cfg(const PatchParams& p, int npix_max, hipStream_t s) {
    PatchParams q = p;
    q.plane_stride = patch_plane_stride(npix_max, Cfg::kPlanes);
    const int lds_bytes = 2 * Cfg::kPlanes * q.plane_stride + kChunk +    // two patch buffers + the dummy chunk
                          (Cfg::kSparse ? kSparseEpilogueLds : 0);         // + the sparse form's result rows
    if (p.g.rm_wo && !Cfg::kWaveSpecialised) return SPARQ_EUNSUPPORTED;
    if (Cfg::kSparse != (p.widx != nullptr) || (Cfg::kSparse && p.out_u8)) return SPARQ_EUNSUPPORTED;
    if (!p.trim_in && !Cfg::kWaveSpecialised && KIND != kTrimNone) return SPARQ_EUNSUPPORTED;
    if ((int64_t)p.N * 4 * kPatchTM >= 0x7FFFFFFF) return SPARQ_EUNSUPPORTED;   // 32-bit offsets inside a tile of results
    if (npix_max > Cfg::kMaxPix || lds_bytes > kLdsPerCu || q.nsteps < Cfg::kUnrolled ||
        ((q.nsteps - Cfg::kUnrolled) & 1))
        return SPARQ_EUNSUPPORTED;
    auto kern = conv_patch_kernel<Cfg, KIND>;
    // largest dynamic LDS size enabled so far, per device (relaxed atomics: concurrent callers at worst repeat the call)
    static std::atomic<int> lds_set_dev[kMaxDevices];
    std::atomic<int>& lds_set = lds_set_dev[current_device_slot()];
    if (lds_bytes > lds_set.load(std::memory_order_relaxed) || current_device_slot() == kMaxDevices - 1) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                lds_bytes) != hipSuccess)
            return SPARQ_ELAUNCH;
        lds_set.store(lds_bytes, std::memory_order_relaxed);
    }
    q.tiles_m = (p.g.M + kPatchTM - 1) / kPatchTM;
    q.tiles_n = (p.N + Cfg::kTN - 1) / Cfg::kTN;
    const int64_t tiles = (int64_t)q.tiles_m * q.tiles_n;
    if (tiles > 0x7FFFFFFF) return SPARQ_EUNSUPPORTED;
    int per_cu = kLdsPerCu / lds_bytes;
    if (per_cu > Cfg::kWgPerCu) per_cu = Cfg::kWgPerCu;
    const int64_t resident = (int64_t)device_cu_count() * per_cu;
    const unsigned blocks = (unsigned)(tiles < resident ? tiles : resident);
    kern<<<blocks, Cfg::kThreads, lds_bytes, s>>>(q);
    return launch_status();
}

template <class Cfg>
sparq_status launch_patch_kind(TrimKind kind, const PatchParams& p, int npix_max, hipStream_t s) {
    switch (kind) {
        case kTrimNone: return launch_patch_cfg<Cfg, kTrimNone>(p, npix_max, s);
        case kTrimFloor: return launch_patch_cfg<Cfg, kTrimFloor>(p, npix_max, s);
        case kTrimFloorPair: return launch_patch_cfg<Cfg, kTrimFloorPair>(p, npix_max, s);
        case kTrimFloorPairWide: return launch_patch_cfg<Cfg, kTrimFloorPairWide>(p, npix_max, s);
        case kTrimRound: return launch_patch_cfg<Cfg, kTrimRound>(p, npix_max, s);
        case kTrimRound4: return launch_patch_cfg<Cfg, kTrimRound4>(p, npix_max, s);
        case kTrimRoundPairWide: return launch_patch_cfg<Cfg, kTrimRoundPairWide>(p, npix_max, s);
        case kTrimRoundPair4: return launch_patch_cfg<Cfg, kTrimRoundPair4>(p, npix_max, s);
        default: return SPARQ_EUNSUPPORTED;
    }
}

// Sparse form: the trim variants that look at one activation at a time (with pairing on, the caller expands the
// problem first and the kernel runs at plain 8 bits).
template <class Cfg>
sparq_status launch_patch_kind_sparse(TrimKind kind, const PatchParams& p, int npix_max, hipStream_t s) {
    static_assert(Cfg::kSparse, "sparse configuration expected");
    switch (kind) {
        case kTrimNone: return launch_patch_cfg<Cfg, kTrimNone>(p, npix_max, s);
        case kTrimFloor: return launch_patch_cfg<Cfg, kTrimFloor>(p, npix_max, s);
        case kTrimRound: return launch_patch_cfg<Cfg, kTrimRound>(p, npix_max, s);
        case kTrimRound4: return launch_patch_cfg<Cfg, kTrimRound4>(p, npix_max, s);
        default: return SPARQ_EUNSUPPORTED;
    }
}

// One translation unit per tile shape instantiates every trim variant and exports a launcher.
typedef sparq_status (*PatchLauncher)(TrimKind, const PatchParams&, int, hipStream_t);
#define SPARQ_DECLARE_PATCH(name) sparq_status name(TrimKind kind, const PatchParams& p, int npix_max, hipStream_t s)
SPARQ_DECLARE_PATCH(launch_patch_ws_n64_a2c1);
SPARQ_DECLARE_PATCH(launch_patch_ws_n64_a4c1);
SPARQ_DECLARE_PATCH(launch_patch_ws_n64_a8c1);
SPARQ_DECLARE_PATCH(launch_patch_ws_n64_a12c1);
SPARQ_DECLARE_PATCH(launch_patch_ws_n64_a4c2);
SPARQ_DECLARE_PATCH(launch_patch_ws_n64_a8c4);
SPARQ_DECLARE_PATCH(launch_patch_ws_n128_a2c1);
SPARQ_DECLARE_PATCH(launch_patch_ws_n128_a4c1);
SPARQ_DECLARE_PATCH(launch_patch_ws_n128_a8c1);
SPARQ_DECLARE_PATCH(launch_patch_ws_n128_a12c1);
SPARQ_DECLARE_PATCH(launch_patch_ws_n128_a4c2);
SPARQ_DECLARE_PATCH(launch_patch_ws_n128_a8c4);
SPARQ_DECLARE_PATCH(launch_patch_ws_n256_a2c1);
SPARQ_DECLARE_PATCH(launch_patch_ws_n256_a4c1);
SPARQ_DECLARE_PATCH(launch_patch_ws_n256_a8c1);
SPARQ_DECLARE_PATCH(launch_patch_ws_n256_a12c1);
SPARQ_DECLARE_PATCH(launch_patch_ws_n256_a4c2);
SPARQ_DECLARE_PATCH(launch_patch_ws_n256_a8c4);
SPARQ_DECLARE_PATCH(launch_patch_sp_n64_a2c1);
SPARQ_DECLARE_PATCH(launch_patch_sp_n64_a4c1);
SPARQ_DECLARE_PATCH(launch_patch_sp_n64_a8c1);
SPARQ_DECLARE_PATCH(launch_patch_sp_n64_a12c1);
SPARQ_DECLARE_PATCH(launch_patch_sp_n64_a4c2);
SPARQ_DECLARE_PATCH(launch_patch_sp_n64_a8c4);
SPARQ_DECLARE_PATCH(launch_patch_sp_n128_a2c1);
SPARQ_DECLARE_PATCH(launch_patch_sp_n128_a4c1);
SPARQ_DECLARE_PATCH(launch_patch_sp_n128_a8c1);
SPARQ_DECLARE_PATCH(launch_patch_sp_n128_a12c1);
SPARQ_DECLARE_PATCH(launch_patch_sp_n128_a4c2);
SPARQ_DECLARE_PATCH(launch_patch_sp_n128_a8c4);
SPARQ_DECLARE_PATCH(launch_patch_sp_n256_a2c1);
SPARQ_DECLARE_PATCH(launch_patch_sp_n256_a4c1);
SPARQ_DECLARE_PATCH(launch_patch_sp_n256_a8c1);
SPARQ_DECLARE_PATCH(launch_patch_sp_n256_a12c1);
SPARQ_DECLARE_PATCH(launch_patch_sp_n256_a4c2);
SPARQ_DECLARE_PATCH(launch_patch_sp_n256_a8c4);
SPARQ_DECLARE_PATCH(launch_patch_n64_a12c1);
SPARQ_DECLARE_PATCH(launch_patch_n128_a12c1);
SPARQ_DECLARE_PATCH(launch_patch_n256_a12c1);
SPARQ_DECLARE_PATCH(launch_patch_n64_a2c1);
SPARQ_DECLARE_PATCH(launch_patch_n64_a4c1);
SPARQ_DECLARE_PATCH(launch_patch_n64_a8c1);
SPARQ_DECLARE_PATCH(launch_patch_n64_a4c2);
SPARQ_DECLARE_PATCH(launch_patch_n64_a8c4);
SPARQ_DECLARE_PATCH(launch_patch_n128_a2c1);
SPARQ_DECLARE_PATCH(launch_patch_n128_a4c1);
SPARQ_DECLARE_PATCH(launch_patch_n128_a8c1);
SPARQ_DECLARE_PATCH(launch_patch_n128_a4c2);
SPARQ_DECLARE_PATCH(launch_patch_n128_a8c4);
SPARQ_DECLARE_PATCH(launch_patch_n256_a2c1);
SPARQ_DECLARE_PATCH(launch_patch_n256_a4c1);
SPARQ_DECLARE_PATCH(launch_patch_n256_a8c1);
SPARQ_DECLARE_PATCH(launch_patch_n256_a4c2);
SPARQ_DECLARE_PATCH(launch_patch_n256_a8c4);

}  // namespace sparq
