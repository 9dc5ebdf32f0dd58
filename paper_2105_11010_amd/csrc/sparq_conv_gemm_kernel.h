// Fused SPARQ convolution-as-GEMM for gfx950.
//
//   acc[m][n] = sum_k T(x)[m, k] * w[n][k]          (Eq. 1 over trimmed activations)
//
// The im2col matrix is never materialised: every workgroup gathers its
// activation tile straight from the NHWC tensor with 128-bit loads (one load =
// 16 consecutive channels of one pixel = 8 vSPARQ pairs inside one lane), trims
// the four packed words in registers (sparq_swar.h), flips them to signed
// (x - 128, a single xor) and stages them in LDS, from where all wavefronts of
// the workgroup read them.  Weights are pre-packed in matrix-instruction
// fragment order and go from L2 straight into registers.  The contraction runs
// on v_mfma_i32_32x32x32_i8; the epilogue adds back 128 * sum_k w[n][k], which
// makes the result exact in int32, and optionally applies the per-channel
// dequantisation factor (Section 5).
//
// This mirrors the paper's placement of the trimming unit in front of the
// array (Section 5: it runs at a much lower rate than the multipliers): an
// activation is trimmed once when its tile is loaded and then reused for all
// output channels the workgroup covers.
#pragma once
#include <atomic>

#include "sparq_common.h"
#include "sparq_fastdiv.h"

namespace sparq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

struct GemmParams {
    const uint8_t* x;        // activations, NHWC with C a multiple of 16
    const uint8_t* wpk;      // packed weight tiles
    const int32_t* colsum;   // sum_k w[n][k], Np entries
    int32_t* acc;            // [M][N] or null
    const float* scale;      // [N] or null
    float* out;              // [M][N] or null
    uint8_t* out_u8;         // [M][N] requantised output or null (then it is the only output; scale holds its factors)
    int trim_out;            // out_u8 with N % 4 == 0 only: trim the requantised bytes with this launch's own mode as well
    int64_t M;
    uint32_t x_bytes;
    int N, Np, Kk, nkb;
    int scale_n;             // scale[] has this many entries and is indexed by n % scale_n (pixel-folded layers repeat it)
    int H, W, C, Cq, Ho, Wo, KH, KW, sh, sw, ph, pw;   // C: channels per pixel in x; Cq: per tap in the packed weights
    int tiles_m, tiles_n;
    float rcp_c, rcp_kw;     // 1/Cq and 1/KW for the branch-free reduction-index decode
    FastDiv div_wo, div_ho;  // output row -> (image, oy, ox) by multiply-high; valid when rows_fit_31
    int rows_fit_31;         // M < 2^31
    TrimLuts luts;
};

constexpr uint32_t kInvalidOffset = 0x80000000u;   // beyond any buffer this kernel accepts (< 2 GiB)

constexpr int gcd2(int a, int b) { return b == 0 ? a : gcd2(b, a % b); }
constexpr int lcm3(int a, int b, int c) { int l = a / gcd2(a, b) * b; return l / gcd2(l, c) * c; }

// Tile shape: TM output pixels x TN output channels per workgroup, WGM x WGN
// wavefronts.  PA / PB: how many reduction steps ahead of their consumption the
// activation / weight loads are issued.
//
// HALF selects the main loop pipelined by half steps (32 reduction indices): operand fragments are double-buffered
// per half rather than per step, which halves their registers and leaves room for activation requests several
// steps ahead even when a wavefront's accumulators fill the whole accumulation register file (128 x 128 results).
// There PA counts the steps between an activation's request and its trim (the ring holds PA + 1 steps) and PB the
// halves a weight fragment is requested ahead.
template <int TM, int TN, int WGM, int WGN, int PA, int PB, bool SPLIT = false, int WPC = 0, bool HALF = false>
struct TileCfg {
    static constexpr bool kHalfPipe = HALF;
    static constexpr bool kSplitTrim = SPLIT;                   // trim half of the activations in each scheduling region
    static constexpr int kTM = TM, kTN = TN, kWGM = WGM, kWGN = WGN, kPA = PA, kPB = PB;
    static constexpr int kThreads = 64 * WGM * WGN;
    static constexpr int kWTM = TM / WGM, kWTN = TN / WGN;      // per-wavefront tile
    static constexpr int kFM = kWTM / 32, kFN = kWTN / 32;      // 32x32 fragments per wavefront
    static constexpr int kAChunks = TM * 4 / kThreads;          // 16-byte activation loads per lane per step
    // Only activations go through LDS (they are trimmed once and shared by all
    // wavefronts); every wavefront reads its own weight fragments straight from the
    // packed buffer.  A stage holds four 16-byte-chunk planes, [plane][row][16]; planes
    // are padded by 64 bytes so that the four lanes that write one row's 64 bytes (one
    // chunk each, into four different planes) land on different banks.
    static constexpr int kPlaneA = TM * kChunk + 64;
    static constexpr int kLdsA = 4 * kPlaneA;                   // bytes per stage
    static constexpr int kStages = HALF ? 4 : 3;                // written two steps ahead, read one step ahead
    static constexpr int kLdsBytes = kStages * kLdsA;
    static constexpr int kUnroll = HALF ? 4 : lcm3(2, PA, PB);  // main-loop unroll: every ring index compile-time
    // resident workgroups per CU the register budget is set for (0: two with small accumulators, else one)
    static constexpr int kWgPerCu = WPC ? WPC : ((kFM * kFN * 16 <= 64) ? 2 : 1);
    // the widest tile has no registers to spare for a third epilogue copy: no requantised-byte output
    static constexpr bool kByteOutput = kFM * kFN * 16 <= 128;
    static_assert(TM % (32 * WGM) == 0 && TN % (32 * WGN) == 0, "tile must split into 32x32 fragments");
    static_assert((TM * 4) % kThreads == 0, "activation loads must divide evenly");
    static_assert(PA >= 1 && PA <= 4 && PB >= 1 && PB <= 8, "prefetch depth");
    static_assert(HALF || (kUnroll % 2 == 0 && kUnroll % PA == 0 && kUnroll % PB == 0), "unroll must cover all rings");
    static_assert(!HALF || (PA == 3 && (PB == 2 || PB == 4 || PB == 8) && kAChunks % 2 == 0), "half-step loop: rings of four steps / PB halves");
};

template <class Cfg, int KIND>
__global__ __launch_bounds__(Cfg::kThreads, Cfg::kWgPerCu * Cfg::kThreads / 256) void conv_gemm_kernel(const GemmParams p) {
    constexpr int TM = Cfg::kTM, NT = Cfg::kThreads, PA = Cfg::kPA, PB = Cfg::kPB, U = Cfg::kUnroll;
    constexpr int FM = Cfg::kFM, FN = Cfg::kFN, AC = Cfg::kAChunks;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];   // [3][4][TM (+pad)][16]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % Cfg::kWGM, wn = wave / Cfg::kWGM;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int kc = tid & 3;                  // which 16-byte chunk of a row's 64-byte step this lane gathers
    const int nkb = p.nkb;
    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(p.x), 0, (int)p.x_bytes, 0x00020000);
    const int ntiles = p.tiles_m * p.tiles_n;

    // Persistent workgroups: each one walks over tiles blockIdx.x, blockIdx.x + gridDim.x, ...
    // so that the result stores of one tile drain while the next tile's loads and matrix
    // instructions already run.  The output-channel tile is the fast index: consecutive
    // tile numbers share their activation rows.
    for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int tile_n = tile % p.tiles_n;
        const int tile_m = tile / p.tiles_n;
        const int64_t m0 = (int64_t)tile_m * TM;
        const int n0 = tile_n * Cfg::kTN;

        // ---- activation gather bookkeeping (fixed per lane and tile) ----
        int32_t row_base[AC];                    // byte offset of (b, oy*sh-ph, ox*sw-pw, 0)
        int32_t row_iy[AC], row_ix[AC];
#pragma unroll
        for (int i = 0; i < AC; ++i) {
            int64_t m = m0 + (tid >> 2) + i * (NT / 4);
            if (m >= p.M) m = p.M - 1;
            int ox, oy, b;
            if (p.rows_fit_31) {                 // uniform; every shape of the paper's networks takes this side
                const uint32_t mu = (uint32_t)m;
                const uint32_t t = fastdiv(mu, p.div_wo);
                const uint32_t img = fastdiv(t, p.div_ho);
                ox = (int)(mu - t * (uint32_t)p.Wo);
                oy = (int)(t - img * (uint32_t)p.Ho);
                b = (int)img;
            } else {
                ox = (int)(m % p.Wo);
                const int64_t t = m / p.Wo;
                oy = (int)(t % p.Ho);
                b = (int)(t / p.Ho);
            }
            const int iy0 = oy * p.sh - p.ph, ix0 = ox * p.sw - p.pw;
            row_iy[i] = iy0;
            row_ix[i] = ix0;
            row_base[i] = (int32_t)((((int64_t)b * p.H + iy0) * p.W + ix0) * p.C);
        }

        // Per-channel constants of the epilogue (128 * sum_k w[n][k] and the dequantisation / requantisation factor),
        // requested when the tile starts where the registers allow it: a request at the tile's end exposes a memory
        // latency per tile, which short reductions (a network's first layer: six steps) cannot afford.
        constexpr bool kEarlyConsts = FM * FN * 16 <= 128;
        int32_t corr_t[FN];
        float sc_t[FN];
        if constexpr (kEarlyConsts) {
            const bool scaled = p.out || p.out_u8;
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int n = n0 + wn * Cfg::kWTN + j * 32 + l32;
                const int nc = n < p.N ? n : 0;
                corr_t[j] = 128 * p.colsum[nc];
                sc_t[j] = scaled ? p.scale[nc % p.scale_n] : 0.0f;
            }
        }

        // Everything inside the main loop is branch-free so that the loop body stays one
        // basic block and outstanding loads can be waited on exactly.  Steps past the end
        // request out-of-range activations (returned as zeros) and re-read the last weight
        // step; they are staged but never multiplied.
        int a_step = 0;                          // next activation step to request
        // (opaque, so that the address arithmetic of the first requests is not computed once for all tiles and
        // then kept in registers the main loop has no room for)
        asm volatile("" : "+s"(a_step));
        // Half-step form: the host picks it only when a tap's extent is a multiple of the 64-byte step, so the
        // tap of a step is the same for all lanes and is tracked in scalar registers, advanced by one step per
        // request (the general form below decodes the reduction index per lane).
        int s_c0 = 0, s_kh = 0, s_kw = 0;
        auto load_a = [&](v4u (&ar)[AC]) {
            if constexpr (Cfg::kHalfPipe) {
                const bool k_ok = a_step < nkb;
                const int32_t tap_off = (s_kh * p.W + s_kw) * p.C + s_c0 + kc * kChunk;
                const bool c_ok = s_c0 + kc * kChunk < p.C;          // false in a tap's channel padding
#pragma unroll
                for (int i = 0; i < AC; ++i) {
                    const bool ok = k_ok & c_ok & ((unsigned)(row_iy[i] + s_kh) < (unsigned)p.H) &
                                    ((unsigned)(row_ix[i] + s_kw) < (unsigned)p.W);
                    const uint32_t off = ok ? (uint32_t)(row_base[i] + tap_off) : kInvalidOffset;
                    ar[i] = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, (int)off, 0, 0);
                }
                s_c0 += kStepK;
                const bool wrap_c = s_c0 >= p.Cq;
                s_c0 = wrap_c ? 0 : s_c0;
                s_kw += wrap_c;
                const bool wrap_w = s_kw >= p.KW;
                s_kw = wrap_w ? 0 : s_kw;
                s_kh += wrap_w;
                ++a_step;
                return;
            }
            // where this lane's 16 bytes sit in the (kh, kw, c) reduction index
            const int k = a_step * kStepK + kc * kChunk;
            int tap = (int)((float)k * p.rcp_c);
            int c0 = k - tap * p.Cq;
            tap += (c0 >= p.Cq) - (c0 < 0);
            c0 = k - tap * p.Cq;
            int kh = (int)((float)tap * p.rcp_kw);
            int kw = tap - kh * p.KW;
            kh += (kw >= p.KW) - (kw < 0);
            kw = tap - kh * p.KW;
            const bool k_ok = (k < p.Kk) & (c0 < p.C);   // false in a tap's channel padding and past the end
            const int32_t tap_off = (kh * p.W + kw) * p.C + c0;
#pragma unroll
            for (int i = 0; i < AC; ++i) {
                const bool ok = k_ok & ((unsigned)(row_iy[i] + kh) < (unsigned)p.H) &
                                ((unsigned)(row_ix[i] + kw) < (unsigned)p.W);
                const uint32_t off = ok ? (uint32_t)(row_base[i] + tap_off) : kInvalidOffset;
                ar[i] = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, (int)off, 0, 0);   // out of range reads 0
            }
            ++a_step;
        };

        // trim + flip to signed + stage in LDS; chunks [i0, i1) of this lane
        auto store_a = [&](int stage, const v4u (&ar)[AC], int i0, int i1) {
            uint8_t* sa = lds + stage * Cfg::kLdsA + kc * Cfg::kPlaneA + (tid >> 2) * kChunk;
#pragma unroll
            for (int i = i0; i < i1; ++i) {
                v4u v = ar[i];
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = trim4_kind<KIND>(v[j], p.luts) ^ 0x80808080u;
                *reinterpret_cast<v4u*>(sa + i * (NT / 4) * kChunk) = v;
            }
        };

        // weight fragments: lane (l32, lhi) of fragment j, half ks holds
        // w[n0 + wn*WTN + j*32 + l32][k = 16*(2*ks + lhi) .. +15]
        const uint8_t* wsrc = p.wpk + ((size_t)lhi * p.Np + n0 + wn * Cfg::kWTN + l32) * kChunk;
        const size_t w_half = (size_t)2 * p.Np * kChunk;      // bytes between the two 32-wide halves of a step
        int b_step = 0;
        auto load_b = [&](v4i (&br)[FN], int ks) {
#pragma unroll
            for (int j = 0; j < FN; ++j) br[j] = *reinterpret_cast<const v4i*>(wsrc + ks * w_half + j * 32 * kChunk);
        };
        auto advance_b = [&]() {
            ++b_step;
            wsrc += (b_step < nkb) ? 2 * w_half : 0;
        };

        auto load_frags = [&](int stage, v4i (&af)[2][FM]) {
            const uint8_t* sa = lds + stage * Cfg::kLdsA + (wm * Cfg::kWTM + l32) * kChunk + lhi * Cfg::kPlaneA;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int i = 0; i < FM; ++i)
                    af[ks][i] = *reinterpret_cast<const v4i*>(sa + ks * 2 * Cfg::kPlaneA + i * 32 * kChunk);
        };

        v16i c[FM][FN];
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) c[i][j][v] = 0;

        if constexpr (Cfg::kHalfPipe) {
        // ---- main loop pipelined by half steps ----
        // Step s: requested at step s-2-PA, trimmed and staged during step s-2 (one half of a lane's chunks in
        // each half step), its fragments read one half ahead of the matrix instructions that use them.  Weights
        // of half h are requested at half h-PB, right after the matrix instructions that read the same registers.
        constexpr int RA = PA + 1, RB = PB;
        static_assert(RA == 4, "ring indices below assume four activation steps in flight");
        v4u a_reg[RA][AC];            // activation requests in flight: step s in slot s % 4
        v4i b_frag[RB][FN];           // weight fragments: half h in slot h % RB
        v4i a_frag[2][FM];            // activation fragments: half h in slot h % 2
        const int nhalves = 2 * nkb;
        int b_half = 0;
        auto load_bh = [&](v4i (&br)[FN]) {
#pragma unroll
            for (int j = 0; j < FN; ++j) br[j] = *reinterpret_cast<const v4i*>(wsrc + j * 32 * kChunk);
            ++b_half;
            wsrc += (b_half < nhalves) ? w_half : 0;
        };
        auto frags = [&](int stage, int ks, v4i (&a)[FM]) {
            const uint8_t* sa = lds + stage * Cfg::kLdsA + (2 * ks + lhi) * Cfg::kPlaneA + (wm * Cfg::kWTM + l32) * kChunk;
#pragma unroll
            for (int i = 0; i < FM; ++i) a[i] = *reinterpret_cast<const v4i*>(sa + i * 32 * kChunk);
        };
        auto multiply = [&](const v4i (&a)[FM], const v4i (&b)[FN]) {
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int i = 0; i < FM; ++i) c[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], c[i][j], 0, 0, 0);
        };
        {
            load_a(a_reg[0]);
            load_a(a_reg[1]);
            load_a(a_reg[2]);
            load_a(a_reg[3]);
#pragma unroll
            for (int h = 0; h < RB; ++h) load_bh(b_frag[h]);
            store_a(0, a_reg[0], 0, AC);
            load_a(a_reg[0]);                                          // step 4
            store_a(1, a_reg[1], 0, AC);
        }
        // Every request so far (and any register the compiler parked in scratch memory and reloads here) completes
        // before the loop, so that inside it the counts of outstanding loads are exact from the first step on.
        __builtin_amdgcn_s_waitcnt(0x0F70);                            // vmcnt(0)
        __syncthreads();
        frags(0, 0, a_frag[0]);
        auto step = [&](auto u_) {
            constexpr int u = decltype(u_)::value;                     // step number modulo 4
            constexpr int st2 = (u + 2) % 4;
            // first half: fragments of this step's second half, request step +5, multiply, trim half of step +2
            frags(u, 1, a_frag[1]);
            load_a(a_reg[(u + 1) % 4]);
            multiply(a_frag[0], b_frag[(2 * u) % RB]);
            load_bh(b_frag[(2 * u) % RB]);
            store_a(st2, a_reg[st2], 0, AC / 2);
#pragma unroll
            for (int k = 0; k < FM * FN; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, (150 + FM * FN - 1) / (FM * FN), 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            // second half: fragments of the next step's first half, multiply, trim the other half
            frags((u + 1) % 4, 0, a_frag[0]);
            multiply(a_frag[1], b_frag[(2 * u + 1) % RB]);
            load_bh(b_frag[(2 * u + 1) % RB]);
            store_a(st2, a_reg[st2], AC / 2, AC);
#pragma unroll
            for (int k = 0; k < FM * FN; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, (110 + FM * FN - 1) / (FM * FN), 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
        };
        const int nfull = nkb / 4 * 4;
        for (int kb0 = 0; kb0 < nfull; kb0 += 4) {
            step(std::integral_constant<int, 0>{});
            step(std::integral_constant<int, 1>{});
            step(std::integral_constant<int, 2>{});
            step(std::integral_constant<int, 3>{});
        }
        if (nfull < nkb) step(std::integral_constant<int, 0>{});
        if (nfull + 1 < nkb) step(std::integral_constant<int, 1>{});
        if (nfull + 2 < nkb) step(std::integral_constant<int, 2>{});
        } else {
        v4u a_reg[PA][AC];            // activation loads in flight
        v4i b_reg[PB][2][FN];         // weight fragments in flight / in use
        v4i a_frag[2][2][FM];         // activation fragments: [current / next step][half][fragment]

        // ---- prologue ----
        // Activations of step s are requested at step s-1-PA, staged in LDS at s-2, read into
        // fragments at s-1 and multiplied at s; weights of step s are requested at s-PB.
        // Ring slots: activations of step s in a_reg[s % PA], weights in b_reg[s % PB].
        {
            v4u a0[AC], a1[AC];
            load_a(a0);
            load_a(a1);
#pragma unroll
            for (int s = 2; s <= PA; ++s) load_a(a_reg[s % PA]);       // steps 2 .. PA
#pragma unroll
            for (int u = 0; u < PB; ++u) {                             // steps 0 .. PB-1
                load_b(b_reg[u][0], 0);
                load_b(b_reg[u][1], 1);
                advance_b();
            }
            store_a(0, a0, 0, AC);
            store_a(1, a1, 0, AC);
        }
        __syncthreads();
        load_frags(0, a_frag[0]);

        // One reduction step, in two scheduling regions the compiler may not move code
        // across (otherwise it sinks the global loads next to their uses to save registers,
        // which serialises memory latency with the matrix instructions):
        //   first half : fragments of step kb+1 from LDS, request activations of step
        //                kb+1+PA, multiply half 0, request weights of step kb+PB (half 0);
        //   second half: trim and stage the activations of step kb+2, multiply half 1,
        //                request weights of step kb+PB (half 1).
        // The activations are the matrix instruction's row operand, so a lane ends up with
        // one output channel (column l32) of 16 output pixels per fragment.
        auto body = [&](int kb, v4i (&cur)[2][FM], v4i (&nxt)[2][FM], v4u (&a_new)[AC], const v4u (&a_old)[AC],
                        v4i (&br)[2][FN]) {
            const int st = kb % 3;                  // LDS stage of step kb
            const int st1 = st == 2 ? 0 : st + 1;   // ... of step kb+1 (complete since the last barrier)
            const int st2 = st1 == 2 ? 0 : st1 + 1; // ... of step kb+2 (free since the last barrier)
            load_frags(st1, nxt);
            load_a(a_new);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    c[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur[0][i], br[0][j], c[i][j], 0, 0, 0);
            load_b(br[0], 0);
            constexpr int kFirst = Cfg::kSplitTrim ? AC / 2 : 0;
            store_a(st2, a_old, 0, kFirst);
            // issue the fragment reads, the gather's address arithmetic and the weight requests between the
            // matrix instructions rather than in front of them (not for the largest tile: no registers
            // to spare for the longer live ranges)
#pragma unroll
            for (int k = 0; k < (FM * FN * 16 <= 128 ? FM * FN : 0); ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, (2 * FM + FM * FN - 1) / (FM * FN), 0);
                __builtin_amdgcn_sched_group_barrier(0x002, (48 + FM * FN - 1) / (FM * FN), 0);
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            store_a(st2, a_old, kFirst, AC);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    c[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur[1][i], br[1][j], c[i][j], 0, 0, 0);
            load_b(br[1], 1);
            advance_b();
            // the trim arithmetic of this half (about 85 instructions per 16-byte chunk) goes between its
            // matrix instructions as well
#pragma unroll
            for (int k = 0; k < (FM * FN * 16 <= 128 ? FM * FN : 0); ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, (100 * AC + FM * FN - 1) / (FM * FN), 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
        };

        const int nfull = nkb / U * U;
        for (int kb0 = 0; kb0 < nfull; kb0 += U) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                body(kb0 + u, a_frag[u & 1], a_frag[(u & 1) ^ 1], a_reg[(u + 1 + PA) % PA], a_reg[(u + 2) % PA],
                     b_reg[u % PB]);
        }
#pragma unroll
        for (int u = 0; u < U - 1; ++u)
            if (nfull + u < nkb)
                body(nfull + u, a_frag[u & 1], a_frag[(u & 1) ^ 1], a_reg[(u + 1 + PA) % PA], a_reg[(u + 2) % PA],
                     b_reg[u % PB]);

        }   // main loop form

        // ---- epilogue: undo the -128 offset, store int32 and/or dequantised fp32 ----
        // Register v of fragment (i, j) is pixel 8*(v/4) + 4*lhi + v%4, channel l32: each store
        // instruction writes two full 128-byte runs of consecutive channels.  Buffer stores relative
        // to the tile's first row: the lane's part of the offset is computed once, every row adds a
        // uniform multiple of the row pitch, and rows past M or channels past N fall outside the
        // buffer's range and are dropped by the hardware.  One copy per combination of outputs.
        {
            const int64_t left = p.M - m0;
            const int rows = left < Cfg::kTM ? (int)left : Cfg::kTM;
            const float* scale_or_dummy = (p.out || p.out_u8) ? p.scale : reinterpret_cast<const float*>(p.colsum);
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
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    const int n = n0 + wn * Cfg::kWTN + j * 32 + l32;
                    const int nc = n < p.N ? n : 0;
                    // both constants are loaded on every path (a load under a condition makes the
                    // compiler put a full memory wait in front of every store below)
                    int32_t corr;
                    float sc;
                    if constexpr (kEarlyConsts) {
                        corr = corr_t[j];
                        sc = sc_t[j];
                    } else {
                        corr = 128 * p.colsum[nc];
                        sc = scale_or_dummy[(kOut || kU8) ? nc % p.scale_n : nc];
                    }
                    const uint32_t lane_off = n < p.N ? (uint32_t)((wm * Cfg::kWTM + 4 * lhi) * pitch + n * kElem) : kInvalidOffset;
                    asm volatile("" : "+v"(corr), "+v"(sc));
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int row_bytes = (i * 32 + 8 * (v / 4) + (v % 4)) * pitch;
                            const int32_t r = c[i][j][v] + corr;
                            const int off = (int)(lane_off + (uint32_t)row_bytes);
                            if constexpr (kAcc) __builtin_amdgcn_raw_buffer_store_b32(r, arsrc, off, 0, kResultStorePolicy);
                            if constexpr (kOut)
                                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, __fmul_rn((float)r, sc)), orsrc, off, 0, kResultStorePolicy);
                            if constexpr (kU8)
                                __builtin_amdgcn_raw_buffer_store_b8((unsigned char)requant_u8(r, sc), orsrc, off, 0, 0);
                        }
                }
            };
            // Requantised bytes, N a multiple of 4: the four rows a lane holds of one channel are exchanged
            // inside groups of four lanes for four channels of one row: one 32-bit store instead of four byte
            // stores (the byte form is bound by the number of store instructions).
            auto store_tile_u8_packed = [&](auto trim_) __attribute__((always_inline)) {
                constexpr bool kTrimOut = decltype(trim_)::value;   // the next layer's trim applied here, once per result
                const int pitch = p.N;
                const __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(
                    (void*)(p.out_u8 + m0 * p.N), 0, rows * pitch, 0x00020000);
                const QuadSel qs = quad_transpose_selectors(l32);
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    const int n = n0 + wn * Cfg::kWTN + j * 32 + l32;
                    const int nc = n < p.N ? n : 0;
                    int32_t corr;
                    float sc;
                    if constexpr (kEarlyConsts) {
                        corr = corr_t[j];
                        sc = sc_t[j];
                    } else {
                        corr = 128 * p.colsum[nc];
                        sc = p.scale[nc % p.scale_n];
                    }
                    const int n4 = n & ~3;
                    const uint32_t lane_off = n4 < p.N ? (uint32_t)((wm * Cfg::kWTM + 4 * lhi + (l32 & 3)) * pitch + n4) : kInvalidOffset;
                    asm volatile("" : "+v"(corr), "+v"(sc));
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const uint32_t w = requant_u8x4(c[i][j][4 * q] + corr, c[i][j][4 * q + 1] + corr, c[i][j][4 * q + 2] + corr,
                                                            c[i][j][4 * q + 3] + corr, sc);
                            // after the transpose the word holds channels n4 .. n4+3 of one pixel: two pairs
                            uint32_t t = quad_transpose_bytes(w, qs);
                            if constexpr (kTrimOut) t = trim4_kind<KIND>(t, p.luts);
                            __builtin_amdgcn_raw_buffer_store_b32((int)t, orsrc, (int)(lane_off + (uint32_t)((i * 32 + 8 * q) * pitch)), 0, 0);
                        }
                }
            };
            if (Cfg::kByteOutput && p.out_u8) {
                if constexpr (Cfg::kByteOutput) {
                    if ((p.N & 3) == 0) {
                        if (KIND != kTrimNone && p.trim_out) store_tile_u8_packed(std::true_type{});
                        else store_tile_u8_packed(std::false_type{});
                    } else store_tile(std::false_type{}, std::false_type{}, std::true_type{});
                }
            } else if (p.acc && p.out) store_tile(std::true_type{}, std::true_type{}, std::false_type{});
            else if (p.out) store_tile(std::false_type{}, std::true_type{}, std::false_type{});
            else store_tile(std::true_type{}, std::false_type{}, std::false_type{});
        }
    }   // tile loop
}

template <class Cfg, int KIND>
sparq_status launch_cfg(const GemmParams& p, hipStream_t s) {
    static std::atomic<bool> attr_set_dev[kMaxDevices];      // per device; concurrent callers at worst repeat the call
    const int slot = current_device_slot();
    auto kern = conv_gemm_kernel<Cfg, KIND>;
    if (slot == kMaxDevices - 1 || !attr_set_dev[slot].load(std::memory_order_relaxed)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                Cfg::kLdsBytes) != hipSuccess)
            return SPARQ_ELAUNCH;
        attr_set_dev[slot].store(true, std::memory_order_relaxed);
    }
    if (p.out_u8 && !Cfg::kByteOutput) return SPARQ_EUNSUPPORTED;
    GemmParams q = p;
    q.tiles_m = (int)((p.M + Cfg::kTM - 1) / Cfg::kTM);
    q.tiles_n = (p.N + Cfg::kTN - 1) / Cfg::kTN;
    const int64_t tiles = (int64_t)q.tiles_m * q.tiles_n;
    if (tiles > 0x7FFFFFFF) return SPARQ_EUNSUPPORTED;
    const int64_t resident = (int64_t)device_cu_count() * Cfg::kWgPerCu;
    const unsigned blocks = (unsigned)(tiles < resident ? tiles : resident);
    kern<<<blocks, Cfg::kThreads, Cfg::kLdsBytes, s>>>(q);
    return launch_status();
}

template <class Cfg>
sparq_status launch_kind(TrimKind kind, const GemmParams& p, hipStream_t s) {
    switch (kind) {
        case kTrimNone: return launch_cfg<Cfg, kTrimNone>(p, s);
        case kTrimFloor: return launch_cfg<Cfg, kTrimFloor>(p, s);
        case kTrimFloorPair: return launch_cfg<Cfg, kTrimFloorPair>(p, s);
        case kTrimFloorPairWide: return launch_cfg<Cfg, kTrimFloorPairWide>(p, s);
        case kTrimRound: return launch_cfg<Cfg, kTrimRound>(p, s);
        case kTrimRound4: return launch_cfg<Cfg, kTrimRound4>(p, s);
        case kTrimRoundPair4: return launch_cfg<Cfg, kTrimRoundPair4>(p, s);
        default: return launch_cfg<Cfg, kTrimRoundPairWide>(p, s);
    }
}

// One translation unit per tile shape (sparq_conv_gemm_tile*.hip) instantiates the
// kernel for every trim variant and exports a launcher with this signature.
typedef sparq_status (*TileLauncher)(TrimKind, const GemmParams&, hipStream_t);
#define SPARQ_DECLARE_TILE(name) sparq_status name(TrimKind kind, const GemmParams& p, hipStream_t s)
SPARQ_DECLARE_TILE(launch_tile_128x128_w2x2_a4b2);
SPARQ_DECLARE_TILE(launch_tile_128x256_w1x4_a2b3);
SPARQ_DECLARE_TILE(launch_tile_128x512_w1x4_half);

}  // namespace sparq
