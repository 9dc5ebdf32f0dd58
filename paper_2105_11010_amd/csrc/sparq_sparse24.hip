// 2:4 structured weight sparsity (Section 4, sparse tensor core; Section 5.3): the expansion that makes the
// pair-dependent trim an ordinary contraction, and the operand formats of the dense and the sparse matrix
// instruction for it.
//
// Of every four adjacent weights along the input channels an output channel keeps two, stored with their
// coordinates; the coordinates pick two of the four activations, and the picked two form that output channel's
// vSPARQ pair (Eq. 2).  The trim of an activation therefore depends on WHICH other activation the output channel
// picks with it -- but only through one bit: whether that partner is zero.  With
//     T_i = bSPARQ(x_i)              (partner non-zero)
//     W_i = x_i with 2n bits kept    (partner zero; n = 4: x_i itself)
//     B_i = min(T_i, W_i),
// the value channel n sees is  B_i + F_ij,  F_ij = (x_j == 0 ? W_i : T_i) - B_i >= 0,  j = its partner.  So a
// group of four input channels is expanded into 16 unsigned bytes -- B_0..B_3 and the twelve F_ij (i, then j
// ascending) -- and an output channel's two kept weights are written at the four matching places of a
// 16-byte weight group (w_i at B_i and at F_ij).  The plain-8-bit contraction of the expanded tensors is
// then exactly the sparse, pair-trimmed dot product.  The expanded weights are again 2:4 sparse (two non-zeros in
// 16), so they also go, as kept bytes plus positions, to the sparse matrix instruction (the SP form of the
// input-patch kernel): two instructions' worth of work per kept weight pair instead of four dense ones.
// With vSPARQ off (or a plain 8-bit layer) nothing depends on the partner: the problem is the layer itself.
#include "sparq_common.h"

namespace sparq {

namespace {

constexpr int kSpThreads = 256;

int sp_grid(int64_t items) {
    int64_t blocks = (items + kSpThreads - 1) / kSpThreads;
    if (blocks > 256 * 16) blocks = 256 * 16;
    return (int)(blocks < 1 ? 1 : blocks);
}

// One lane per group of four channels of one pixel: 4 bytes in, 16 bytes out.
__global__ __launch_bounds__(kSpThreads) void expand_act_kernel(const uint32_t* __restrict__ x, uint4* __restrict__ xe,
                                                                 int64_t groups, TrimLuts Ln, TrimLuts Lw, int wide,
                                                                 int round_nearest) {
    const int64_t stride = (int64_t)gridDim.x * kSpThreads;
    for (int64_t i = (int64_t)blockIdx.x * kSpThreads + threadIdx.x; i < groups; i += stride) {
        const uint32_t v = x[i];
        const uint32_t t = trim4_any(v, Ln, round_nearest != 0, false);              // every byte trimmed on its own
        const uint32_t w = wide ? trim4_any(v, Lw, round_nearest != 0, false) : v;   // 2n-bit windows (n < 4) or untouched
        uint32_t T[4], W[4], B[4], Z[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            T[k] = (t >> (8 * k)) & 255u;
            W[k] = (w >> (8 * k)) & 255u;
            B[k] = T[k] < W[k] ? T[k] : W[k];
            Z[k] = ((v >> (8 * k)) & 255u) == 0u;
        }
        uint32_t o[4] = {B[0] | (B[1] << 8) | (B[2] << 16) | (B[3] << 24), 0, 0, 0};
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            int r = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (b == a) continue;
                const uint32_t f = (Z[b] ? W[a] : T[a]) - B[a];
                const int e = 4 + 3 * a + r++;
                o[e >> 2] |= f << (8 * (e & 3));
            }
        }
        xe[i] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

// One lane per (output channel, tap, group): two kept weights and their coordinates -> a dense group.
// EXPAND: 16 bytes (w_i at B_i and at F_ij); otherwise the four bytes of the decompressed group.
template <bool EXPAND>
__global__ __launch_bounds__(kSpThreads) void expand_weights_kernel(const int8_t* __restrict__ vals, const uint8_t* __restrict__ idx,
                                                                     uint32_t* __restrict__ dense, int64_t groups) {
    const int64_t stride = (int64_t)gridDim.x * kSpThreads;
    for (int64_t i = (int64_t)blockIdx.x * kSpThreads + threadIdx.x; i < groups; i += stride) {
        const uint32_t w0 = (uint8_t)vals[2 * i], w1 = (uint8_t)vals[2 * i + 1];
        const int i0 = idx[2 * i] & 3, i1 = idx[2 * i + 1] & 3;                   // (coordinates are a precondition; masked for safety)
        uint32_t o[4] = {0, 0, 0, 0};
        o[0] = (w0 << (8 * i0)) | (w1 << (8 * i1));
        if (EXPAND) {
            const int e0 = 4 + 3 * i0 + (i1 < i0 ? i1 : i1 - 1);                  // F_{i0,i1}: rank of i1 among the others
            const int e1 = 4 + 3 * i1 + (i0 < i1 ? i0 : i0 - 1);
            if (i0 != i1) {
                o[e0 >> 2] |= w0 << (8 * (e0 & 3));
                o[e1 >> 2] |= w1 << (8 * (e1 & 3));
            }
            reinterpret_cast<uint4*>(dense)[i] = make_uint4(o[0], o[1], o[2], o[3]);
        } else {
            dense[i] = o[0];
        }
    }
}

// Operands of the sparse matrix instruction from dense weights w[N][taps][C] that hold at most two non-zeros in
// every aligned group of four channels (the expanded groups above do, and so do decompressed 2:4 weights).
// One lane per (64-index reduction step, half h, output channel n < Np): the 32 weights w[n][step*64 + 32h ..]
// -- taps padded to Cq channels, as in the dense packed tiles -- become 16 kept bytes (two per group of four, in
// position order) and one word of positions (bits [4g+1:4g] and [4g+3:4g+2] for group g, first < second, which
// is the layout v_smfmac_i32_32x32x64_i8 reads from lane (n % 32, h)).  Groups with fewer than two non-zeros keep
// zeros at unused positions.  vals[step][h][Np][16], pos[step][h][Np].
__global__ __launch_bounds__(kSpThreads) void pack_sparse_operand_kernel(const int8_t* __restrict__ w, uint4* __restrict__ vals,
                                                                          uint32_t* __restrict__ pos, int N, int Np, int taps,
                                                                          int C, int Cq, int64_t items) {
    const int64_t stride = (int64_t)gridDim.x * kSpThreads;
    const int steps_tap = Cq / 64;
    for (int64_t it = (int64_t)blockIdx.x * kSpThreads + threadIdx.x; it < items; it += stride) {
        const int n = (int)(it % Np);
        const int64_t sh = it / Np;
        const int h = (int)(sh & 1);
        const int64_t step = sh >> 1;
        const int tap = (int)(step / steps_tap);
        const int c0 = (int)(step % steps_tap) * 64 + 32 * h;
        uint32_t out[4] = {0, 0, 0, 0}, word = 0;
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            const int c = c0 + 4 * g;
            uint32_t v = 0;
            if (n < N && c < C) v = *reinterpret_cast<const uint32_t*>(w + ((int64_t)n * taps + tap) * C + c);   // C % 4 == 0
            int p0 = -1, p1 = -1;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if ((v >> (8 * k)) & 255u) { if (p0 < 0) p0 = k; else if (p1 < 0) p1 = k; }
            if (p0 < 0) { p0 = 0; p1 = 1; }
            else if (p1 < 0) { if (p0 == 3) { p1 = 3; p0 = 2; } else p1 = 3; }
            const uint32_t b0 = (v >> (8 * p0)) & 255u, b1 = (v >> (8 * p1)) & 255u;
            const int e = 2 * g;
            out[e >> 2] |= (b0 << (8 * (e & 3))) | (b1 << (8 * ((e + 1) & 3)));
            word |= (uint32_t)(p0 | (p1 << 2)) << (4 * g);
        }
        vals[it] = make_uint4(out[0], out[1], out[2], out[3]);
        pos[it] = word;
    }
}

}  // namespace

sparq_status launch_sparse24_pack_operand(const int8_t* dense, uint8_t* vals, uint32_t* pos, int N, int Np, int taps, int C,
                                          int Cq, hipStream_t s) {
    const int64_t items = (int64_t)taps * (Cq / 64) * 2 * Np;
    if (items == 0) return SPARQ_OK;
    pack_sparse_operand_kernel<<<sp_grid(items), kSpThreads, 0, s>>>(dense, reinterpret_cast<uint4*>(vals), pos, N, Np, taps, C, Cq, items);
    return launch_status();
}

sparq_status launch_sparse24_expand_act(const uint8_t* x, uint8_t* xe, int64_t pixels, int C, const sparq_mode* mode,
                                        hipStream_t s) {
    const int n = mode->window_bits;
    const int64_t groups = pixels * (C / 4);
    if (groups == 0) return SPARQ_OK;
    const TrimLuts Ln = make_luts(n, mode->shift_mask);
    const bool wide = 2 * n < 8;
    const TrimLuts Lw = wide ? make_luts(2 * n, wide_shift_mask(n, mode->shift_mask)) : Ln;
    expand_act_kernel<<<sp_grid(groups), kSpThreads, 0, s>>>(reinterpret_cast<const uint32_t*>(x), reinterpret_cast<uint4*>(xe),
                                                            groups, Ln, Lw, wide ? 1 : 0, mode->round_nearest);
    return launch_status();
}

sparq_status launch_sparse24_expand_weights(const int8_t* vals, const uint8_t* idx, int8_t* dense, int64_t groups, bool expand,
                                            hipStream_t s) {
    if (groups == 0) return SPARQ_OK;
    if (expand)
        expand_weights_kernel<true><<<sp_grid(groups), kSpThreads, 0, s>>>(vals, idx, reinterpret_cast<uint32_t*>(dense), groups);
    else
        expand_weights_kernel<false><<<sp_grid(groups), kSpThreads, 0, s>>>(vals, idx, reinterpret_cast<uint32_t*>(dense), groups);
    return launch_status();
}

}  // namespace sparq
