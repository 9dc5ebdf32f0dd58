/*
 * SPARQ CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, step-by-step host implementation of the SPARQ activation
 * trim (bSPARQ, Section 3.1; vSPARQ, Section 3.2, Eq. 1-2) followed by the
 * integer dot product of Eq. 1 arranged as a convolution, and the
 * per-output-channel dequantisation and the requantisation to the next
 * layer's unsigned 8-bit activations implied by the quantisation scheme of
 * Section 5.  It exists to check the GPU library and to serve as the timed
 * CPU baseline.  Nothing in the product path may call it, and it shares no
 * code, header, table or helper with the GPU library.
 *
 * All pointers are HOST pointers.  Every function returns 0 on success and a
 * positive code on a rejected argument (1 = invalid argument).
 *
 * Readings of points the paper leaves open:
 *   - rounding by the residual low bits (Section 3.1) is round half up inside
 *     the chosen window;
 *   - the window position is fixed by the leading one of the UNROUNDED value
 *     and a rounding carry out of the window saturates at 2^n - 1;
 *   - the dot-product vector of Eq. 1 is ordered (kh, kw, c) with the input
 *     channel c fastest, so a pair is two consecutive input channels of one
 *     pixel; an odd last channel has an implicit zero partner;
 *   - for n < 4 a value whose partner is zero gets a 2n-bit window (Section
 *     5.1: total window sizes of 6 and 4 bits) whose allowed shifts are the
 *     t for which both t and t+n are allowed n-bit shifts (the two n-bit
 *     multipliers of Eq. 4 acting as the high and low half);
 *   - requantisation rounds to nearest with ties to even, product and
 *     rounding in fp32 (the paper names the quantiser, not its arithmetic).
 *
 * Parity status: the tie direction, the saturate-versus-renormalise choice
 * and the 2n-bit shift set are readings, not printed values -- they are
 * "parity unpinned" against the authors' own code; everything else is pinned
 * by the tests under tests/ (worked examples of Section 3.1, closed forms,
 * an independently written second formulation, brute force, library conv).
 */
#ifndef SPARQ_ORACLE_H
#define SPARQ_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t  window_bits;   /* n = 4, 3, 2; 8 = layer left at plain 8 bits (Section 5, first conv) */
    uint32_t shift_mask;    /* bit t set <=> window [t+n-1 : t] is a placement option              */
    int32_t  round_nearest; /* 0 = plain trim, 1 = "+R"                                            */
    int32_t  pair;          /* 1 = vSPARQ on, 0 = "-vS"                                            */
} sparq_ref_mode;

typedef struct {
    int32_t B, H, W, C;          /* input  NHWC uint8                */
    int32_t N, KH, KW;           /* weight [N][KH][KW][C] int8       */
    int32_t stride_h, stride_w;
    int32_t pad_h, pad_w;
} sparq_ref_conv;

/* 0 if the mode is usable, 1 otherwise. */
int sparq_ref_mode_check(const sparq_ref_mode *mode);

/* Shift set of the 2n-bit window granted to a value whose partner is zero. */
uint32_t sparq_ref_wide_shift_mask(int32_t n, uint32_t shift_mask);

/* bSPARQ on one value: returns the trimmed value q << s; *shift_out (may be
 * NULL) receives s.  x in [0,255], n in [1,8]; S must cover bit 7. */
int sparq_ref_trim_value(int x, int n, uint32_t S, int round_nearest, int *shift_out);

/* vSPARQ + bSPARQ over rows of C contiguous channels. y may alias x. */
int sparq_trim_ref(const uint8_t *x, uint8_t *y, int64_t rows, int32_t C,
                   const sparq_ref_mode *mode);

/* Trimmed convolution by definition.  If row_idx != NULL only the n_rows
 * output rows m = row_idx[i] (m = (b*Ho + oy)*Wo + ox) are computed and
 * stored densely as [n_rows][N]; otherwise all M rows (n_rows ignored).
 * acc (int32) and out (double, = acc * scale[n]) may each be NULL.
 * Returns 2 if an accumulator leaves the int32 range. */
int sparq_conv_gemm_ref(const uint8_t *x, const int8_t *w,
                        const sparq_ref_conv *desc, const sparq_ref_mode *mode,
                        const int64_t *row_idx, int64_t n_rows,
                        int32_t *acc, const float *scale, double *out);

/* out[m][n] = (double)acc[m][n] * (double)scale[n] */
int sparq_dequant_ref(const int32_t *acc, const float *scale, double *out,
                      int64_t M, int32_t N);

/* Requantisation to unsigned 8 bits: y = clamp(rint((float)acc * factor[n]), 0, 255), fp32, ties to even. */
int sparq_requant_ref(const int32_t *acc, const float *factor, uint8_t *y,
                      int64_t M, int32_t N);

/* ---- 2:4 structured weight sparsity (Section 4, sparse tensor core; Section 5.3) ----------------------------
 * Of every four adjacent weights along the input channels two are kept, stored with their coordinates:
 * w_vals [N][KH][KW][C/2] int8 and w_idx [N][KH][KW][C/2], entries 2g and 2g+1 of a tap holding the positions
 * (0..3, ascending, distinct) of the kept weights of group g (channels 4g .. 4g+3).  The coordinates select the
 * activations that are multiplied, and vSPARQ then looks at pairs of the selected activations: the two
 * activations an output channel picks from a group form its vSPARQ pair (a reading: the figure that shows
 * the pairing is not available), so the trim of an activation depends on the output channel's coordinates.
 *   acc[m][n] = sum over taps, groups g of  ta * w_vals[..2g] + tb * w_vals[..2g+1],
 *   (ta, tb) = the pair rule of Eq. 2 on (x[..4g + idx0], x[..4g + idx1])   (each trimmed alone if vSPARQ is off).
 * C must be a multiple of 4.  Returns 1 on bad arguments (also on bad coordinates), 2 on int32 overflow.
 * Parity unpinned against the authors' simulation on the choice of pairs; everything else follows Eq. 1-2. */
int sparq_conv_gemm_sparse24_ref(const uint8_t *x, const int8_t *w_vals, const uint8_t *w_idx,
                                 const sparq_ref_conv *desc, const sparq_ref_mode *mode,
                                 const int64_t *row_idx, int64_t n_rows,
                                 int32_t *acc, const float *scale, double *out);

/* ---- packed storage of trimmed activations (Section 3.1: an n-bit window travels with an identifier of
 * its position; Section 5.1: per 4-bit datum a ShiftCtrl field and, with vSPARQ, a 1-bit MuxCtrl; Section 6:
 * ShiftCtrl may be shared by a number of activations) --------------------------------------------------------
 *
 * What is stored is what the multiplier of Eq. 4 consumes: per pair of channels two n-bit data, each with the
 * shift that puts it back in place (ShiftCtrl = rank of that shift among the allowed ones) and, with vSPARQ, a
 * MuxCtrl bit naming the channel of the pair whose weight it multiplies.  A pair with two non-zero values
 * stores their two windows; a value whose partner is zero stores its 2n-bit window as a high and a low half
 * (shifts t+n and t), both steered to that value's channel.  Decoding a channel is the sum of data << shift
 * over the data steered to it.
 *
 * Layout (a reading: the paper fixes the fields, not their order in memory): a row of C channels is cut into
 * records of 32 channels (the last one zero-filled); a record is three areas of whole little-endian 32-bit
 * words: data (n words; datum k in bits [k*n, k*n+n) of the area), ShiftCtrl (field k in bits [k*sb, k*sb+sb),
 * sb = bits needed to number the allowed shifts; with group = G > 1 one field per G consecutive channels),
 * MuxCtrl (one word, bit k for datum k; absent when vSPARQ is off).  group > 1 is only defined with vSPARQ
 * off: the group's shift is the one bSPARQ picks for its largest value, and every value of the group is
 * trimmed (floor, or round half up saturating) at that shift -- a coarser quantiser than the per-value trim.
 * This grouped form is a reading of a direction the paper leaves to future work: parity unpinned.
 */

/* Bytes of one 32-channel record; 0 if the mode cannot be packed (plain 8 bits, invalid, group not a divisor
 * of 32, group > 1 with vSPARQ on). */
int32_t sparq_ref_packed_record_bytes(const sparq_ref_mode *mode, int32_t group);

/* packed receives rows * ceil(C/32) records holding T(x) (the trim is part of packing). */
int sparq_pack_act_ref(const uint8_t *x, uint8_t *packed, int64_t rows, int32_t C,
                       const sparq_ref_mode *mode, int32_t group);

/* y[r][c] = the value the records encode. */
int sparq_unpack_act_ref(const uint8_t *packed, uint8_t *y, int64_t rows, int32_t C,
                         const sparq_ref_mode *mode, int32_t group);

#ifdef __cplusplus
}
#endif
#endif
