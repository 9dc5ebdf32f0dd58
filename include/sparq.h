/*
 * libsparq -- SPARQ activation-trimmed convolution-as-GEMM for AMD MI355X (gfx950).
 *
 * SPARQ (post-training sparsity-aware quantisation) trims already-quantised
 * uint8 activations on the fly:
 *   bSPARQ (Section 3.1)  keeps an n-bit window placed at the leading one,
 *          choosing the smallest allowed shift whose window reaches it,
 *          either dropping the residual LSBs or rounding on them;
 *   vSPARQ (Section 3.2, Eq. 1-2) looks at pairs of consecutive activations
 *          of the dot product: if one is zero the other keeps the whole 2n-bit
 *          budget (all 8 bits for n = 4), otherwise both go through bSPARQ.
 * The trimmed value is q << s, i.e. an ordinary 8-bit integer, so Eq. 1 is
 * evaluated as an int8 x int8 -> int32 contraction on the matrix cores, then
 * dequantised with one fp32 factor per output channel (Section 5: per-layer
 * activation scale times per-kernel weight scale).
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     never allocates, frees or keeps a pointer after the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).  All
 *     entry points only enqueue work on that stream and return immediately.
 *   - Structs passed by pointer are HOST memory, read during the call only.
 *   - Layouts: activations uint8 NHWC [B][H][W][C]; weights int8
 *     [N][KH][KW][C]; outputs row-major [M][N] with M = B*Ho*Wo, row
 *     m = (b*Ho + oy)*Wo + ox; the dot-product index runs (kh, kw, c) with c
 *     fastest, so a vSPARQ pair is two consecutive input channels (2j, 2j+1)
 *     of one pixel; with odd C the last channel has an implicit zero partner.
 *   - Errors are reported by return code only.  Arguments are validated on
 *     the host before anything is enqueued; on an error nothing was launched.
 *   - Calls on different streams and from different threads may overlap.  The
 *     only state the library keeps between calls: the kernel-choice override
 *     of sparq_set_tuning (a test hook, off by default), the per-GPU scratch of
 *     sparq_conv_gemm_static_ws, and small caches of device properties.  The
 *     environment is not read.
 */
#ifndef SPARQ_H
#define SPARQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SPARQ_OK = 0,
    SPARQ_EINVAL = 1,       /* null pointer, bad dimension, bad mode, misaligned buffer */
    SPARQ_EUNSUPPORTED = 2, /* valid but outside what the kernels cover (e.g. tensor >= 2 GiB) */
    SPARQ_EWORKSPACE = 3,   /* workspace / packed buffer smaller than required */
    SPARQ_ELAUNCH = 4       /* the HIP runtime refused a launch */
} sparq_status;

/* How activations are trimmed.
 *   window_bits   n: 4 (the paper's default), 3 or 2 (Section 5.1, Table 4);
 *                 8 = leave the layer at plain 8 bits (the first convolution,
 *                 Section 5) -- the other fields are then ignored.
 *   shift_mask    bit t set <=> the window may sit at bits [t+n-1 : t].
 *                 n = 4: 5opt 0x1F, 3opt 0x15, 2opt 0x11 (Section 3.1);
 *                 n = 3: 6opt 0x3F; n = 2: 7opt 0x7F.  Must contain bit 0 and
 *                 bit 8-n and nothing above; with pair = 1 and n < 4 the set
 *                 {t : t and t+n allowed} of 2n-bit placements must contain 0
 *                 and 8-2n.
 *   round_nearest 0 = plain trim, 1 = round half up on the residual LSBs
 *                 inside the chosen window, saturating at 2^n - 1 ("+R").
 *   pair          1 = vSPARQ on, 0 = every value trimmed on its own ("-vS").
 */
typedef struct {
    int32_t  window_bits;
    uint32_t shift_mask;
    int32_t  round_nearest;
    int32_t  pair;
} sparq_mode;

/* A convolution (dilation 1, groups 1).  Ho = (H + 2*pad_h - KH)/stride_h + 1,
 * Wo likewise.  A plain matrix product A[M][K] * W[N][K]^T is the case
 * B = 1, H = M, W = 1, C = K, KH = KW = 1, stride 1, pad 0. */
typedef struct {
    int32_t B, H, W, C;
    int32_t N, KH, KW;
    int32_t stride_h, stride_w;
    int32_t pad_h, pad_w;
} sparq_conv_desc;

/* Standalone trim (Sections 3.1-3.2): y[r][c] = trimmed x[r][c] for `rows`
 * vectors of C contiguous channels; pairs are (2j, 2j+1) inside one vector.
 * y may alias x exactly (in place); partial overlap is not allowed. */
sparq_status sparq_trim(const uint8_t *x, uint8_t *y, int64_t rows, int32_t C,
                        const sparq_mode *mode, void *stream);

/* Size in bytes of the packed form of the weights of `desc` (0 if desc is invalid). */
size_t sparq_packed_bytes(const sparq_conv_desc *desc);

/* Reorders w [N][KH][KW][C] into the tile order the contraction kernel reads
 * and stores sum_k w[n][k] per output channel (needed because activations
 * enter the signed matrix instruction as x - 128).  Done once per layer; the
 * packed buffer is read-only afterwards.  `packed` must be 256-byte aligned. */
sparq_status sparq_pack_weights(const int8_t *w, const sparq_conv_desc *desc,
                                void *packed, size_t packed_bytes, void *stream);

/* Scratch the convolution may need for this descriptor and mode on the current
 * device: room for a trimmed, channel-padded copy of the input when C is not a
 * multiple of 16.  0 for most layers.  The buffer is overwritten by every call that uses it;
 * calls that share one workspace must not overlap. */
size_t sparq_workspace_bytes(const sparq_conv_desc *desc, const sparq_mode *mode);

/* Which kernel and tiling sparq_conv_gemm would use for this descriptor and mode
 * on the current device, as a short human-readable line (for logs and profiles;
 * the wording is not an interface).  text receives at most text_bytes bytes
 * including the terminator. */
sparq_status sparq_conv_plan(const sparq_conv_desc *desc, const sparq_mode *mode,
                             char *text, size_t text_bytes);

/* Eq. 1 over trimmed activations as an implicit GEMM:
 *   acc[m][n] = sum_{kh,kw,c} T(x)[b, oy*stride_h - pad_h + kh, ox*stride_w - pad_w + kw, c] * w[n][kh][kw][c]
 * (zero outside the image), exact in int32, and optionally
 *   out[m][n] = (float)acc[m][n] * scale[n].
 * At least one of acc / out must be given; out requires scale.  x must be
 * 16-byte aligned, acc/out 16-byte aligned, scale 4-byte aligned, packed_w as produced by
 * sparq_pack_weights for the same desc.  workspace (256-byte aligned, at least
 * sparq_workspace_bytes() bytes) may be NULL when that size is 0; too small a
 * buffer returns SPARQ_EWORKSPACE before anything is launched.  Rejected with SPARQ_EINVAL when K = KH*KW*C
 * is large enough for 255*127*K to leave the int32 range. */
sparq_status sparq_conv_gemm(const uint8_t *x, const void *packed_w,
                             const sparq_conv_desc *desc, const sparq_mode *mode,
                             int32_t *acc, const float *scale, float *out,
                             void *workspace, size_t workspace_bytes, void *stream);

/* sparq_conv_gemm for callers that cannot allocate device memory or carry a
 * workspace around: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments and results as
 * sparq_conv_gemm without the workspace: whatever scratch the layer needs (the
 * channel-padded copy, split-reduction sums) is taken from an array inside the
 * library's device image, SPARQ_STATIC_WORKSPACE_BYTES per GPU, held from the
 * library's first use on that GPU until the process ends.  A layer whose
 * sparq_workspace_bytes() exceeds that size returns SPARQ_EWORKSPACE before
 * anything is launched.  The call allocates and frees nothing (no hipMalloc,
 * no hipFree, no allocating library routine); its first call on a device
 * looks the array's address up once.  All calls on one GPU share the one
 * array: calls that may overlap on a GPU (different streams, different
 * threads) race on it and must be ordered by the caller. */
#define SPARQ_STATIC_WORKSPACE_BYTES (64u << 20)
sparq_status sparq_conv_gemm_static_ws(const uint8_t *x, const void *packed_w,
                                       const sparq_conv_desc *desc, const sparq_mode *mode,
                                       int32_t *acc, const float *scale, float *out,
                                       void *stream);

/* Per-output-channel dequantisation (Section 5): out[m][n] = (float)acc[m][n] * scale[n]. */
sparq_status sparq_dequant(const int32_t *acc, const float *scale, float *out,
                           int64_t M, int32_t N, void *stream);

/* The same convolution with its result requantised to the next layer's
 * unsigned 8-bit activations (Section 5, first paragraph: uniform min-max
 * quantisation, symmetric unsigned per layer for activations, symmetric signed
 * per kernel for weights):
 *   y[m][n] = clamp(round(acc[m][n] * factor[n]), 0, 255),
 *   factor[n] = s_x * s_w[n] / s_y   (input scale, weight scale of kernel n, output scale),
 * so that y is the NHWC uint8 input of the next layer and its lower clamp is
 * the ReLU.  The product and the rounding (to nearest, ties to even) are done
 * in fp32: y is defined by exactly that arithmetic.  Neither acc nor a float
 * tensor is written: one byte leaves per output instead of four.
 * out_mode (NULL or window_bits = 8: none) additionally trims y as the NEXT
 * layer would on loading it, y = T(y) with pairs (2j, 2j+1) of one pixel's N
 * channels (Sections 3.1-3.2), so that the next layer can run with
 * window_bits = 8 and every activation is trimmed once.  This happens inside
 * the convolution's epilogue when out_mode equals mode and N is a multiple of
 * 4, and as one in-place sparq_trim pass over y otherwise; the result is the
 * same.  factor and y (both device memory) must be 16-byte aligned;
 * everything else as for sparq_conv_gemm with acc == NULL, including the
 * workspace. */
sparq_status sparq_conv_gemm_u8(const uint8_t *x, const void *packed_w,
                                const sparq_conv_desc *desc, const sparq_mode *mode,
                                const float *factor, uint8_t *y, const sparq_mode *out_mode,
                                void *workspace, size_t workspace_bytes, void *stream);

/* The requantisation of sparq_conv_gemm_u8 as a pass of its own over int32
 * accumulators: y[m][n] = clamp(round(acc[m][n] * factor[n]), 0, 255), fp32
 * product, ties to even.  Device pointers; M may be 0. */
sparq_status sparq_requant(const int32_t *acc, const float *factor, uint8_t *y,
                           int64_t M, int32_t N, void *stream);

/* ---- Packed storage of trimmed activations -------------------------------
 * What SPARQ's multiplier consumes (Eq. 4) in place of 8-bit values: per pair
 * of channels two n-bit data, each with a ShiftCtrl field (Section 3.1: the
 * identifier of the window position; the rank of the shift among the allowed
 * ones) and, with vSPARQ, a 1-bit MuxCtrl (Section 5.1) naming the channel of
 * the pair whose weight it multiplies.  Two non-zero values store their two
 * windows; a value whose partner is zero (second value zero first, as Eq. 2
 * orders its cases) stores its 2n-bit window as a high half (shift t+n) and a
 * low half (shift t), both steered to that value's channel.
 * Layout: a row of C channels is cut into records of 32 channels (the last
 * zero-filled); a record is, in little-endian 32-bit words: n data words
 * (datum k in bits [k*n, k*n+n)), ceil(F*sb/32) ShiftCtrl words (field f in
 * bits [f*sb, f*sb+sb), sb = bits to number the allowed shifts, F = 32/group),
 * one MuxCtrl word (bit k: datum k goes to the odd channel; absent when
 * mode->pair is 0).  Bits per activation: n + sb/group + pair, i.e. 4+3 for
 * 5opt without vSPARQ, 4+2+1 for 3opt with it (the figures of Sections 3.1
 * and 5.1), 8 for 5opt with vSPARQ.
 * group = 1: per-value ShiftCtrl; unpacking gives exactly sparq_trim(x).
 * group = 2, 4, 8, 16, 32 (mode->pair must be 0): ShiftCtrl shared by that
 * many consecutive channels (Section 6) -- the placement bSPARQ picks for the
 * group's largest value, every value of the group trimmed at it (floor, or
 * round half up saturating): fewer bytes, a coarser quantiser.
 * x, y: [rows][C] uint8; packed: 4-byte aligned, sparq_packed_act_bytes()
 * bytes (0 = this mode / group has no packed form: plain 8 bits, invalid
 * mode, bad group).  Too small a packed buffer returns SPARQ_EWORKSPACE. */
size_t sparq_packed_act_bytes(int64_t rows, int32_t C, const sparq_mode *mode, int32_t group);

/* packed = the records of T(x): the trim is part of packing. */
sparq_status sparq_pack_act(const uint8_t *x, void *packed, size_t packed_bytes,
                            int64_t rows, int32_t C, const sparq_mode *mode,
                            int32_t group, void *stream);

/* y = the 8-bit values the records encode. */
sparq_status sparq_unpack_act(const void *packed, size_t packed_bytes, uint8_t *y,
                              int64_t rows, int32_t C, const sparq_mode *mode,
                              int32_t group, void *stream);

/* sparq_conv_gemm on an input stored in packed form (as written by
 * sparq_pack_act with the same mode and group over rows = B*H*W pixels of C
 * channels): Eq. 1 over the values the records encode.  The records are
 * expanded into the workspace and contracted at plain 8 bits, so workspace
 * must hold sparq_conv_packed_workspace_bytes() bytes (256-byte aligned). */
size_t sparq_conv_packed_workspace_bytes(const sparq_conv_desc *desc, const sparq_mode *mode);
sparq_status sparq_conv_gemm_packed(const void *packed_x, size_t packed_x_bytes, int32_t group,
                                    const void *packed_w, const sparq_conv_desc *desc,
                                    const sparq_mode *mode, int32_t *acc, const float *scale,
                                    float *out, void *workspace, size_t workspace_bytes,
                                    void *stream);

/* ---- 2:4 pruned weights (Section 4, sparse tensor core; Section 5.3) --------
 * Of every four adjacent weights along the input channels two are kept and
 * stored with their coordinates: w_vals int8 [N][KH][KW][C/2] and w_idx uint8
 * [N][KH][KW][C/2], entries 2g and 2g+1 of a tap being the positions (0..3,
 * ascending, distinct -- a precondition, not checked on the device) of the
 * kept weights of group g (channels 4g..4g+3); C must be a multiple of 4.
 * The coordinates pick two of the four activations, and the picked two are
 * that output channel's vSPARQ pair:
 *   acc[m][n] = sum over taps and groups of ta * w_vals[..2g] + tb * w_vals[..2g+1],
 *   (ta, tb) = the pair rule of Eq. 2 on the two picked activations (each
 *   trimmed on its own when mode->pair is 0).
 * MI355X has no datapath that trims after a sparse selection; with vSPARQ on
 * the result is computed exactly over an expanded problem (16 expanded channels
 * per group of four, in which the kept weights are again 2:4 sparse); with it
 * off the problem is the layer itself.  Where the layer's plan is the
 * wave-specialised input-patch kernel the weights go to the sparse matrix
 * instruction as its sparse operand; otherwise the decompressed weights run
 * on the dense path.
 * sparq_sparse24_plan reports which (a text line as from sparq_conv_plan plus
 * "expanded_x4" and "sparse_mfma" / "dense_mfma").
 * packed: 256-byte aligned, sparq_sparse24_packed_bytes() bytes, filled once
 * by sparq_pack_weights_sparse24 for the same desc and mode; workspace:
 * 256-byte aligned, sparq_sparse24_workspace_bytes() bytes.  Everything else
 * as for sparq_conv_gemm (x 16-byte aligned, acc / out / scale). */
size_t sparq_sparse24_packed_bytes(const sparq_conv_desc *desc, const sparq_mode *mode);
sparq_status sparq_pack_weights_sparse24(const int8_t *w_vals, const uint8_t *w_idx,
                                         const sparq_conv_desc *desc, const sparq_mode *mode,
                                         void *packed, size_t packed_bytes, void *stream);
size_t sparq_sparse24_workspace_bytes(const sparq_conv_desc *desc, const sparq_mode *mode);
sparq_status sparq_conv_gemm_sparse24(const uint8_t *x, const void *packed,
                                      const sparq_conv_desc *desc, const sparq_mode *mode,
                                      int32_t *acc, const float *scale, float *out,
                                      void *workspace, size_t workspace_bytes, void *stream);
sparq_status sparq_sparse24_plan(const sparq_conv_desc *desc, const sparq_mode *mode,
                                 char *text, size_t text_bytes);

/* Test and tuning hook: overrides, for the whole process and until changed
 * again, which kernel and tiling the convolution entry points choose (the
 * tests use it to drive every kernel over every shape; results never depend
 * on it).  spec is a comma-separated list of key=value, NULL or "" clears it:
 *   path=gather|patch        one of the two convolution kernels, where eligible
 *   tile=128x128|128x256|128x512   gather kernel tile
 *   patch_tn=64|128|256      input-patch kernel: output channels per tile
 *   patch_ws=0|1             input-patch kernel: plain / wave-specialised form
 * Anything else returns SPARQ_EINVAL and leaves the override as it was.
 * Changing it while convolution calls are in flight on other threads makes
 * those calls pick either setting. */
sparq_status sparq_set_tuning(const char *spec);

/* Static description of a status code. */
const char *sparq_strerror(sparq_status status);

#ifdef __cplusplus
}
#endif
#endif /* SPARQ_H */
