/*
 * SPARQ CPU oracle -- TEST INFRASTRUCTURE ONLY (see sparq_oracle.h).
 *
 * Written for clarity, one paper step per function, no blocking, no fusion.
 * The only concession to run time is an OpenMP "parallel for" over
 * independent rows.
 */
#include "sparq_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* bSPARQ (Section 3.1)                                                      */
/* ------------------------------------------------------------------------ */

/* Position of the most significant toggled bit of x > 0 (Section 3.1: the
 * window is found by searching for the first most significant toggled bit). */
static int leading_one(int x)
{
    int p = -1;
    while (x > 0) {
        x >>= 1;
        ++p;
    }
    return p;
}

int sparq_ref_trim_value(int x, int n, uint32_t S, int round_nearest, int *shift_out)
{
    int s = 0;
    if (x > 0) {
        const int p = leading_one(x);
        /* Smallest allowed placement whose top bit s+n-1 reaches the leading
         * one.  With every placement allowed this is s = p-n+1, the paper's
         * example 27 -> bits [4:1]; with 3opt the same value gets [5:2] and
         * with 2opt [7:4] (Section 3.1). */
        while (s <= 8 && !(((S >> s) & 1u) && s + n - 1 >= p))
            ++s;
    }
    int q = x >> s;                          /* plain trim: drop the s residual LSBs */
    if (round_nearest && s > 0) {
        q = (x + (1 << (s - 1))) >> s;       /* round half up on the residual LSBs   */
        if (q > (1 << n) - 1)
            q = (1 << n) - 1;                /* carry out of the window saturates    */
    }
    if (shift_out)
        *shift_out = s;
    return q << s;
}

/* ------------------------------------------------------------------------ */
/* mode handling                                                             */
/* ------------------------------------------------------------------------ */

uint32_t sparq_ref_wide_shift_mask(int32_t n, uint32_t shift_mask)
{
    /* A 2n-bit window at shift t is served by the two n-bit multipliers of
     * Eq. 4 as halves at shifts t+n and t, so both must be placement options. */
    uint32_t wide = 0;
    for (int t = 0; t + 2 * n <= 8; ++t)
        if (((shift_mask >> t) & 1u) && ((shift_mask >> (t + n)) & 1u))
            wide |= 1u << t;
    return wide;
}

int sparq_ref_mode_check(const sparq_ref_mode *mode)
{
    if (!mode)
        return 1;
    const int n = mode->window_bits;
    if (n == 8)
        return 0;                            /* plain 8-bit layer, nothing else matters */
    if (n != 2 && n != 3 && n != 4)
        return 1;
    const uint32_t S = mode->shift_mask;
    if (S >> (8 - n + 1))
        return 1;                            /* a window may not stick out above bit 7  */
    if (!(S & 1u) || !((S >> (8 - n)) & 1u))
        return 1;                            /* small values and bit 7 must be coverable */
    if (mode->round_nearest != 0 && mode->round_nearest != 1)
        return 1;
    if (mode->pair != 0 && mode->pair != 1)
        return 1;
    if (mode->pair) {
        const uint32_t S2 = sparq_ref_wide_shift_mask(n, S);
        if (!(S2 & 1u) || !((S2 >> (8 - 2 * n)) & 1u))
            return 1;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* vSPARQ over one channel vector (Section 3.2, Eq. 2)                       */
/* ------------------------------------------------------------------------ */

static void trim_vector(const uint8_t *x, uint8_t *y, int32_t C, const sparq_ref_mode *mode)
{
    const int n = mode->window_bits;
    if (n == 8) {
        memmove(y, x, (size_t)C);
        return;
    }
    const uint32_t S = mode->shift_mask;
    const int R = mode->round_nearest;
    if (!mode->pair) {
        for (int32_t c = 0; c < C; ++c)
            y[c] = (uint8_t)sparq_ref_trim_value(x[c], n, S, R, NULL);
        return;
    }
    const uint32_t S2 = sparq_ref_wide_shift_mask(n, S);
    for (int32_t c = 0; c < C; c += 2) {
        const int a = x[c];
        const int b = (c + 1 < C) ? x[c + 1] : 0;    /* odd tail: implicit zero partner */
        int ta, tb;
        if (a == 0 || b == 0) {
            /* One of the two is zero: the other spans both budgets, 2n bits
             * (n = 4: all eight bits, the value is untouched). */
            ta = sparq_ref_trim_value(a, 2 * n, S2, R, NULL);
            tb = sparq_ref_trim_value(b, 2 * n, S2, R, NULL);
        } else {
            ta = sparq_ref_trim_value(a, n, S, R, NULL);
            tb = sparq_ref_trim_value(b, n, S, R, NULL);
        }
        y[c] = (uint8_t)ta;
        if (c + 1 < C)
            y[c + 1] = (uint8_t)tb;
    }
}

int sparq_trim_ref(const uint8_t *x, uint8_t *y, int64_t rows, int32_t C,
                   const sparq_ref_mode *mode)
{
    if (!x || !y || rows < 0 || C <= 0 || sparq_ref_mode_check(mode))
        return 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        trim_vector(x + r * C, y + r * C, C, mode);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* trimmed convolution (Eq. 1 with the vector ordered kh, kw, c)             */
/* ------------------------------------------------------------------------ */

int sparq_conv_gemm_ref(const uint8_t *x, const int8_t *w,
                        const sparq_ref_conv *d, const sparq_ref_mode *mode,
                        const int64_t *row_idx, int64_t n_rows,
                        int32_t *acc, const float *scale, double *out)
{
    if (!x || !w || !d || sparq_ref_mode_check(mode))
        return 1;
    if (d->B <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->N <= 0 ||
        d->KH <= 0 || d->KW <= 0 || d->stride_h <= 0 || d->stride_w <= 0 ||
        d->pad_h < 0 || d->pad_w < 0)
        return 1;
    if (d->H + 2 * d->pad_h < d->KH || d->W + 2 * d->pad_w < d->KW)
        return 1;
    if (out && !scale)
        return 1;
    const int64_t Ho = (d->H + 2 * d->pad_h - d->KH) / d->stride_h + 1;
    const int64_t Wo = (d->W + 2 * d->pad_w - d->KW) / d->stride_w + 1;
    const int64_t M = (int64_t)d->B * Ho * Wo;
    const int64_t rows = row_idx ? n_rows : M;
    if (row_idx)
        for (int64_t i = 0; i < rows; ++i)
            if (row_idx[i] < 0 || row_idx[i] >= M)
                return 1;

    /* Step 1: trim the input tensor, pixel by pixel along the channels. */
    const int64_t pixels = (int64_t)d->B * d->H * d->W;
    uint8_t *xt = (uint8_t *)malloc((size_t)(pixels * d->C));
    if (!xt)
        return 1;
    sparq_trim_ref(x, xt, pixels, d->C, mode);

    /* Step 2: every output is the integer dot product over its receptive
     * field; positions outside the image contribute zero. */
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (int64_t i = 0; i < rows; ++i) {
        const int64_t m = row_idx ? row_idx[i] : i;
        const int64_t ox = m % Wo;
        const int64_t oy = (m / Wo) % Ho;
        const int64_t b = m / (Wo * Ho);
        for (int32_t n = 0; n < d->N; ++n) {
            int64_t sum = 0;
            for (int32_t kh = 0; kh < d->KH; ++kh) {
                const int64_t iy = oy * d->stride_h - d->pad_h + kh;
                if (iy < 0 || iy >= d->H)
                    continue;
                for (int32_t kw = 0; kw < d->KW; ++kw) {
                    const int64_t ix = ox * d->stride_w - d->pad_w + kw;
                    if (ix < 0 || ix >= d->W)
                        continue;
                    const uint8_t *xp = xt + ((b * d->H + iy) * d->W + ix) * d->C;
                    const int8_t *wp = w + (((int64_t)n * d->KH + kh) * d->KW + kw) * d->C;
                    for (int32_t c = 0; c < d->C; ++c)
                        sum += (int64_t)xp[c] * (int64_t)wp[c];
                }
            }
            if (sum > INT32_MAX || sum < INT32_MIN)
                overflow = 1;
            if (acc)
                acc[i * d->N + n] = (int32_t)sum;
            if (out)
                out[i * d->N + n] = (double)sum * (double)scale[n];
        }
    }
    free(xt);
    return overflow ? 2 : 0;
}

/* ------------------------------------------------------------------------ */
/* 2:4 weight sparsity: activations picked by the weights' coordinates, then */
/* paired (Section 4, sparse tensor core; Section 5.3)                        */
/* ------------------------------------------------------------------------ */

int sparq_conv_gemm_sparse24_ref(const uint8_t *x, const int8_t *w_vals, const uint8_t *w_idx,
                                 const sparq_ref_conv *d, const sparq_ref_mode *mode,
                                 const int64_t *row_idx, int64_t n_rows,
                                 int32_t *acc, const float *scale, double *out)
{
    if (!x || !w_vals || !w_idx || !d || sparq_ref_mode_check(mode))
        return 1;
    if (d->B <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->C % 4 != 0 || d->N <= 0 ||
        d->KH <= 0 || d->KW <= 0 || d->stride_h <= 0 || d->stride_w <= 0 ||
        d->pad_h < 0 || d->pad_w < 0)
        return 1;
    if (d->H + 2 * d->pad_h < d->KH || d->W + 2 * d->pad_w < d->KW)
        return 1;
    if (out && !scale)
        return 1;
    const int64_t half = (int64_t)d->N * d->KH * d->KW * (d->C / 2);
    for (int64_t i = 0; i < half; i += 2)
        if (w_idx[i] > 3 || w_idx[i + 1] > 3 || w_idx[i] >= w_idx[i + 1])
            return 1;                        /* two distinct positions inside the group, smaller first */
    const int64_t Ho = (d->H + 2 * d->pad_h - d->KH) / d->stride_h + 1;
    const int64_t Wo = (d->W + 2 * d->pad_w - d->KW) / d->stride_w + 1;
    const int64_t M = (int64_t)d->B * Ho * Wo;
    const int64_t rows = row_idx ? n_rows : M;
    if (row_idx)
        for (int64_t i = 0; i < rows; ++i)
            if (row_idx[i] < 0 || row_idx[i] >= M)
                return 1;
    const int groups = d->C / 4;
    const sparq_ref_mode pair_mode = *mode;
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (int64_t i = 0; i < rows; ++i) {
        const int64_t m = row_idx ? row_idx[i] : i;
        const int64_t ox = m % Wo;
        const int64_t oy = (m / Wo) % Ho;
        const int64_t b = m / (Wo * Ho);
        for (int32_t n = 0; n < d->N; ++n) {
            int64_t sum = 0;
            for (int32_t kh = 0; kh < d->KH; ++kh) {
                const int64_t iy = oy * d->stride_h - d->pad_h + kh;
                if (iy < 0 || iy >= d->H)
                    continue;                /* outside the image every picked activation is zero */
                for (int32_t kw = 0; kw < d->KW; ++kw) {
                    const int64_t ix = ox * d->stride_w - d->pad_w + kw;
                    if (ix < 0 || ix >= d->W)
                        continue;
                    const uint8_t *xp = x + ((b * d->H + iy) * d->W + ix) * d->C;
                    const int64_t wbase = (((int64_t)n * d->KH + kh) * d->KW + kw) * (d->C / 2);
                    for (int g = 0; g < groups; ++g) {
                        /* the multiplexers of the sparse tensor core: the coordinates pick two of the four */
                        const uint8_t picked[2] = { xp[4 * g + w_idx[wbase + 2 * g]],
                                                    xp[4 * g + w_idx[wbase + 2 * g + 1]] };
                        uint8_t trimmed[2];
                        /* ... and the two picked values are one vSPARQ pair (a vector of two channels) */
                        trim_vector(picked, trimmed, 2, &pair_mode);
                        sum += (int64_t)trimmed[0] * w_vals[wbase + 2 * g] +
                               (int64_t)trimmed[1] * w_vals[wbase + 2 * g + 1];
                    }
                }
            }
            if (sum > INT32_MAX || sum < INT32_MIN)
                overflow = 1;
            if (acc)
                acc[i * d->N + n] = (int32_t)sum;
            if (out)
                out[i * d->N + n] = (double)sum * (double)scale[n];
        }
    }
    return overflow ? 2 : 0;
}

/* ------------------------------------------------------------------------ */
/* dequantisation (Section 5: per-layer activation scale times per-kernel    */
/* weight scale, folded into one factor per output channel)                  */
/* ------------------------------------------------------------------------ */

int sparq_dequant_ref(const int32_t *acc, const float *scale, double *out,
                      int64_t M, int32_t N)
{
    if (!acc || !scale || !out || M < 0 || N <= 0)
        return 1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int32_t n = 0; n < N; ++n)
            out[m * N + n] = (double)acc[m * N + n] * (double)scale[n];
    return 0;
}

/* ------------------------------------------------------------------------ */
/* requantisation to the next layer's activations (Section 5, first          */
/* paragraph: uniform min-max quantisation, symmetric and unsigned per layer */
/* for activations, so a layer's result is scaled, rounded and clamped to    */
/* [0, 255]; factor[n] = input scale * weight scale of kernel n / output     */
/* scale).  The paper does not fix the arithmetic: the product and the       */
/* rounding (to nearest, ties to even) are taken in fp32, and the result is  */
/* defined by exactly that arithmetic.                                        */
/* ------------------------------------------------------------------------ */

int sparq_requant_ref(const int32_t *acc, const float *factor, uint8_t *y,
                      int64_t M, int32_t N)
{
    if (!acc || !factor || !y || M < 0 || N <= 0)
        return 1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int32_t n = 0; n < N; ++n) {
            const float a = (float)acc[m * N + n];   /* int32 -> fp32, round to nearest even     */
            volatile float p = a * factor[n];        /* one fp32 product, not contracted, not kept wider */
            float r = rintf(p);                      /* to nearest integer, ties to even          */
            if (!(r >= 0.0f))
                r = 0.0f;                            /* lower clamp: the unsigned range (the ReLU) */
            if (r > 255.0f)
                r = 255.0f;
            y[m * N + n] = (uint8_t)r;
        }
    return 0;
}


/* ------------------------------------------------------------------------ */
/* packed storage of trimmed activations (Sections 3.1, 5.1, 6; Eq. 4)        */
/* ------------------------------------------------------------------------ */

static int popcount32(uint32_t v)
{
    int c = 0;
    for (; v; v >>= 1)
        c += (int)(v & 1u);
    return c;
}

/* bits needed to number the placement options of S (5 options: 3 bits, 3 options: 2 bits, 2 options: 1 bit) */
static int shift_ctrl_bits(uint32_t S)
{
    const int options = popcount32(S);
    int bits = 0;
    while ((1 << bits) < options)
        ++bits;
    return bits;
}

/* ShiftCtrl code of shift s: its rank among the allowed shifts, smallest first */
static int shift_code(uint32_t S, int s)
{
    return popcount32(S & ((1u << s) - 1u));
}

static int shift_of_code(uint32_t S, int code)
{
    for (int t = 0; t < 8; ++t)
        if ((S >> t) & 1u) {
            if (code == 0)
                return t;
            --code;
        }
    return 0;
}

static void put_bits(uint8_t *area, int pos, int nbits, uint32_t value)
{
    for (int i = 0; i < nbits; ++i, ++pos)
        if ((value >> i) & 1u)
            area[pos >> 3] |= (uint8_t)(1u << (pos & 7));
}

static uint32_t get_bits(const uint8_t *area, int pos, int nbits)
{
    uint32_t v = 0;
    for (int i = 0; i < nbits; ++i, ++pos)
        v |= (uint32_t)((area[pos >> 3] >> (pos & 7)) & 1u) << i;
    return v;
}

static int words_for_bits(int bits)
{
    return (bits + 31) / 32;
}

int32_t sparq_ref_packed_record_bytes(const sparq_ref_mode *mode, int32_t group)
{
    if (sparq_ref_mode_check(mode) || mode->window_bits == 8)
        return 0;
    if (group < 1 || group > 32 || 32 % group != 0 || (group > 1 && mode->pair))
        return 0;
    const int sb = shift_ctrl_bits(mode->shift_mask);
    return 4 * (mode->window_bits + words_for_bits(32 / group * sb) + (mode->pair ? 1 : 0));
}

typedef struct {
    int q, shift, owner;          /* n-bit datum, its shift-left, channel of the pair it is steered to (0 / 1) */
} datum;

/* The two data of a pair (a, b) as the multiplier of Eq. 4 takes them. */
static void encode_pair(int a, int b, const sparq_ref_mode *mode, datum *d0, datum *d1)
{
    const int n = mode->window_bits;
    const uint32_t S = mode->shift_mask;
    const int R = mode->round_nearest;
    int s;
    if (mode->pair && (a == 0 || b == 0)) {
        /* Eq. 2, cases in its order: second value zero -> the first keeps 2n bits; else first value zero -> the
         * second does.  The kept value travels as a high and a low n-bit half steered to the same weight. */
        const int owner = (b == 0) ? 0 : 1;
        const int v = (b == 0) ? a : b;
        const int tv = sparq_ref_trim_value(v, 2 * n, sparq_ref_wide_shift_mask(n, S), R, &s);
        d0->q = (tv >> (s + n)) & ((1 << n) - 1);
        d0->shift = s + n;
        d1->q = (tv >> s) & ((1 << n) - 1);
        d1->shift = s;
        d0->owner = d1->owner = owner;
        return;
    }
    const int ta = sparq_ref_trim_value(a, n, S, R, &s);
    d0->q = ta >> s;
    d0->shift = s;
    d0->owner = 0;
    const int tb = sparq_ref_trim_value(b, n, S, R, &s);
    d1->q = tb >> s;
    d1->shift = s;
    d1->owner = 1;
}

int sparq_pack_act_ref(const uint8_t *x, uint8_t *packed, int64_t rows, int32_t C,
                       const sparq_ref_mode *mode, int32_t group)
{
    const int32_t rec = sparq_ref_packed_record_bytes(mode, group);
    if (!x || !packed || rows < 0 || C <= 0 || rec == 0)
        return 1;
    const int n = mode->window_bits;
    const uint32_t S = mode->shift_mask;
    const int sb = shift_ctrl_bits(S);
    const int32_t nrec = (C + 31) / 32;
    const int shift_words = words_for_bits(32 / group * sb);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const uint8_t *xr = x + r * C;
        for (int32_t k = 0; k < nrec; ++k) {
            uint8_t *data = packed + ((size_t)r * nrec + k) * rec;
            uint8_t *shifts = data + 4 * n;
            uint8_t *mux = shifts + 4 * shift_words;
            memset(data, 0, (size_t)rec);
            int v[32];
            for (int i = 0; i < 32; ++i)
                v[i] = (32 * k + i < C) ? xr[32 * k + i] : 0;     /* channels past C: zeros */
            if (group > 1) {
                /* Section 6: one ShiftCtrl for the whole group -- the placement bSPARQ picks for its largest value */
                for (int g0 = 0; g0 < 32; g0 += group) {
                    int top = 0, s;
                    for (int i = g0; i < g0 + group; ++i)
                        top = v[i] > top ? v[i] : top;
                    sparq_ref_trim_value(top, n, S, 0, &s);
                    put_bits(shifts, (g0 / group) * sb, sb, (uint32_t)shift_code(S, s));
                    for (int i = g0; i < g0 + group; ++i) {
                        int q = v[i] >> s;
                        if (mode->round_nearest && s > 0) {
                            q = (v[i] + (1 << (s - 1))) >> s;
                            if (q > (1 << n) - 1)
                                q = (1 << n) - 1;
                        }
                        put_bits(data, i * n, n, (uint32_t)q);
                    }
                }
                continue;
            }
            for (int i = 0; i < 32; i += 2) {
                datum d0, d1;
                encode_pair(v[i], v[i + 1], mode, &d0, &d1);
                put_bits(data, i * n, n, (uint32_t)d0.q);
                put_bits(data, (i + 1) * n, n, (uint32_t)d1.q);
                put_bits(shifts, i * sb, sb, (uint32_t)shift_code(S, d0.shift));
                put_bits(shifts, (i + 1) * sb, sb, (uint32_t)shift_code(S, d1.shift));
                if (mode->pair) {
                    put_bits(mux, i, 1, (uint32_t)d0.owner);
                    put_bits(mux, i + 1, 1, (uint32_t)d1.owner);
                }
            }
        }
    }
    return 0;
}

int sparq_unpack_act_ref(const uint8_t *packed, uint8_t *y, int64_t rows, int32_t C,
                         const sparq_ref_mode *mode, int32_t group)
{
    const int32_t rec = sparq_ref_packed_record_bytes(mode, group);
    if (!packed || !y || rows < 0 || C <= 0 || rec == 0)
        return 1;
    const int n = mode->window_bits;
    const uint32_t S = mode->shift_mask;
    const int sb = shift_ctrl_bits(S);
    const int32_t nrec = (C + 31) / 32;
    const int shift_words = words_for_bits(32 / group * sb);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        uint8_t *yr = y + r * C;
        for (int32_t k = 0; k < nrec; ++k) {
            const uint8_t *data = packed + ((size_t)r * nrec + k) * rec;
            const uint8_t *shifts = data + 4 * n;
            const uint8_t *mux = shifts + 4 * shift_words;
            int out[32];
            for (int i = 0; i < 32; ++i)
                out[i] = 0;
            for (int i = 0; i < 32; ++i) {
                /* Eq. 4: every datum contributes 2^opt * x to the channel its MuxCtrl names */
                const int q = (int)get_bits(data, i * n, n);
                const int s = shift_of_code(S, (int)get_bits(shifts, (i / group) * sb, sb));
                const int ch = mode->pair ? (i & ~1) + (int)get_bits(mux, i, 1) : i;
                out[ch] += q << s;
            }
            for (int i = 0; i < 32 && 32 * k + i < C; ++i)
                yr[32 * k + i] = (uint8_t)out[i];
        }
    }
    return 0;
}
