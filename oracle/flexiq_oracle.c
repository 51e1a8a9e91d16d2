/*
 * FlexiQ CPU oracle  --  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct C implementation of what the channel-level
 * mixed-precision (4-bit / 8-bit) quantized GEMM and convolution of the FlexiQ
 * paper (arXiv 2510.02822) compute.  It exists so that the HIP library can be
 * checked against something written independently from the paper.  Only the
 * test-suite, the smoke check and the benchmark's cpu_baseline leg may call it;
 * the product path never does.  It shares no code, header, table or helper with
 * the HIP library.
 *
 * Every integer sum is formed in 64-bit integers, in the order the defining
 * formula states; there is no blocking, fusion or reordering.  OpenMP is used
 * only as "for each output row, independently".
 *
 * Parity pins (see tests/test_oracle_*.py): every function below is pinned to
 * something other than itself (the paper's worked examples of Section 4.1,
 * closed forms, exhaustive enumeration, numpy int64 matmul at r=0, brute force
 * with Python integers, permutation invariance).  The round-half-up variant
 * of fq_o_bitlower (mode 1) has no printed value in the paper; it is pinned to
 * floor(x + 1/2) in exact rational arithmetic, exhaustively.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* Uniform symmetric quantisation  (Section 2.1, Eq. 1)                      */
/*   x_q = clip(round(x / S), Qn, Qp),  round = nearest, ties to even.       */
/* The inputs are fp32 and the decision is taken in fp32: x / S is one        */
/* correctly rounded single-precision division, then rounded to an integer.  */
/* ------------------------------------------------------------------------ */

/* S = max|x| / 127 (fp32); an all-zero tensor gets S = 1 so x/S is defined. */
float fq_o_absmax_scale(const float *x, int64_t n)
{
    float amax = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        float a = fabsf(x[i]);
        if (a > amax) amax = a;
    }
    if (amax == 0.0f) return 1.0f;
    return amax / 127.0f;
}

/* Eq. 1 with [Qn, Qp] = [qmin, qmax]. */
void fq_o_quantize(const float *x, int64_t n, float S, int32_t qmin, int32_t qmax, int8_t *q)
{
    for (int64_t i = 0; i < n; ++i) {
        float t = nearbyintf(x[i] / S); /* default rounding mode: ties to even */
        if (t < (float)qmin) t = (float)qmin;
        if (t > (float)qmax) t = (float)qmax;
        q[i] = (int8_t)t;
    }
}

/* Channel-wise (per output channel) weight quantisation: one scale per row
 * of W[N][K]  (Section 4.1, last paragraph; Section 8 settings).            */
void fq_o_quantize_rows(const float *W, int64_t N, int64_t K, float *scale, int8_t *q)
{
    for (int64_t n = 0; n < N; ++n) {
        scale[n] = fq_o_absmax_scale(W + n * K, K);
        fq_o_quantize(W + n * K, K, scale[n], -127, 127, q + n * K);
    }
}

/* ------------------------------------------------------------------------ */
/* Effective-bit extraction  (Section 4.1, Fig. 3)                           */
/* ------------------------------------------------------------------------ */

/* Extraction position for a set of 8-bit values with extremes [vmin, vmax]:
 * the number s of low bits that must be dropped so that the four bits kept
 * still hold the sign, i.e. the smallest s in 0..4 with
 *     -8 * 2^s <= vmin   and   vmax <= 8 * 2^s - 1.
 * (4 - s) is the number of unused high bits below the sign bit.
 * Worked examples of Section 4.1: max < 32 -> two unused bits -> s = 2;
 * min > -16 -> three unused bits -> s = 1.                                  */
int32_t fq_o_shift_for_range(int32_t vmin, int32_t vmax)
{
    for (int32_t s = 0; s < 4; ++s) {
        int32_t lim = 8 * (1 << s);
        if (vmin >= -lim && vmax <= lim - 1) return s;
    }
    return 4;
}

/* The same position found the way Section 4.1 describes the dynamic variant:
 * OR together the magnitude bits of all values (ones' complement for the
 * negative ones), look for the highest set bit p (-1 if none); three more
 * bits below the sign can be kept, so s = max(0, p - 2).                     */
int32_t fq_o_shift_from_values(const int8_t *v, int64_t n, int64_t stride)
{
    uint32_t m = 0;
    for (int64_t i = 0; i < n; ++i) {
        int32_t x = v[i * stride];
        m |= (uint32_t)(x >= 0 ? x : ~x) & 0x7Fu;
    }
    int32_t p = -1;
    for (int32_t b = 6; b >= 0; --b)
        if (m & (1u << b)) { p = b; break; }
    return p - 2 > 0 ? p - 2 : 0;
}

/* floor(q / 2^s) without relying on the sign behaviour of >> */
static int32_t floor_div_pow2(int32_t q, int32_t s)
{
    int32_t d = 1 << s;
    if (q >= 0) return q / d;
    return -((-q + d - 1) / d);
}

/* Bit-lowering of one 8-bit value at extraction position s:
 * drop the s low bits and store the low four bits of what is left
 * (Section 4.1: "shifting and storing low four bits").  Values outside the
 * range the position was chosen for saturate to [-8, 7] (Appendix, saturated
 * channels).  mode 0: truncation (floor), the definition used everywhere;
 * mode 1: round-half-up variant (nearest integer of q / 2^s, ties upwards).  */
int32_t fq_o_bitlower(int32_t q, int32_t s, int32_t mode)
{
    int32_t t;
    if (mode == 1 && s > 0)
        t = floor_div_pow2(q + (1 << (s - 1)), s);
    else
        t = floor_div_pow2(q, s);
    if (t < -8) t = -8;
    if (t > 7) t = 7;
    return t;
}

/* Bit-lower a matrix src[rows][C] into packed 4-bit codes dst[rows][C/2]:
 * the code of channel c sits in byte c/2, low half for even c, high half for
 * odd c, as a two's-complement nibble.  shifts is [rows][G] when per_row is
 * non-zero, else [G], with G = C / group_size.                              */
void fq_o_bitlower_pack(const int8_t *src, uint8_t *dst, int64_t rows, int32_t C, int32_t group_size,
                        const uint8_t *shifts, int32_t per_row, int32_t mode)
{
    int32_t G = C / group_size;
    for (int64_t r = 0; r < rows; ++r)
        for (int32_t c = 0; c < C; c += 2) {
            const uint8_t *sh = per_row ? shifts + r * G : shifts;
            int32_t lo = fq_o_bitlower(src[r * C + c], sh[c / group_size], mode) & 0xF;
            int32_t hi = fq_o_bitlower(src[r * C + c + 1], sh[(c + 1) / group_size], mode) & 0xF;
            dst[r * (C / 2) + c / 2] = (uint8_t)(lo | (hi << 4));
        }
}

/* ------------------------------------------------------------------------ */
/* Channel scores, order, extraction positions (Sections 4.2 and 5)          */
/* ------------------------------------------------------------------------ */

/* Error-estimation score of each input (feature) channel c: the largest
 * weight magnitude of that channel over all output channels and filter taps,
 * times the channel's activation range, both in the 8-bit integer domain
 * (Section 4.2).  Wq is [N][T][C] (T filter taps, 1 for a linear layer);
 * act_range_q[c] is the quantised calibration range of channel c.           */
void fq_o_channel_scores(const int8_t *Wq, int64_t N, int32_t T, int32_t C, const int32_t *act_range_q,
                         int64_t *score)
{
    for (int32_t c = 0; c < C; ++c) {
        int32_t wmax = 0;
        for (int64_t n = 0; n < N; ++n)
            for (int32_t t = 0; t < T; ++t) {
                int32_t w = Wq[(n * T + t) * C + c];
                if (w < 0) w = -w;
                if (w > wmax) wmax = w;
            }
        score[c] = (int64_t)wmax * (int64_t)act_range_q[c];
    }
}

/* Ascending stable order of the scores: perm[j] = original index of the
 * channel stored at position j.  Small scores first, so that any prefix of
 * the order is the greedy low-bitwidth selection and the selections for
 * increasing ratios are nested (Section 4.2, last paragraph; Section 5).
 * Insertion sort: obviously stable, C is a few thousand at most.            */
void fq_o_order_by_score(const int64_t *score, int32_t C, int32_t *perm)
{
    for (int32_t c = 0; c < C; ++c) {
        int32_t j = c;
        while (j > 0 && score[perm[j - 1]] > score[c]) {
            perm[j] = perm[j - 1];
            --j;
        }
        perm[j] = c;
    }
}

/* Quantised calibration range of a channel: the 8-bit code of max|x|. */
int32_t fq_o_range_code(float absmax, float x_scale)
{
    float t = nearbyintf(absmax / x_scale);
    if (t > 127.0f) t = 127.0f;
    if (t < 0.0f) t = 0.0f;
    return (int32_t)t;
}

/* Activation extraction position of each channel group: the position that
 * fits the symmetric range [-a, a], a = largest calibration range code among
 * the group's channels (ranges given in stored, i.e. permuted, order).      */
void fq_o_act_shifts(const int32_t *range_q_perm, int32_t C, int32_t group_size, uint8_t *a_shift)
{
    for (int32_t g = 0; g < C / group_size; ++g) {
        int32_t a = 0;
        for (int32_t j = 0; j < group_size; ++j)
            if (range_q_perm[g * group_size + j] > a) a = range_q_perm[g * group_size + j];
        a_shift[g] = (uint8_t)fq_o_shift_for_range(-a, a);
    }
}

/* Weight extraction position, one per (output channel, channel group), taken
 * over all filter taps of the group (Fig. 4: positions are chosen
 * independently across output channels).  Wq is [N][T][C] in stored order.  */
void fq_o_weight_shifts(const int8_t *Wq, int64_t N, int32_t T, int32_t C, int32_t group_size,
                        uint8_t *w_shift)
{
    int32_t G = C / group_size;
    for (int64_t n = 0; n < N; ++n)
        for (int32_t g = 0; g < G; ++g) {
            int32_t vmin = 0, vmax = 0;
            for (int32_t t = 0; t < T; ++t)
                for (int32_t j = 0; j < group_size; ++j) {
                    int32_t w = Wq[(n * T + t) * C + g * group_size + j];
                    if (w < vmin) vmin = w;
                    if (w > vmax) vmax = w;
                }
            w_shift[n * G + g] = (uint8_t)fq_o_shift_for_range(vmin, vmax);
        }
}

/* Number of 4-bit channel groups for a requested low-bit ratio r: the
 * smallest count whose share of the G groups is at least r (problem
 * statement, Section 2.3: the number of low-bit channels is at least the
 * target ratio).                                                            */
int32_t fq_o_groups_for_ratio(double r, int32_t G)
{
    int32_t g4 = (int32_t)ceil(r * (double)G - 1e-6);
    if (g4 < 0) g4 = 0;
    if (g4 > G) g4 = G;
    return g4;
}

/* ------------------------------------------------------------------------ */
/* Mixed-precision GEMM and convolution (Sections 2.3, 7)                    */
/* ------------------------------------------------------------------------ */

/* acc[m][n] = sum over 4-bit groups g < G4 of
 *                 2^(sa[g] + sw[n][g]) * sum_{k in g} L(X[m][k], sa[g]) * L(W[n][k], sw[n][g])
 *           + sum over the remaining channels k >= G4*gs of X[m][k] * W[n][k]
 * X is [M][K], W is [N][K], both in stored (permuted) channel order; the
 * 4-bit products are shifted back by the two extraction positions before
 * they join the 8-bit sum (Section 7).  group_partial_absmax, if not NULL,
 * receives the largest |sum_{k in g} L*L| seen (the NPU of Section 7 keeps
 * such a partial in 16 bits).  Returns the number of accumulators that do
 * not fit int32 (expected 0).                                               */
int64_t fq_o_mixed_gemm(const int8_t *X, const int8_t *W, int64_t M, int64_t N, int32_t K, int32_t group_size,
                        int32_t G4, const uint8_t *a_shift, const uint8_t *w_shift, int32_t mode,
                        int32_t *acc, int64_t *group_partial_absmax)
{
    int32_t G = K / group_size;
    int64_t overflow = 0, gpmax = 0;
#pragma omp parallel for schedule(static) reduction(+ : overflow) reduction(max : gpmax)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t sum = 0;
            for (int32_t g = 0; g < G4; ++g) {
                int32_t sa = a_shift[g], sw = w_shift[n * G + g];
                int64_t part = 0;
                for (int32_t j = 0; j < group_size; ++j) {
                    int32_t k = g * group_size + j;
                    part += (int64_t)fq_o_bitlower(X[m * K + k], sa, mode) *
                            (int64_t)fq_o_bitlower(W[n * K + k], sw, mode);
                }
                int64_t ap = part < 0 ? -part : part;
                if (ap > gpmax) gpmax = ap;
                sum += part * ((int64_t)1 << (sa + sw));
            }
            for (int32_t k = G4 * group_size; k < K; ++k)
                sum += (int64_t)X[m * K + k] * (int64_t)W[n * K + k];
            if (sum > INT32_MAX || sum < INT32_MIN) ++overflow;
            acc[m * N + n] = (int32_t)sum;
        }
    if (group_partial_absmax) *group_partial_absmax = gpmax;
    return overflow;
}

/* Direct convolution with the same mixed-precision sum: the reduction index
 * is (filter row dy, filter column dx, input channel c); the channel groups,
 * the activation positions a_shift[g] and the 4-bit prefix G4 are the same
 * for every tap, the weight position w_shift[n][g] is shared by the taps.
 * X is NHWC [B][H][Wd][C], Wt is [N][R][S][C], channels in stored order,
 * zero padding (the integer code of real zero under symmetric quantisation).
 * acc is [B][Ho][Wo][N].  Returns the number of int32 overflows (expect 0). */
int64_t fq_o_mixed_conv(const int8_t *X, const int8_t *Wt, int32_t B, int32_t H, int32_t Wd, int32_t C,
                        int64_t N, int32_t R, int32_t S, int32_t stride, int32_t pad, int32_t group_size,
                        int32_t G4, const uint8_t *a_shift, const uint8_t *w_shift, int32_t mode,
                        int32_t *acc)
{
    int32_t G = C / group_size;
    int32_t Ho = (H + 2 * pad - R) / stride + 1;
    int32_t Wo = (Wd + 2 * pad - S) / stride + 1;
    int64_t overflow = 0;
    int64_t rows = (int64_t)B * Ho * Wo;
#pragma omp parallel for schedule(static) reduction(+ : overflow)
    for (int64_t row = 0; row < rows; ++row) {
        int32_t b = (int32_t)(row / ((int64_t)Ho * Wo));
        int32_t ho = (int32_t)((row / Wo) % Ho);
        int32_t wo = (int32_t)(row % Wo);
        for (int64_t n = 0; n < N; ++n) {
            int64_t sum = 0;
            for (int32_t dy = 0; dy < R; ++dy)
                for (int32_t dx = 0; dx < S; ++dx) {
                    int32_t hi = ho * stride + dy - pad;
                    int32_t wi = wo * stride + dx - pad;
                    if (hi < 0 || hi >= H || wi < 0 || wi >= Wd) continue; /* zero padding */
                    const int8_t *x = X + (((int64_t)b * H + hi) * Wd + wi) * C;
                    const int8_t *w = Wt + ((n * R + dy) * S + dx) * C;
                    for (int32_t g = 0; g < G; ++g) {
                        if (g < G4) {
                            int32_t sa = a_shift[g], sw = w_shift[n * G + g];
                            int64_t part = 0;
                            for (int32_t j = 0; j < group_size; ++j)
                                part += (int64_t)fq_o_bitlower(x[g * group_size + j], sa, mode) *
                                        (int64_t)fq_o_bitlower(w[g * group_size + j], sw, mode);
                            sum += part * ((int64_t)1 << (sa + sw));
                        } else {
                            for (int32_t j = 0; j < group_size; ++j)
                                sum += (int64_t)x[g * group_size + j] * (int64_t)w[g * group_size + j];
                        }
                    }
                }
            if (sum > INT32_MAX || sum < INT32_MIN) ++overflow;
            acc[row * N + n] = (int32_t)sum;
        }
    }
    return overflow;
}

/* ------------------------------------------------------------------------ */
/* Epilogue: per-output-channel dequantisation and requantisation            */
/* ------------------------------------------------------------------------ */

/* Dequantised output, the plain definition in double precision:
 *   y[m][n] = acc[m][n] * S_x * S_w[n] + bias[n]                            */
void fq_o_dequant_f64(const int32_t *acc, int64_t M, int64_t N, float x_scale, const float *w_scale,
                      const float *bias, double *y)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            y[m * N + n] = (double)acc[m * N + n] * (double)x_scale * (double)w_scale[n] +
                           (bias ? (double)bias[n] : 0.0);
}

/* Requantised 8-bit output for the next layer: Eq. 1 applied to the
 * dequantised output y with the output scale S_out, the plain definition in
 * double precision (the paper fixes neither precision nor operation order of
 * this step, so the checker is the real-number formula itself):
 *   t[m][n] = (acc[m][n] * S_x * S_w[n] + bias[n]) / S_out
 *   q[m][n] = clip(round_half_even(t), -128, 127)
 * `t_out` (optional) receives t, so that a comparison can tell how close an
 * element lies to a rounding tie.                                            */
void fq_o_requant_i8(const int32_t *acc, int64_t M, int64_t N, float x_scale, const float *w_scale,
                     const float *bias, float out_scale, int8_t *q, double *t_out)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double y = (double)acc[m * N + n] * (double)x_scale * (double)w_scale[n] +
                       (bias ? (double)bias[n] : 0.0);
            double t = y / (double)out_scale;
            double c = nearbyint(t); /* default rounding mode: ties to even */
            if (c < -128.0) c = -128.0;
            if (c > 127.0) c = 127.0;
            q[m * N + n] = (int8_t)c;
            if (t_out) t_out[m * N + n] = t;
        }
}
