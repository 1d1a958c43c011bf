/*
 * CPU oracle, layer primitives.  TEST INFRASTRUCTURE ONLY (see orc.h).
 *
 * Layout: activations NHWC, conv weights [C_out][kh][kw][C_in], depthwise weights [C][kh][kw].
 * Convolution is cross-correlation with zero padding; H_out = floor((H + 2*pad - k) / stride) + 1.
 */
#include "orc.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

static int fits_i32(int64_t v) { return v >= INT32_MIN && v <= INT32_MAX; }

/* ---------------------------------------------------------------------------------------
 * Convolution as the GEMM of Sec. II-C: output pixel (y,x) is a row of the R x P input
 * matrix, (r,s,c) runs over its P columns, output channel o over the C columns of the
 * weight matrix.  Direct evaluation: the sum over P is written out per output element.
 * ------------------------------------------------------------------------------------- */
int orc_conv_acc_i8_hw(const int8_t* x, int n, int h, int w, int ci, const int8_t* wt, const int32_t* bias,
                       int co, int kh, int kw, int stride, int pad, int pad_w, int32_t* acc)
{
    if (!x || !wt || !acc || n < 0 || h <= 0 || w <= 0 || ci <= 0 || co <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0 || pad_w < 0)
        return ORC_ERR_ARG;
    const int ho = (h + 2 * pad - kh) / stride + 1, wo = (w + 2 * pad_w - kw) / stride + 1;
    if (ho <= 0 || wo <= 0) return ORC_ERR_SHAPE;
    int overflow = 0;
#pragma omp parallel for collapse(2) reduction(| : overflow) schedule(static)
    for (int b = 0; b < n; ++b)
        for (int y = 0; y < ho; ++y)
            for (int xo = 0; xo < wo; ++xo)
                for (int o = 0; o < co; ++o) {
                    int64_t sum = bias ? bias[o] : 0;
                    for (int r = 0; r < kh; ++r) {
                        const int iy = y * stride + r - pad;
                        if (iy < 0 || iy >= h) continue;
                        for (int s = 0; s < kw; ++s) {
                            const int ix = xo * stride + s - pad_w;
                            if (ix < 0 || ix >= w) continue;
                            const int8_t* xp = x + (((int64_t)b * h + iy) * w + ix) * ci;
                            const int8_t* wp = wt + (((int64_t)o * kh + r) * kw + s) * ci;
                            int64_t part = 0;
                            for (int c = 0; c < ci; ++c) part += (int32_t)xp[c] * (int32_t)wp[c];
                            sum += part;
                        }
                    }
                    if (!fits_i32(sum)) overflow = 1;
                    acc[(((int64_t)b * ho + y) * wo + xo) * co + o] = (int32_t)sum;
                }
    return overflow ? ORC_ERR_OVERFLOW : ORC_OK;
}

/* square padding: `pad` rows and `pad` columns on every side */
int orc_conv_acc_i8(const int8_t* x, int n, int h, int w, int ci, const int8_t* wt, const int32_t* bias,
                    int co, int kh, int kw, int stride, int pad, int32_t* acc)
{
    return orc_conv_acc_i8_hw(x, n, h, w, ci, wt, bias, co, kh, kw, stride, pad, pad, acc);
}

/* Second, independent formulation: build the R x P Toeplitz (im2col) matrix of each sample
 * and the P x C weight matrix explicitly, then multiply them with a plain triple loop. */
int orc_conv_acc_i8_toeplitz_hw(const int8_t* x, int n, int h, int w, int ci, const int8_t* wt,
                                const int32_t* bias, int co, int kh, int kw, int stride, int pad, int pad_w, int32_t* acc)
{
    if (!x || !wt || !acc || n < 0) return ORC_ERR_ARG;
    const int ho = (h + 2 * pad - kh) / stride + 1, wo = (w + 2 * pad_w - kw) / stride + 1;
    if (ho <= 0 || wo <= 0) return ORC_ERR_SHAPE;
    const int64_t R = (int64_t)ho * wo, P = (int64_t)kh * kw * ci, C = co;
    int8_t* X = (int8_t*)malloc((size_t)(R * P));
    int8_t* W = (int8_t*)malloc((size_t)(P * C));
    if (!X || !W) { free(X); free(W); return ORC_ERR_ARG; }
    for (int64_t p = 0; p < P; ++p)          /* weight matrix: column o holds filter o, flattened (r,s,c) */
        for (int64_t o = 0; o < C; ++o) W[p * C + o] = wt[o * P + p];
    int overflow = 0;
    for (int b = 0; b < n; ++b) {
        for (int64_t row = 0; row < R; ++row) {
            const int y = (int)(row / wo), xo = (int)(row % wo);
            for (int64_t p = 0; p < P; ++p) {
                const int c = (int)(p % ci), s = (int)((p / ci) % kw), r = (int)(p / ((int64_t)ci * kw));
                const int iy = y * stride + r - pad, ix = xo * stride + s - pad_w;
                X[row * P + p] = (iy < 0 || iy >= h || ix < 0 || ix >= w) ? 0 : x[(((int64_t)b * h + iy) * w + ix) * ci + c];
            }
        }
        for (int64_t row = 0; row < R; ++row)
            for (int64_t o = 0; o < C; ++o) {
                int64_t sum = bias ? bias[o] : 0;
                for (int64_t p = 0; p < P; ++p) sum += (int32_t)X[row * P + p] * (int32_t)W[p * C + o];
                if (!fits_i32(sum)) overflow = 1;
                acc[((int64_t)b * R + row) * C + o] = (int32_t)sum;
            }
    }
    free(X); free(W);
    return overflow ? ORC_ERR_OVERFLOW : ORC_OK;
}

int orc_conv_acc_i8_toeplitz(const int8_t* x, int n, int h, int w, int ci, const int8_t* wt,
                             const int32_t* bias, int co, int kh, int kw, int stride, int pad, int32_t* acc)
{
    return orc_conv_acc_i8_toeplitz_hw(x, n, h, w, ci, wt, bias, co, kh, kw, stride, pad, pad, acc);
}

/* Depthwise: the same sum with output channel == input channel (P = kh*kw). */
int orc_dwconv_acc_i8(const int8_t* x, int n, int h, int w, int c, const int8_t* wt, const int32_t* bias,
                      int kh, int kw, int stride, int pad, int32_t* acc)
{
    if (!x || !wt || !acc || n < 0 || c <= 0 || stride <= 0) return ORC_ERR_ARG;
    const int ho = (h + 2 * pad - kh) / stride + 1, wo = (w + 2 * pad - kw) / stride + 1;
    if (ho <= 0 || wo <= 0) return ORC_ERR_SHAPE;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < n; ++b)
        for (int y = 0; y < ho; ++y)
            for (int xo = 0; xo < wo; ++xo)
                for (int ch = 0; ch < c; ++ch) {
                    int64_t sum = bias ? bias[ch] : 0;
                    for (int r = 0; r < kh; ++r)
                        for (int s = 0; s < kw; ++s) {
                            const int iy = y * stride + r - pad, ix = xo * stride + s - pad;
                            if (iy < 0 || iy >= h || ix < 0 || ix >= w) continue;
                            sum += (int32_t)x[(((int64_t)b * h + iy) * w + ix) * c + ch] * (int32_t)wt[((int64_t)ch * kh + r) * kw + s];
                        }
                    acc[(((int64_t)b * ho + y) * wo + xo) * c + ch] = (int32_t)sum;   /* |sum| <= 9*127*128 + |bias| */
                }
    return ORC_OK;
}

/* Residual add and power-of-two requantisation:
 *   t = acc + (res << res_shift);  q = round-half-up(t / 2^shift) = (t + 2^(shift-1)) >> shift;
 *   y = clamp(q, lo, hi).
 * t and t + 2^(shift-1) must fit int32 (so that an int32 implementation is exact). */
int orc_requant_i8(const int32_t* acc, const int8_t* res, int64_t count, int shift, int res_shift,
                   int lo, int hi, int8_t* y)
{
    if (!acc || !y || count < 0 || shift < 0 || shift > 30 || res_shift < 0 || res_shift > 23 || lo < -128 || hi > 127 || lo > hi)
        return ORC_ERR_ARG;
    int overflow = 0;
    for (int64_t i = 0; i < count; ++i) {
        int64_t t = acc[i];
        if (res) t += (int64_t)res[i] * ((int64_t)1 << res_shift);
        if (shift > 0) t += (int64_t)1 << (shift - 1);
        if (!fits_i32(t)) overflow = 1;
        int64_t q = t >> shift;              /* arithmetic shift: floor division by 2^shift */
        if (q < lo) q = lo;
        if (q > hi) q = hi;
        y[i] = (int8_t)q;
    }
    return overflow ? ORC_ERR_OVERFLOW : ORC_OK;
}

/* Max over the in-range taps only (padding never wins). */
int orc_maxpool_i8(const int8_t* x, int n, int h, int w, int c, int k, int stride, int pad, int8_t* y)
{
    if (!x || !y || n < 0 || k <= 0 || stride <= 0 || pad < 0 || pad >= k) return ORC_ERR_ARG;
    const int ho = (h + 2 * pad - k) / stride + 1, wo = (w + 2 * pad - k) / stride + 1;
    if (ho <= 0 || wo <= 0) return ORC_ERR_SHAPE;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < n; ++b)
        for (int yo = 0; yo < ho; ++yo)
            for (int xo = 0; xo < wo; ++xo)
                for (int ch = 0; ch < c; ++ch) {
                    int best = -129;
                    for (int r = 0; r < k; ++r)
                        for (int s = 0; s < k; ++s) {
                            const int iy = yo * stride + r - pad, ix = xo * stride + s - pad;
                            if (iy < 0 || iy >= h || ix < 0 || ix >= w) continue;
                            const int v = x[(((int64_t)b * h + iy) * w + ix) * c + ch];
                            if (v > best) best = v;
                        }
                    y[(((int64_t)b * ho + yo) * wo + xo) * c + ch] = (int8_t)best;
                }
    return ORC_OK;
}

/* Average pool k x k: the sum over ALL k*k taps with padding counted as zero, divided by k*k and rounded half up
 * (the divisor does not shrink at the border):  y = floor((2 * sum + k*k) / (2 * k*k)). */
int orc_avgpool_i8(const int8_t* x, int n, int h, int w, int c, int k, int stride, int pad, int8_t* y)
{
    if (!x || !y || n < 0 || k <= 0 || k > 15 || stride <= 0 || pad < 0 || pad >= k) return ORC_ERR_ARG;
    const int ho = (h + 2 * pad - k) / stride + 1, wo = (w + 2 * pad - k) / stride + 1;
    if (ho <= 0 || wo <= 0) return ORC_ERR_SHAPE;
    const int64_t kk = (int64_t)k * k;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < n; ++b)
        for (int yo = 0; yo < ho; ++yo)
            for (int xo = 0; xo < wo; ++xo)
                for (int ch = 0; ch < c; ++ch) {
                    int64_t sum = 0;
                    for (int r = 0; r < k; ++r)
                        for (int s = 0; s < k; ++s) {
                            const int iy = yo * stride + r - pad, ix = xo * stride + s - pad;
                            if (iy < 0 || iy >= h || ix < 0 || ix >= w) continue;
                            sum += x[(((int64_t)b * h + iy) * w + ix) * c + ch];
                        }
                    const int64_t num = 2 * sum + kk, den = 2 * kk;          /* floor division, also for negative num */
                    int64_t q = num / den;
                    if (num % den != 0 && num < 0) --q;
                    y[(((int64_t)b * ho + yo) * wo + xo) * c + ch] = (int8_t)q;  /* |q| <= 128 * ... / kk stays in range */
                }
    return ORC_OK;
}

/* Global average pool: S_c = sum over pixels (int32), g_c = clamp(round-half-up(S_c / 2^gap_shift)). */
int orc_gap_i8(const int8_t* x, int n, int h, int w, int c, int gap_shift, int32_t* sums, int8_t* g)
{
    if (!x || !g || n < 0 || gap_shift < 0 || gap_shift > 30) return ORC_ERR_ARG;
    for (int b = 0; b < n; ++b)
        for (int ch = 0; ch < c; ++ch) {
            int64_t s = 0;
            for (int64_t p = 0; p < (int64_t)h * w; ++p) s += x[((int64_t)b * h * w + p) * c + ch];
            if (!fits_i32(s)) return ORC_ERR_OVERFLOW;
            if (sums) sums[(int64_t)b * c + ch] = (int32_t)s;
            int64_t q = gap_shift ? (s + ((int64_t)1 << (gap_shift - 1))) >> gap_shift : s;
            if (q < -128) q = -128;
            if (q > 127) q = 127;
            g[(int64_t)b * c + ch] = (int8_t)q;
        }
    return ORC_OK;
}

/* Fully connected: a_j = b_j + sum_c g_c * W[j][c]. */
int orc_fc_i8(const int8_t* g, int n, int c, const int8_t* wfc, const int32_t* bfc, int n_cls, int32_t* a)
{
    if (!g || !wfc || !a || n < 0) return ORC_ERR_ARG;
    for (int b = 0; b < n; ++b)
        for (int j = 0; j < n_cls; ++j) {
            int64_t s = bfc ? bfc[j] : 0;
            for (int ch = 0; ch < c; ++ch) s += (int32_t)g[(int64_t)b * c + ch] * (int32_t)wfc[(int64_t)j * c + ch];
            if (!fits_i32(s)) return ORC_ERR_OVERFLOW;
            a[(int64_t)b * n_cls + j] = (int32_t)s;
        }
    return ORC_OK;
}

/* 2^30 * 2^(-i/256), i = 0..255, rounded to nearest. */
static uint32_t g_exp2[256];
static int g_exp2_ready = 0;
const uint32_t* orc_exp2_table(void)
{
    if (!g_exp2_ready) {
        for (int i = 0; i < 256; ++i) g_exp2[i] = (uint32_t)llround(ldexp(exp2(-(double)i / 256.0), 30));
        g_exp2_ready = 1;
    }
    return g_exp2;
}

/* Integer softmax top-1 (base-2 softmax of the logits a_j * 2^-frac_bits):
 *   m = max_j a_j, label = lowest j with a_j = m,
 *   d_j = m - a_j,  q_j = d_j >> f,  r_j = the top 8 bits of the fraction of d_j,
 *   e_j = (q_j >= 31) ? 0 : T[r_j] >> q_j,  score S = sum_j e_j   (the arg-max term is exactly 2^30).
 * The confidence is 2^30 / S; a sample exits when S <= S_thr (orc_score_threshold). */
int orc_softmax_top1_i8(const int32_t* a, int n, int n_cls, int frac_bits, int32_t* label, int64_t* score)
{
    if (!a || !label || !score || n < 0 || n_cls <= 0 || frac_bits < 0 || frac_bits > 30) return ORC_ERR_ARG;
    const uint32_t* T = orc_exp2_table();
    for (int b = 0; b < n; ++b) {
        const int32_t* ab = a + (int64_t)b * n_cls;
        int32_t m = ab[0];
        int arg = 0;
        for (int j = 1; j < n_cls; ++j)
            if (ab[j] > m) { m = ab[j]; arg = j; }
        int64_t S = 0;
        for (int j = 0; j < n_cls; ++j) {
            const int64_t d = (int64_t)m - ab[j];
            const int64_t q = d >> frac_bits;
            const int64_t frac = d & (((int64_t)1 << frac_bits) - 1);
            const int64_t r = frac_bits >= 8 ? frac >> (frac_bits - 8) : frac << (8 - frac_bits);
            S += q >= 31 ? 0 : (int64_t)(T[r] >> q);
        }
        label[b] = arg;
        score[b] = S;
    }
    return ORC_OK;
}

/* Threshold on the confidence 2^30/S >= thr, moved to the score: S <= floor(2^30 / thr). */
int64_t orc_score_threshold(float thr)
{
    if (!(thr > 0.0f)) return INT64_MAX;
    if (thr > 1.0f) return 0;
    return (int64_t)floor(1073741824.0 / (double)thr);
}

/* ---------------------------------------------------------------------------------------
 * bf16 path
 * ------------------------------------------------------------------------------------- */
float orc_bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

uint16_t orc_f32_to_bf16(float v)   /* round to nearest, ties to even */
{
    uint32_t u;
    memcpy(&u, &v, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);   /* NaN stays NaN */
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static uint16_t finish_bf16(double accd, float bias, const uint16_t* res, int64_t idx, float lo, float hi)
{
    float v = (float)accd;          /* the one rounding of the accumulator */
    v = v + bias;
    if (res) v = v + orc_bf16_to_f32(res[idx]);
    if (v < lo) v = lo;
    if (v > hi) v = hi;
    return orc_f32_to_bf16(v);
}

int orc_conv_bf16_hw(const uint16_t* x, int n, int h, int w, int ci, const uint16_t* wt, const float* bias,
                     int co, int kh, int kw, int stride, int pad, int pad_w, const uint16_t* res, float f_lo, float f_hi,
                     uint16_t* y)
{
    if (!x || !wt || !y || n < 0 || stride <= 0 || pad < 0 || pad_w < 0) return ORC_ERR_ARG;
    const int ho = (h + 2 * pad - kh) / stride + 1, wo = (w + 2 * pad_w - kw) / stride + 1;
    if (ho <= 0 || wo <= 0) return ORC_ERR_SHAPE;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < n; ++b)
        for (int yo = 0; yo < ho; ++yo)
            for (int xo = 0; xo < wo; ++xo)
                for (int o = 0; o < co; ++o) {
                    double sum = 0.0;
                    for (int r = 0; r < kh; ++r) {
                        const int iy = yo * stride + r - pad;
                        if (iy < 0 || iy >= h) continue;
                        for (int s = 0; s < kw; ++s) {
                            const int ix = xo * stride + s - pad_w;
                            if (ix < 0 || ix >= w) continue;
                            const uint16_t* xp = x + (((int64_t)b * h + iy) * w + ix) * ci;
                            const uint16_t* wp = wt + (((int64_t)o * kh + r) * kw + s) * ci;
                            for (int c = 0; c < ci; ++c) sum += (double)orc_bf16_to_f32(xp[c]) * (double)orc_bf16_to_f32(wp[c]);
                        }
                    }
                    const int64_t idx = (((int64_t)b * ho + yo) * wo + xo) * co + o;
                    y[idx] = finish_bf16(sum, bias ? bias[o] : 0.0f, res, idx, f_lo, f_hi);
                }
    return ORC_OK;
}

int orc_conv_bf16(const uint16_t* x, int n, int h, int w, int ci, const uint16_t* wt, const float* bias,
                  int co, int kh, int kw, int stride, int pad, const uint16_t* res, float f_lo, float f_hi,
                  uint16_t* y)
{
    return orc_conv_bf16_hw(x, n, h, w, ci, wt, bias, co, kh, kw, stride, pad, pad, res, f_lo, f_hi, y);
}

int orc_dwconv_bf16(const uint16_t* x, int n, int h, int w, int c, const uint16_t* wt, const float* bias,
                    int kh, int kw, int stride, int pad, float f_lo, float f_hi, uint16_t* y)
{
    if (!x || !wt || !y || n < 0 || stride <= 0) return ORC_ERR_ARG;
    const int ho = (h + 2 * pad - kh) / stride + 1, wo = (w + 2 * pad - kw) / stride + 1;
    if (ho <= 0 || wo <= 0) return ORC_ERR_SHAPE;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < n; ++b)
        for (int yo = 0; yo < ho; ++yo)
            for (int xo = 0; xo < wo; ++xo)
                for (int ch = 0; ch < c; ++ch) {
                    double sum = 0.0;
                    for (int r = 0; r < kh; ++r)
                        for (int s = 0; s < kw; ++s) {
                            const int iy = yo * stride + r - pad, ix = xo * stride + s - pad;
                            if (iy < 0 || iy >= h || ix < 0 || ix >= w) continue;
                            sum += (double)orc_bf16_to_f32(x[(((int64_t)b * h + iy) * w + ix) * c + ch]) *
                                   (double)orc_bf16_to_f32(wt[((int64_t)ch * kh + r) * kw + s]);
                        }
                    const int64_t idx = (((int64_t)b * ho + yo) * wo + xo) * c + ch;
                    y[idx] = finish_bf16(sum, bias ? bias[ch] : 0.0f, NULL, idx, f_lo, f_hi);
                }
    return ORC_OK;
}

int orc_maxpool_bf16(const uint16_t* x, int n, int h, int w, int c, int k, int stride, int pad, uint16_t* y)
{
    if (!x || !y || n < 0 || k <= 0 || stride <= 0 || pad < 0 || pad >= k) return ORC_ERR_ARG;
    const int ho = (h + 2 * pad - k) / stride + 1, wo = (w + 2 * pad - k) / stride + 1;
    if (ho <= 0 || wo <= 0) return ORC_ERR_SHAPE;
    for (int b = 0; b < n; ++b)
        for (int yo = 0; yo < ho; ++yo)
            for (int xo = 0; xo < wo; ++xo)
                for (int ch = 0; ch < c; ++ch) {
                    int have = 0;
                    float best = 0.0f;
                    uint16_t bits = 0;
                    for (int r = 0; r < k; ++r)
                        for (int s = 0; s < k; ++s) {
                            const int iy = yo * stride + r - pad, ix = xo * stride + s - pad;
                            if (iy < 0 || iy >= h || ix < 0 || ix >= w) continue;
                            const uint16_t vb = x[(((int64_t)b * h + iy) * w + ix) * c + ch];
                            const float v = orc_bf16_to_f32(vb);
                            if (!have || v > best) { best = v; bits = vb; have = 1; }
                        }
                    y[(((int64_t)b * ho + yo) * wo + xo) * c + ch] = bits;
                }
    return ORC_OK;
}

/* Average pool, float path: the taps are added in double (padding contributes zero), divided by k*k, rounded once to
 * float and then to bf16. */
int orc_avgpool_bf16(const uint16_t* x, int n, int h, int w, int c, int k, int stride, int pad, uint16_t* y)
{
    if (!x || !y || n < 0 || k <= 0 || stride <= 0 || pad < 0 || pad >= k) return ORC_ERR_ARG;
    const int ho = (h + 2 * pad - k) / stride + 1, wo = (w + 2 * pad - k) / stride + 1;
    if (ho <= 0 || wo <= 0) return ORC_ERR_SHAPE;
    for (int b = 0; b < n; ++b)
        for (int yo = 0; yo < ho; ++yo)
            for (int xo = 0; xo < wo; ++xo)
                for (int ch = 0; ch < c; ++ch) {
                    double sum = 0.0;
                    for (int r = 0; r < k; ++r)
                        for (int s = 0; s < k; ++s) {
                            const int iy = yo * stride + r - pad, ix = xo * stride + s - pad;
                            if (iy < 0 || iy >= h || ix < 0 || ix >= w) continue;
                            sum += (double)orc_bf16_to_f32(x[(((int64_t)b * h + iy) * w + ix) * c + ch]);
                        }
                    y[(((int64_t)b * ho + yo) * wo + xo) * c + ch] = orc_f32_to_bf16((float)(sum / (double)(k * k)));
                }
    return ORC_OK;
}

/* Exit head, float path: g_c = mean over pixels (float), z_j = logit_scale * (b_j + sum_c g_c W[j][c]),
 * confidence = softmax top-1 = 1 / sum_j exp(z_j - z_max), label = lowest arg-max. */
int orc_head_bf16(const uint16_t* x, int n, int h, int w, int c, const uint16_t* wfc, const float* bfc,
                  int n_cls, float logit_scale, float* logits, int32_t* label, float* conf)
{
    if (!x || !wfc || !label || !conf || n < 0 || n_cls <= 0) return ORC_ERR_ARG;
    float* g = (float*)malloc(sizeof(float) * (size_t)c);
    float* z = (float*)malloc(sizeof(float) * (size_t)n_cls);
    if (!g || !z) { free(g); free(z); return ORC_ERR_ARG; }
    for (int b = 0; b < n; ++b) {
        for (int ch = 0; ch < c; ++ch) {
            double s = 0.0;
            for (int64_t p = 0; p < (int64_t)h * w; ++p) s += (double)orc_bf16_to_f32(x[((int64_t)b * h * w + p) * c + ch]);
            g[ch] = (float)(s / (double)((int64_t)h * w));
        }
        int arg = 0;
        for (int j = 0; j < n_cls; ++j) {
            double s = bfc ? (double)bfc[j] : 0.0;
            for (int ch = 0; ch < c; ++ch) s += (double)g[ch] * (double)orc_bf16_to_f32(wfc[(int64_t)j * c + ch]);
            z[j] = (float)((double)logit_scale * s);
            if (z[j] > z[arg]) arg = j;
        }
        double den = 0.0;
        for (int j = 0; j < n_cls; ++j) den += exp((double)z[j] - (double)z[arg]);
        label[b] = arg;
        conf[b] = (float)(1.0 / den);
        if (logits) memcpy(logits + (int64_t)b * n_cls, z, sizeof(float) * (size_t)n_cls);
    }
    free(g); free(z);
    return ORC_OK;
}
