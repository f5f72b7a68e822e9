/*
 * CPU oracle: plain definitions in double.  TEST INFRASTRUCTURE ONLY; see
 * oracle.h.  No tiling, no blocking, no reordering of the sums: every output
 * is one ascending-k sum of exact products, then the epilogue.
 * OpenMP only spreads independent outputs over cores.
 */
#include "oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- exact widening of stored bits ------------------------------------ */

static double widen_bf16(uint16_t b)
{
    /* bf16 is the upper half of an IEEE binary32 */
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double widen_f16(uint16_t b)
{
    int sign = (b >> 15) & 1;
    int e = (b >> 10) & 0x1F;
    int m = b & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);                  /* zero and subnormals */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m | 0x400), e - 25);     /* 1.m * 2^(e-15) */
    return sign ? -v : v;
}

/* OCP 8-bit floating point (OFP8 specification): sign, E exponent bits with
 * bias 2^(E-1)-1, M mantissa bits; exponent 0 = subnormal. */
static double widen_fp8_e4m3(uint8_t b)
{
    int sign = b >> 7, e = (b >> 3) & 0xF, m = b & 7;
    double v;
    if (e == 15 && m == 7) v = NAN;                  /* the only non-finite code */
    else if (e == 0) v = ldexp((double)m, -9);       /* m/8 * 2^-6 */
    else v = ldexp((double)(8 + m), e - 10);         /* (1 + m/8) * 2^(e-7) */
    return sign ? -v : v;
}

static double widen_fp8_e5m2(uint8_t b)
{
    int sign = b >> 7, e = (b >> 2) & 0x1F, m = b & 3;
    double v;
    if (e == 31) v = m ? NAN : INFINITY;
    else if (e == 0) v = ldexp((double)m, -16);      /* m/4 * 2^-14 */
    else v = ldexp((double)(4 + m), e - 17);         /* (1 + m/4) * 2^(e-15) */
    return sign ? -v : v;
}

double oracle_widen(uint32_t bits, int dtype)
{
    if (dtype == ORACLE_FP8_E4M3) return widen_fp8_e4m3((uint8_t)bits);
    if (dtype == ORACLE_FP8_E5M2) return widen_fp8_e5m2((uint8_t)bits);
    if (dtype == ORACLE_BF16) return widen_bf16((uint16_t)bits);
    if (dtype == ORACLE_F16) return widen_f16((uint16_t)bits);
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static inline double load(const void* p, int dtype, int64_t idx)
{
    if (dtype == ORACLE_F32) return (double)((const float*)p)[idx];
    if (dtype == ORACLE_BF16) return widen_bf16(((const uint16_t*)p)[idx]);
    if (dtype == ORACLE_F16) return widen_f16(((const uint16_t*)p)[idx]);
    if (dtype == ORACLE_FP8_E4M3) return widen_fp8_e4m3(((const uint8_t*)p)[idx]);
    return widen_fp8_e5m2(((const uint8_t*)p)[idx]);
}

/* ---- rounding to 16-bit formats (for tests of the conversion only) ----- */

/* Round v to a binary format with `prec` significant bits, smallest normal
 * exponent emin (value 2^emin) and overflow threshold 2^emax_plus1. */
static double round_to_format(double v, int prec, int emin, int emax_plus1)
{
    if (isnan(v) || isinf(v) || v == 0.0) return v;
    int e;
    (void)frexp(fabs(v), &e);              /* |v| in [2^(e-1), 2^e) */
    int ulp_exp = e - prec;                /* spacing of the format there */
    int min_ulp_exp = emin - (prec - 1);   /* subnormal spacing */
    if (ulp_exp < min_ulp_exp) ulp_exp = min_ulp_exp;
    double q = ldexp(v, -ulp_exp);         /* exact */
    double r = ldexp(rint(q), ulp_exp);    /* rint: nearest, ties to even */
    if (fabs(r) >= ldexp(1.0, emax_plus1)) return copysign(INFINITY, v);
    return r;
}

uint16_t oracle_round_bf16(double v)
{
    if (isnan(v)) return 0x7FC0;
    double r = round_to_format(v, 8, -126, 128);
    float f = (float)r;                    /* exact: r is a bf16 value */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(u >> 16);
}

uint16_t oracle_round_f16(double v)
{
    if (isnan(v)) return 0x7E00;
    double r = round_to_format(v, 11, -14, 16);
    uint16_t s = signbit(r) ? 0x8000 : 0;
    double a = fabs(r);
    if (isinf(a)) return s | 0x7C00;
    if (a == 0.0) return s;
    if (a < ldexp(1.0, -14))               /* subnormal: a = m * 2^-24 */
        return s | (uint16_t)ldexp(a, 24);
    int e;
    double m = frexp(a, &e);               /* a = m * 2^e, m in [0.5,1) */
    uint16_t mant = (uint16_t)(ldexp(m, 11)) & 0x3FF;   /* 1.xxx -> 10 bits */
    return s | (uint16_t)((e - 1 + 15) << 10) | mant;
}

/* ---- epilogue --------------------------------------------------------- */

double oracle_gelu_tanh(double t)
{
    const double c = 0.7978845608028654;   /* sqrt(2/pi) */
    return 0.5 * t * (1.0 + tanh(c * (t + 0.044715 * t * t * t)));
}

static int epi_has_bias(int epi)
{
    return epi == ORACLE_EPI_BIAS || epi == ORACLE_EPI_BIAS_RELU ||
           epi == ORACLE_EPI_BIAS_GELU_TANH;
}

static double preactivation(double s, double bias, float alpha, int epi)
{
    double t = (double)alpha * s;
    if (epi_has_bias(epi)) t += bias;
    return t;
}

static double activation(double t, int epi)
{
    switch (epi) {
    case ORACLE_EPI_RELU:
    case ORACLE_EPI_BIAS_RELU:
        return isnan(t) ? t : (t > 0.0 ? t : 0.0);
    case ORACLE_EPI_BIAS_GELU_TANH:
    case ORACLE_EPI_GELU_TANH:
        return oracle_gelu_tanh(t);
    default:
        return t;
    }
}

double oracle_epilogue(double s, double bias, float alpha, int epi)
{
    return activation(preactivation(s, bias, alpha, epi), epi);
}

static int check_common(int dtype, int epi, const float* bias)
{
    if (dtype < ORACLE_F32 || dtype > ORACLE_FP8_E5M2) return -1;
    if (epi < ORACLE_EPI_NONE || epi > ORACLE_EPI_GELU_TANH) return -2;
    if (epi_has_bias(epi) && !bias) return -3;
    return 0;
}

/* ---- matmul ------------------------------------------------------------ */

/* one output of one batch entry: sum over k ascending of A[i][k]*B[k][j] */
static double dot_ik_kj(const void* A, const void* B, int dtype, int trans_b,
                        int64_t a_off, int64_t b_off, int64_t lda, int64_t ldb,
                        int64_t i, int64_t j, int64_t K)
{
    double s = 0.0;
    for (int64_t k = 0; k < K; ++k) {
        double a = load(A, dtype, a_off + i * lda + k);
        double b = trans_b ? load(B, dtype, b_off + j * ldb + k)
                           : load(B, dtype, b_off + k * ldb + j);
        s += a * b;
    }
    return s;
}

int oracle_batched_matmul(const void* A, const void* B, const float* bias,
                          double* out, double* preact,
                          int64_t batch, int64_t M, int64_t N, int64_t K,
                          int64_t lda, int64_t ldb, int64_t ldo,
                          int64_t stride_a, int64_t stride_b, int64_t stride_o,
                          int dtype, int trans_b, float alpha, int epi)
{
    int rc = check_common(dtype, epi, bias);
    if (rc) return rc;
    if (batch < 0 || M < 0 || N < 0 || K < 0) return -4;
    if (lda < K || ldo < N || ldb < (trans_b ? K : N)) return -5;
    if (!out || ((!A || !B) && K > 0 && M > 0 && N > 0 && batch > 0)) return -6;

    for (int64_t b = 0; b < batch; ++b) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t i = 0; i < M; ++i) {
            for (int64_t j = 0; j < N; ++j) {
                double s = dot_ik_kj(A, B, dtype, trans_b, b * stride_a, b * stride_b,
                                     lda, ldb, i, j, K);
                double t = preactivation(s, epi_has_bias(epi) ? (double)bias[j] : 0.0,
                                         alpha, epi);
                int64_t o = b * stride_o + i * ldo + j;
                if (preact) preact[o] = t;
                out[o] = activation(t, epi);
            }
        }
    }
    return 0;
}

int oracle_matmul(const void* A, const void* B, const float* bias,
                  double* out, double* preact,
                  int64_t M, int64_t N, int64_t K,
                  int64_t lda, int64_t ldb, int64_t ldo,
                  int dtype, int trans_b, float alpha, int epi)
{
    return oracle_batched_matmul(A, B, bias, out, preact, 1, M, N, K, lda, ldb, ldo,
                                 0, 0, 0, dtype, trans_b, alpha, epi);
}

int oracle_batched_matmul_at(const void* A, const void* B, const float* bias,
                             double* out, double* preact,
                             int64_t batch, int64_t M, int64_t N, int64_t K,
                             int64_t lda, int64_t ldb,
                             int64_t stride_a, int64_t stride_b,
                             int dtype, int trans_b, float alpha, int epi,
                             int64_t nsamp, const int64_t* sb,
                             const int64_t* si, const int64_t* sj)
{
    int rc = check_common(dtype, epi, bias);
    if (rc) return rc;
    if (batch < 1 || M < 1 || N < 1 || K < 0 || nsamp < 0) return -4;
    if (lda < K || ldb < (trans_b ? K : N)) return -5;
    if (!out || !A || !B || !sb || !si || !sj) return -6;
    for (int64_t s = 0; s < nsamp; ++s)
        if (sb[s] < 0 || sb[s] >= batch || si[s] < 0 || si[s] >= M || sj[s] < 0 || sj[s] >= N)
            return -7;

#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t s = 0; s < nsamp; ++s) {
        double acc = dot_ik_kj(A, B, dtype, trans_b, sb[s] * stride_a, sb[s] * stride_b,
                               lda, ldb, si[s], sj[s], K);
        double t = preactivation(acc, epi_has_bias(epi) ? (double)bias[sj[s]] : 0.0,
                                 alpha, epi);
        if (preact) preact[s] = t;
        out[s] = activation(t, epi);
    }
    return 0;
}

/* ---- direct convolution ------------------------------------------------ */

int64_t oracle_conv_out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad, int64_t dil)
{
    if (in < 1 || k < 1 || stride < 1 || pad < 0 || dil < 1) return -1;
    int64_t span = in + 2 * pad - dil * (k - 1) - 1;
    if (span < 0) return -1;
    return span / stride + 1;
}

/* one output pixel/channel: sum over kh, kw, c ascending */
static double conv_point(const void* x, const void* w, int dtype,
                         int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                         int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                         int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                         int64_t n, int64_t oh, int64_t ow, int64_t co)
{
    double s = 0.0;
    for (int64_t kh = 0; kh < KH; ++kh) {
        int64_t ih = oh * stride_h - pad_h + kh * dil_h;
        if (ih < 0 || ih >= H) continue;
        for (int64_t kw = 0; kw < KW; ++kw) {
            int64_t iw = ow * stride_w - pad_w + kw * dil_w;
            if (iw < 0 || iw >= W) continue;
            for (int64_t c = 0; c < Cin; ++c) {
                double xv = load(x, dtype, ((n * H + ih) * W + iw) * Cin + c);
                double wv = load(w, dtype, ((kh * KW + kw) * Cin + c) * Cout + co);
                s += xv * wv;
            }
        }
    }
    return s;
}

int oracle_conv2d_nhwc(const void* x, const void* w, const float* bias,
                       double* out, double* preact,
                       int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                       int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                       int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                       int dtype, float alpha, int epi)
{
    int rc = check_common(dtype, epi, bias);
    if (rc) return rc;
    if (N < 0 || Cin < 1 || Cout < 1) return -4;
    int64_t OH = oracle_conv_out_dim(H, KH, stride_h, pad_h, dil_h);
    int64_t OW = oracle_conv_out_dim(W, KW, stride_w, pad_w, dil_w);
    if (OH < 0 || OW < 0) return -5;
    if (!x || !w || !out) return -6;

    for (int64_t n = 0; n < N; ++n) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t oh = 0; oh < OH; ++oh) {
            for (int64_t ow = 0; ow < OW; ++ow) {
                for (int64_t co = 0; co < Cout; ++co) {
                    double s = conv_point(x, w, dtype, H, W, Cin, Cout, KH, KW,
                                          stride_h, stride_w, pad_h, pad_w, dil_h, dil_w,
                                          n, oh, ow, co);
                    double t = preactivation(s, epi_has_bias(epi) ? (double)bias[co] : 0.0,
                                             alpha, epi);
                    int64_t o = ((n * OH + oh) * OW + ow) * Cout + co;
                    if (preact) preact[o] = t;
                    out[o] = activation(t, epi);
                }
            }
        }
    }
    return 0;
}

int oracle_conv2d_nhwc_at(const void* x, const void* w, const float* bias,
                          double* out, double* preact,
                          int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                          int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                          int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                          int dtype, float alpha, int epi,
                          int64_t nsamp, const int64_t* sn, const int64_t* soh,
                          const int64_t* sow, const int64_t* sco)
{
    int rc = check_common(dtype, epi, bias);
    if (rc) return rc;
    if (N < 1 || Cin < 1 || Cout < 1 || nsamp < 0) return -4;
    int64_t OH = oracle_conv_out_dim(H, KH, stride_h, pad_h, dil_h);
    int64_t OW = oracle_conv_out_dim(W, KW, stride_w, pad_w, dil_w);
    if (OH < 0 || OW < 0) return -5;
    if (!x || !w || !out || !sn || !soh || !sow || !sco) return -6;
    for (int64_t s = 0; s < nsamp; ++s)
        if (sn[s] < 0 || sn[s] >= N || soh[s] < 0 || soh[s] >= OH ||
            sow[s] < 0 || sow[s] >= OW || sco[s] < 0 || sco[s] >= Cout)
            return -7;

#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t s = 0; s < nsamp; ++s) {
        double acc = conv_point(x, w, dtype, H, W, Cin, Cout, KH, KW,
                                stride_h, stride_w, pad_h, pad_w, dil_h, dil_w,
                                sn[s], soh[s], sow[s], sco[s]);
        double t = preactivation(acc, epi_has_bias(epi) ? (double)bias[sco[s]] : 0.0,
                                 alpha, epi);
        if (preact) preact[s] = t;
        out[s] = activation(t, epi);
    }
    return 0;
}

/* ---- convolution with four-sided padding -------------------------------- */

static int64_t conv_out_dim2(int64_t in, int64_t k, int64_t stride, int64_t pad_lo, int64_t pad_hi, int64_t dil)
{
    if (in < 1 || k < 1 || stride < 1 || pad_lo < 0 || pad_hi < 0 || dil < 1) return -1;
    int64_t span = in + pad_lo + pad_hi - dil * (k - 1) - 1;
    if (span < 0) return -1;
    return span / stride + 1;
}

int oracle_conv2d_nhwc_pad4(const void* x, const void* w, const float* bias,
                            double* out, double* preact,
                            int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                            int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                            int64_t pad_top, int64_t pad_bottom, int64_t pad_left, int64_t pad_right,
                            int64_t dil_h, int64_t dil_w,
                            int dtype, float alpha, int epi)
{
    int rc = check_common(dtype, epi, bias);
    if (rc) return rc;
    if (N < 0 || Cin < 1 || Cout < 1) return -4;
    int64_t OH = conv_out_dim2(H, KH, stride_h, pad_top, pad_bottom, dil_h);
    int64_t OW = conv_out_dim2(W, KW, stride_w, pad_left, pad_right, dil_w);
    if (OH < 0 || OW < 0) return -5;
    if (!x || !w || !out) return -6;
    /* the far-side padding only decides how many outputs exist; the near side shifts the taps */
    for (int64_t n = 0; n < N; ++n) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t oh = 0; oh < OH; ++oh) {
            for (int64_t ow = 0; ow < OW; ++ow) {
                for (int64_t co = 0; co < Cout; ++co) {
                    double s = conv_point(x, w, dtype, H, W, Cin, Cout, KH, KW,
                                          stride_h, stride_w, pad_top, pad_left, dil_h, dil_w,
                                          n, oh, ow, co);
                    double t = preactivation(s, epi_has_bias(epi) ? (double)bias[co] : 0.0,
                                             alpha, epi);
                    int64_t o = ((n * OH + oh) * OW + ow) * Cout + co;
                    if (preact) preact[o] = t;
                    out[o] = activation(t, epi);
                }
            }
        }
    }
    return 0;
}

/* ---- transposed convolution ---------------------------------------------- */

int64_t oracle_conv_transpose_out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad,
                                      int64_t out_pad, int64_t dil)
{
    if (in < 1 || k < 1 || stride < 1 || pad < 0 || dil < 1 || out_pad < 0) return -1;
    if (out_pad >= stride && out_pad >= dil) return -1;
    int64_t o = (in - 1) * stride - 2 * pad + dil * (k - 1) + out_pad + 1;
    return o >= 1 ? o : -1;
}

/* The definition: every input pixel scatters its value times the filter into
 * the output, s[n][ih*stride - pad + kh*dil][iw*stride - pad + kw*dil][co] +=
 * x[n][ih][iw][c] * w[kh][kw][c][co]; contributions that land outside the
 * output are dropped.  This is the transpose (adjoint) of the convolution
 * with the same filter, stride, padding and dilation. */
int oracle_conv2d_transpose_nhwc(const void* x, const void* w, const float* bias,
                                 double* out, double* preact,
                                 int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                 int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                 int64_t pad_h, int64_t pad_w, int64_t out_pad_h, int64_t out_pad_w,
                                 int64_t dil_h, int64_t dil_w,
                                 int dtype, float alpha, int epi)
{
    int rc = check_common(dtype, epi, bias);
    if (rc) return rc;
    if (N < 0 || Cin < 1 || Cout < 1) return -4;
    int64_t OH = oracle_conv_transpose_out_dim(H, KH, stride_h, pad_h, out_pad_h, dil_h);
    int64_t OW = oracle_conv_transpose_out_dim(W, KW, stride_w, pad_w, out_pad_w, dil_w);
    if (OH < 0 || OW < 0) return -5;
    if (!x || !w || !out) return -6;
    int64_t per_image = OH * OW * Cout;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t n = 0; n < N; ++n) {
        double* acc = out + n * per_image;
        for (int64_t o = 0; o < per_image; ++o) acc[o] = 0.0;
        for (int64_t ih = 0; ih < H; ++ih)
            for (int64_t iw = 0; iw < W; ++iw)
                for (int64_t kh = 0; kh < KH; ++kh) {
                    int64_t oh = ih * stride_h - pad_h + kh * dil_h;
                    if (oh < 0 || oh >= OH) continue;
                    for (int64_t kw = 0; kw < KW; ++kw) {
                        int64_t ow = iw * stride_w - pad_w + kw * dil_w;
                        if (ow < 0 || ow >= OW) continue;
                        for (int64_t c = 0; c < Cin; ++c) {
                            double xv = load(x, dtype, ((n * H + ih) * W + iw) * Cin + c);
                            for (int64_t co = 0; co < Cout; ++co)
                                acc[(oh * OW + ow) * Cout + co] +=
                                    xv * load(w, dtype, ((kh * KW + kw) * Cin + c) * Cout + co);
                        }
                    }
                }
        for (int64_t o = 0; o < per_image; ++o) {
            double t = preactivation(acc[o], epi_has_bias(epi) ? (double)bias[o % Cout] : 0.0,
                                     alpha, epi);
            if (preact) preact[n * per_image + o] = t;
            acc[o] = activation(t, epi);
        }
    }
    return 0;
}

/* The same sums collected per output element (for sampled checks at sizes the
 * scatter loops would take too long for): output row oh receives tap kh from
 * input row ih exactly when ih*stride - pad + kh*dil == oh. */
int oracle_conv2d_transpose_nhwc_at(const void* x, const void* w, const float* bias,
                                    double* out, double* preact,
                                    int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                    int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                    int64_t pad_h, int64_t pad_w, int64_t out_pad_h, int64_t out_pad_w,
                                    int64_t dil_h, int64_t dil_w,
                                    int dtype, float alpha, int epi,
                                    int64_t nsamp, const int64_t* sn, const int64_t* soh,
                                    const int64_t* sow, const int64_t* sco)
{
    int rc = check_common(dtype, epi, bias);
    if (rc) return rc;
    if (N < 1 || Cin < 1 || Cout < 1 || nsamp < 0) return -4;
    int64_t OH = oracle_conv_transpose_out_dim(H, KH, stride_h, pad_h, out_pad_h, dil_h);
    int64_t OW = oracle_conv_transpose_out_dim(W, KW, stride_w, pad_w, out_pad_w, dil_w);
    if (OH < 0 || OW < 0) return -5;
    if (!x || !w || !out || !sn || !soh || !sow || !sco) return -6;
    for (int64_t s = 0; s < nsamp; ++s)
        if (sn[s] < 0 || sn[s] >= N || soh[s] < 0 || soh[s] >= OH ||
            sow[s] < 0 || sow[s] >= OW || sco[s] < 0 || sco[s] >= Cout)
            return -7;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t s = 0; s < nsamp; ++s) {
        double acc = 0.0;
        for (int64_t ih = 0; ih < H; ++ih)
            for (int64_t kh = 0; kh < KH; ++kh) {
                if (ih * stride_h - pad_h + kh * dil_h != soh[s]) continue;
                for (int64_t iw = 0; iw < W; ++iw)
                    for (int64_t kw = 0; kw < KW; ++kw) {
                        if (iw * stride_w - pad_w + kw * dil_w != sow[s]) continue;
                        for (int64_t c = 0; c < Cin; ++c)
                            acc += load(x, dtype, ((sn[s] * H + ih) * W + iw) * Cin + c) *
                                   load(w, dtype, ((kh * KW + kw) * Cin + c) * Cout + sco[s]);
                    }
            }
        double t = preactivation(acc, epi_has_bias(epi) ? (double)bias[sco[s]] : 0.0, alpha, epi);
        if (preact) preact[s] = t;
        out[s] = activation(t, epi);
    }
    return 0;
}

/* ---- int8 contraction with the quantised epilogue ------------------------ */

/* The epilogue of the paper's fused quantised convolution (appendix on
 * quantisation, figure of the fused de-quantisation / quantisation nest), in
 * the paper's precision: every step is one IEEE binary32 operation, in this
 * order, with no contraction into fused multiply-adds:
 *   t = float(acc) * scale[j]            de-quantise (per output channel)
 *   t = t + bias[j]                      (if bias)
 *   if mid_scale > 0:                    the quantise / de-quantise pair that the
 *       q = clamp(roundeven(t / mid_scale), -128, 127);  t = float(q) * mid_scale
 *   the batch-norm step, in one of two forms:
 *     unfolded, as the figure has it (mean, var, gamma, beta per channel and the scalar eps):
 *       r = 1 / sqrt(var[j] + eps)       three operations: add, square root, reciprocal by division
 *       t = t - mean[j];  t = t * r;  t = t * gamma[j];  t = t + beta[j]
 *     folded by the caller into a multiplier and a shift:
 *       t = t * mul[j]   (if mul);  t = t + add[j]   (if add)
 *   t = (t > 0 or t is NaN) ? t : 0      (if relu: the figure's compare is "unordered or greater")
 *   int8 output:  clamp(roundeven(t / out_scale), -128, 127);  float output: t
 * The accumulator is the exact integer sum. */
typedef struct {
    const float* scale;
    const float* bias;
    float mid_scale;
    const float* mul;
    const float* add;
    int relu;
    float out_scale;
    /* unfolded batch norm (all four arrays, or none) */
    const float* mean;
    const float* var;
    const float* gamma;
    const float* beta;
    float eps;
} quant_epi;

static float quantise_step(float t, float step)
{
    volatile float q = t / step;            /* volatile: one rounding per operation, whatever the optimiser does */
    q = rintf(q);                           /* default rounding mode: nearest, ties to even */
    if (q < -128.0f) q = -128.0f;
    if (q > 127.0f) q = 127.0f;
    return q;
}

static float quant_epilogue(int64_t acc, int64_t j, const quant_epi* e)
{
    volatile float t = (float)(int32_t)acc;
    t = t * e->scale[j];
    if (e->bias) t = t + e->bias[j];
    if (e->mid_scale > 0.0f) {
        volatile float q = quantise_step(t, e->mid_scale);
        t = q * e->mid_scale;
    }
    if (e->mean) {
        volatile float r = e->var[j] + e->eps;
        r = sqrtf(r);                       /* IEEE square root: correctly rounded */
        r = 1.0f / r;
        t = t - e->mean[j];
        t = t * r;
        t = t * e->gamma[j];
        t = t + e->beta[j];
    }
    if (e->mul) t = t * e->mul[j];
    if (e->add) t = t + e->add[j];
    if (e->relu) t = !(t <= 0.0f) ? t : 0.0f;      /* greater than zero, or unordered (NaN stays) */
    return t;
}

static int check_quant(const quant_epi* e, int out_int8)
{
    if (!e->scale) return -3;
    if ((e->mean || e->var || e->gamma || e->beta) && !(e->mean && e->var && e->gamma && e->beta)) return -3;
    if (e->mean && (e->mul || e->add)) return -3;          /* one form of the batch norm at a time */
    if (e->mid_scale < 0.0f || (out_int8 && !(e->out_scale > 0.0f))) return -2;
    return 0;
}

static void store_quant(void* out, int64_t o, float t, const quant_epi* e, int out_int8)
{
    if (out_int8) ((int8_t*)out)[o] = (int8_t)quantise_step(t, e->out_scale);
    else ((float*)out)[o] = t;
}

static int matmul_int8_with(const int8_t* A, const int8_t* B, void* out, int32_t* acc_out,
                            int64_t M, int64_t N, int64_t K,
                            int64_t lda, int64_t ldb, int64_t ldo, int trans_b,
                            quant_epi e, int out_int8)
{
    int rc = check_quant(&e, out_int8);
    if (rc) return rc;
    if (M < 0 || N < 0 || K < 0 || K > 131071) return -4;
    if (lda < K || ldo < N || ldb < (trans_b ? K : N)) return -5;
    if ((M && N) && (!out || (K && (!A || !B)))) return -6;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int64_t)A[i * lda + k] * (int64_t)(trans_b ? B[j * ldb + k] : B[k * ldb + j]);
            if (acc_out) acc_out[i * N + j] = (int32_t)acc;
            store_quant(out, i * ldo + j, quant_epilogue(acc, j, &e), &e, out_int8);
        }
    return 0;
}

int oracle_matmul_int8(const int8_t* A, const int8_t* B, void* out, int32_t* acc_out,
                       int64_t M, int64_t N, int64_t K,
                       int64_t lda, int64_t ldb, int64_t ldo, int trans_b,
                       const float* scale, const float* bias, float mid_scale,
                       const float* mul, const float* add, int relu, float out_scale,
                       int out_int8)
{
    quant_epi e = {scale, bias, mid_scale, mul, add, relu, out_scale, NULL, NULL, NULL, NULL, 0.0f};
    return matmul_int8_with(A, B, out, acc_out, M, N, K, lda, ldb, ldo, trans_b, e, out_int8);
}

int oracle_matmul_int8_bn(const int8_t* A, const int8_t* B, void* out, int32_t* acc_out,
                          int64_t M, int64_t N, int64_t K,
                          int64_t lda, int64_t ldb, int64_t ldo, int trans_b,
                          const float* scale, const float* bias, float mid_scale,
                          const float* mean, const float* var, float eps, const float* gamma, const float* beta,
                          int relu, float out_scale, int out_int8)
{
    if (!mean || !var || !gamma || !beta) return -3;
    quant_epi e = {scale, bias, mid_scale, NULL, NULL, relu, out_scale, mean, var, gamma, beta, eps};
    return matmul_int8_with(A, B, out, acc_out, M, N, K, lda, ldb, ldo, trans_b, e, out_int8);
}

static int conv2d_nhwc_int8_with(const int8_t* x, const int8_t* w, void* out, int32_t* acc_out,
                                 int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                 int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                 int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                                 quant_epi e, int out_int8)
{
    int rc = check_quant(&e, out_int8);
    if (rc) return rc;
    if (N < 0 || Cin < 1 || Cout < 1 || KH * KW * Cin > 131071) return -4;
    int64_t OH = oracle_conv_out_dim(H, KH, stride_h, pad_h, dil_h);
    int64_t OW = oracle_conv_out_dim(W, KW, stride_w, pad_w, dil_w);
    if (OH < 0 || OW < 0) return -5;
    if (!x || !w || !out) return -6;
    for (int64_t n = 0; n < N; ++n) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t oh = 0; oh < OH; ++oh)
            for (int64_t ow = 0; ow < OW; ++ow)
                for (int64_t co = 0; co < Cout; ++co) {
                    int64_t acc = 0;
                    for (int64_t kh = 0; kh < KH; ++kh) {
                        int64_t ih = oh * stride_h - pad_h + kh * dil_h;
                        if (ih < 0 || ih >= H) continue;
                        for (int64_t kw = 0; kw < KW; ++kw) {
                            int64_t iw = ow * stride_w - pad_w + kw * dil_w;
                            if (iw < 0 || iw >= W) continue;
                            for (int64_t c = 0; c < Cin; ++c)
                                acc += (int64_t)x[((n * H + ih) * W + iw) * Cin + c] *
                                       (int64_t)w[((kh * KW + kw) * Cin + c) * Cout + co];
                        }
                    }
                    int64_t o = ((n * OH + oh) * OW + ow) * Cout + co;
                    if (acc_out) acc_out[o] = (int32_t)acc;
                    store_quant(out, o, quant_epilogue(acc, co, &e), &e, out_int8);
                }
    }
    return 0;
}

int oracle_conv2d_nhwc_int8(const int8_t* x, const int8_t* w, void* out, int32_t* acc_out,
                            int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                            int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                            int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                            const float* scale, const float* bias, float mid_scale,
                            const float* mul, const float* add, int relu, float out_scale,
                            int out_int8)
{
    quant_epi e = {scale, bias, mid_scale, mul, add, relu, out_scale, NULL, NULL, NULL, NULL, 0.0f};
    return conv2d_nhwc_int8_with(x, w, out, acc_out, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w,
                                 dil_h, dil_w, e, out_int8);
}

int oracle_conv2d_nhwc_int8_bn(const int8_t* x, const int8_t* w, void* out, int32_t* acc_out,
                               int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                               int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                               int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                               const float* scale, const float* bias, float mid_scale,
                               const float* mean, const float* var, float eps, const float* gamma, const float* beta,
                               int relu, float out_scale, int out_int8)
{
    if (!mean || !var || !gamma || !beta) return -3;
    quant_epi e = {scale, bias, mid_scale, NULL, NULL, relu, out_scale, mean, var, gamma, beta, eps};
    return conv2d_nhwc_int8_with(x, w, out, acc_out, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w,
                                 dil_h, dil_w, e, out_int8);
}

/* ---- residual-add epilogue ------------------------------------------------ */

/* out = act(alpha * (A . B) + bias + beta * R): the shortcut branch of a
 * residual block summed into the contraction's output tile (paper Sec. 4.3:
 * pointwise consumers of the tile, here a binary one, fused into it).
 * R has the output's shape (row stride ldr) and element type r_dtype. */
int oracle_matmul_residual(const void* A, const void* B, const float* bias,
                           const void* R, double* out, double* preact,
                           int64_t M, int64_t N, int64_t K,
                           int64_t lda, int64_t ldb, int64_t ldo, int64_t ldr,
                           int dtype, int r_dtype, int trans_b, float alpha, float beta, int epi)
{
    int rc = check_common(dtype, epi, bias);
    if (rc) return rc;
    if (r_dtype != ORACLE_F32 && r_dtype != ORACLE_BF16 && r_dtype != ORACLE_F16) return -1;
    if (M < 0 || N < 0 || K < 0) return -4;
    if (lda < K || ldo < N || ldr < N || ldb < (trans_b ? K : N)) return -5;
    if (!out || !R || ((!A || !B) && K > 0 && M > 0 && N > 0)) return -6;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double s = dot_ik_kj(A, B, dtype, trans_b, 0, 0, lda, ldb, i, j, K);
            double t = preactivation(s, epi_has_bias(epi) ? (double)bias[j] : 0.0, alpha, epi)
                       + (double)beta * load(R, r_dtype, i * ldr + j);
            if (preact) preact[i * ldo + j] = t;
            out[i * ldo + j] = activation(t, epi);
        }
    }
    return 0;
}

/* Same for the convolution; r is [N][OH][OW][Cout] like the output. */
int oracle_conv2d_nhwc_residual(const void* x, const void* w, const float* bias,
                                const void* r, double* out, double* preact,
                                int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                                int dtype, int r_dtype, float alpha, float beta, int epi)
{
    int rc = check_common(dtype, epi, bias);
    if (rc) return rc;
    if (r_dtype != ORACLE_F32 && r_dtype != ORACLE_BF16 && r_dtype != ORACLE_F16) return -1;
    if (N < 0 || Cin < 1 || Cout < 1) return -4;
    int64_t OH = oracle_conv_out_dim(H, KH, stride_h, pad_h, dil_h);
    int64_t OW = oracle_conv_out_dim(W, KW, stride_w, pad_w, dil_w);
    if (OH < 0 || OW < 0) return -5;
    if (!x || !w || !out || !r) return -6;
    for (int64_t n = 0; n < N; ++n) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t oh = 0; oh < OH; ++oh)
            for (int64_t ow = 0; ow < OW; ++ow)
                for (int64_t co = 0; co < Cout; ++co) {
                    double s = conv_point(x, w, dtype, H, W, Cin, Cout, KH, KW, stride_h, stride_w,
                                          pad_h, pad_w, dil_h, dil_w, n, oh, ow, co);
                    int64_t o = ((n * OH + oh) * OW + ow) * Cout + co;
                    double t = preactivation(s, epi_has_bias(epi) ? (double)bias[co] : 0.0, alpha, epi)
                               + (double)beta * load(r, r_dtype, o);
                    if (preact) preact[o] = t;
                    out[o] = activation(t, epi);
                }
    }
    return 0;
}

/* ---- attention ---------------------------------------------------------- */

/* One output row (b, i) of  softmax(alpha * Q K^T + bias) V,  by the definition:
 * scores s_j, weights p_j = exp(s_j) / sum_l exp(s_l), out[d] = sum_j p_j V[j][d].
 * exp(s_j) is evaluated as exp(s_j - max_l s_l): the quotient is unchanged and
 * nothing overflows.  `scores` is scratch for Nk doubles. */
static void attention_row(const void* Q, const void* K, const void* V, const float* bias,
                          int dtype, int64_t q_off, int64_t k_off, int64_t v_off,
                          int64_t bias_off, int64_t Nk, int64_t D,
                          int64_t ldk, int64_t ldv, float alpha,
                          double* scores, double* out_row)
{
    double top = -INFINITY;
    for (int64_t j = 0; j < Nk; ++j) {
        double dot = 0.0;
        for (int64_t c = 0; c < D; ++c)
            dot += load(Q, dtype, q_off + c) * load(K, dtype, k_off + j * ldk + c);
        double s = (double)alpha * dot;
        if (bias) s += (double)bias[bias_off + j];
        scores[j] = s;
        if (s > top) top = s;
    }
    double denom = 0.0;
    for (int64_t j = 0; j < Nk; ++j) {
        scores[j] = exp(scores[j] - top);
        denom += scores[j];
    }
    for (int64_t d = 0; d < D; ++d) {
        double acc = 0.0;
        for (int64_t j = 0; j < Nk; ++j)
            acc += scores[j] * load(V, dtype, v_off + j * ldv + d);
        out_row[d] = acc / denom;
    }
}

static int check_attention(const void* Q, const void* K, const void* V, const double* out,
                           int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                           int64_t ldq, int64_t ldk, int64_t ldv, int dtype)
{
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F16) return -1;
    if (batch < 1 || Nq < 1 || Nk < 1 || D < 1) return -4;
    if (ldq < D || ldk < D || ldv < D) return -5;
    if (!Q || !K || !V || !out) return -6;
    return 0;
}

int oracle_attention(const void* Q, const void* K, const void* V, const float* bias,
                     double* out,
                     int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                     int64_t ldq, int64_t ldk, int64_t ldv, int64_t ldo,
                     int64_t stride_q, int64_t stride_k, int64_t stride_v, int64_t stride_o,
                     int64_t ld_bias, int64_t stride_bias,
                     int dtype, float alpha)
{
    int rc = check_attention(Q, K, V, out, batch, Nq, Nk, D, ldq, ldk, ldv, dtype);
    if (rc) return rc;
    if (ldo < D || (bias && ld_bias < Nk)) return -5;
    int failed = 0;
#pragma omp parallel
    {
        double* scores = (double*)malloc((size_t)Nk * sizeof(double));
        if (!scores) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 4)
            for (int64_t r = 0; r < batch * Nq; ++r) {
                int64_t b = r / Nq, i = r % Nq;
                attention_row(Q, K, V, bias, dtype, b * stride_q + i * ldq, b * stride_k,
                              b * stride_v, b * stride_bias + i * ld_bias, Nk, D, ldk, ldv,
                              alpha, scores, out + b * stride_o + i * ldo);
            }
        }
        free(scores);
    }
    return failed ? -8 : 0;
}

int oracle_attention_rows(const void* Q, const void* K, const void* V, const float* bias,
                          double* out,
                          int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                          int64_t ldq, int64_t ldk, int64_t ldv,
                          int64_t stride_q, int64_t stride_k, int64_t stride_v,
                          int64_t ld_bias, int64_t stride_bias,
                          int dtype, float alpha,
                          int64_t nsamp, const int64_t* sb, const int64_t* si)
{
    int rc = check_attention(Q, K, V, out, batch, Nq, Nk, D, ldq, ldk, ldv, dtype);
    if (rc) return rc;
    if ((bias && ld_bias < Nk) || nsamp < 0 || !sb || !si) return -5;
    for (int64_t s = 0; s < nsamp; ++s)
        if (sb[s] < 0 || sb[s] >= batch || si[s] < 0 || si[s] >= Nq) return -7;
    int failed = 0;
#pragma omp parallel
    {
        double* scores = (double*)malloc((size_t)Nk * sizeof(double));
        if (!scores) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 1)
            for (int64_t s = 0; s < nsamp; ++s) {
                int64_t b = sb[s], i = si[s];
                attention_row(Q, K, V, bias, dtype, b * stride_q + i * ldq, b * stride_k,
                              b * stride_v, b * stride_bias + i * ld_bias, Nk, D, ldk, ldv,
                              alpha, scores, out + s * D);
            }
        }
        free(scores);
    }
    return failed ? -8 : 0;
}

/* Causal form: row i sees keys 0 .. i + (Nk - Nq) only (the last query sees every key); the
 * definition above restricted to those keys. */
static int64_t causal_keys(int64_t i, int64_t Nq, int64_t Nk)
{
    int64_t n = i + (Nk - Nq) + 1;
    return n < 0 ? 0 : (n > Nk ? Nk : n);
}

int oracle_attention_causal(const void* Q, const void* K, const void* V,
                            double* out,
                            int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                            int64_t ldq, int64_t ldk, int64_t ldv, int64_t ldo,
                            int64_t stride_q, int64_t stride_k, int64_t stride_v, int64_t stride_o,
                            int dtype, float alpha)
{
    int rc = check_attention(Q, K, V, out, batch, Nq, Nk, D, ldq, ldk, ldv, dtype);
    if (rc) return rc;
    if (ldo < D) return -5;
    int failed = 0;
#pragma omp parallel
    {
        double* scores = (double*)malloc((size_t)Nk * sizeof(double));
        if (!scores) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 4)
            for (int64_t r = 0; r < batch * Nq; ++r) {
                int64_t b = r / Nq, i = r % Nq;
                attention_row(Q, K, V, NULL, dtype, b * stride_q + i * ldq, b * stride_k,
                              b * stride_v, 0, causal_keys(i, Nq, Nk), D, ldk, ldv,
                              alpha, scores, out + b * stride_o + i * ldo);
            }
        }
        free(scores);
    }
    return failed ? -8 : 0;
}

int oracle_attention_causal_rows(const void* Q, const void* K, const void* V,
                                 double* out,
                                 int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                                 int64_t ldq, int64_t ldk, int64_t ldv,
                                 int64_t stride_q, int64_t stride_k, int64_t stride_v,
                                 int dtype, float alpha,
                                 int64_t nsamp, const int64_t* sb, const int64_t* si)
{
    int rc = check_attention(Q, K, V, out, batch, Nq, Nk, D, ldq, ldk, ldv, dtype);
    if (rc) return rc;
    if (nsamp < 0 || !sb || !si) return -5;
    for (int64_t s = 0; s < nsamp; ++s)
        if (sb[s] < 0 || sb[s] >= batch || si[s] < 0 || si[s] >= Nq) return -7;
    int failed = 0;
#pragma omp parallel
    {
        double* scores = (double*)malloc((size_t)Nk * sizeof(double));
        if (!scores) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 1)
            for (int64_t s = 0; s < nsamp; ++s) {
                int64_t b = sb[s], i = si[s];
                attention_row(Q, K, V, NULL, dtype, b * stride_q + i * ldq, b * stride_k,
                              b * stride_v, 0, causal_keys(i, Nq, Nk), D, ldk, ldv,
                              alpha, scores, out + s * D);
            }
        }
        free(scores);
    }
    return failed ? -8 : 0;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
