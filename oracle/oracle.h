/*
 * CPU oracle for the fused dense contraction  out = act(alpha * (A . B) + bias)
 * and for the attention layer  softmax(alpha * Q K^T + bias) V.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain mathematical definition written
 * out in IEEE double: a triple loop for matmul, a seven-deep loop nest for the
 * direct convolution, the epilogue in double, results returned unrounded.  It
 * shares no code with the HIP library and must never be called from it; only
 * tests, the smoke check and the bench's CPU-baseline leg use it.
 *
 * Operator semantics follow the paper: convolution as LHS.RHS with the index
 * map of the "convolution lowered as a 3-d matmul nest" figure (Sec. 4.5),
 * 16-bit inputs extended before the multiply (Sec. 5, evaluation setup), the
 * pointwise tail fused on the output tile (Sec. 4.3).  Accumulation is fp64
 * here (the paper's generated code accumulates in fp32).
 *
 * All pointers are host pointers.  16-bit inputs are raw bit patterns
 * (uint16_t) and 8-bit inputs raw bytes (uint8_t), widened exactly.  Every function returns 0 on success and a
 * negative value on an invalid argument.
 */
#ifndef PBK_ORACLE_H
#define PBK_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element types of A, B, image, weights */
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2,
       ORACLE_FP8_E4M3 = 3,    /* OCP FP8 E4M3: bias 7, no infinities, S.1111.111 = NaN, max 448 */
       ORACLE_FP8_E5M2 = 4 };  /* OCP FP8 E5M2: bias 15, IEEE-like infinities and NaNs, max 57344 */

/* epilogues: t = alpha*s (+ bias[j]);  out = act(t) */
enum {
    ORACLE_EPI_NONE = 0,
    ORACLE_EPI_BIAS = 1,
    ORACLE_EPI_RELU = 2,
    ORACLE_EPI_BIAS_RELU = 3,
    ORACLE_EPI_BIAS_GELU_TANH = 4,
    ORACLE_EPI_GELU_TANH = 5
};

/* out[i*ldo + j] = act(alpha * sum_k A[i][k]*B[k][j] + bias[j]).
 * A is M x K with leading dimension lda.  B is K x N (ldb) or, if trans_b,
 * stored N x K (ldb) and read as B[k][j] = Bt[j][k].  preact (may be NULL)
 * receives t before the activation, same layout as out. */
int oracle_matmul(const void* A, const void* B, const float* bias,
                  double* out, double* preact,
                  int64_t M, int64_t N, int64_t K,
                  int64_t lda, int64_t ldb, int64_t ldo,
                  int dtype, int trans_b, float alpha, int epi);

/* batch independent problems; element strides between consecutive batches
 * (stride_a / stride_b may be 0 to broadcast). */
int oracle_batched_matmul(const void* A, const void* B, const float* bias,
                          double* out, double* preact,
                          int64_t batch, int64_t M, int64_t N, int64_t K,
                          int64_t lda, int64_t ldb, int64_t ldo,
                          int64_t stride_a, int64_t stride_b, int64_t stride_o,
                          int dtype, int trans_b, float alpha, int epi);

/* Direct convolution (cross-correlation, no filter flip).
 * x [N][H][W][Cin], w [KH][KW][Cin][Cout], out [N][OH][OW][Cout],
 * OH = (H + 2*pad_h - dil_h*(KH-1) - 1)/stride_h + 1 (floor), same for OW.
 * Taps that fall outside the image contribute nothing. */
int oracle_conv2d_nhwc(const void* x, const void* w, const float* bias,
                       double* out, double* preact,
                       int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                       int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                       int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                       int dtype, float alpha, int epi);

/* Same definitions evaluated only at listed output coordinates (for sizes at
 * which the full loops would take hours).  out[s], preact[s] per sample. */
int oracle_batched_matmul_at(const void* A, const void* B, const float* bias,
                             double* out, double* preact,
                             int64_t batch, int64_t M, int64_t N, int64_t K,
                             int64_t lda, int64_t ldb,
                             int64_t stride_a, int64_t stride_b,
                             int dtype, int trans_b, float alpha, int epi,
                             int64_t nsamp, const int64_t* sb,
                             const int64_t* si, const int64_t* sj);

int oracle_conv2d_nhwc_at(const void* x, const void* w, const float* bias,
                          double* out, double* preact,
                          int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                          int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                          int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                          int dtype, float alpha, int epi,
                          int64_t nsamp, const int64_t* sn, const int64_t* soh,
                          const int64_t* sow, const int64_t* sco);

/* Convolution with separate padding on the four sides (the "same"-style
 * padding kinds of the frameworks; paper Sec. 4.5 lists padding kinds among the
 * supported configurations).  Output rows: (H + pad_top + pad_bottom -
 * dil_h*(KH-1) - 1)/stride_h + 1, columns likewise; row oh reads input rows
 * oh*stride_h - pad_top + kh*dil_h. */
int oracle_conv2d_nhwc_pad4(const void* x, const void* w, const float* bias,
                            double* out, double* preact,
                            int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                            int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                            int64_t pad_top, int64_t pad_bottom, int64_t pad_left, int64_t pad_right,
                            int64_t dil_h, int64_t dil_w,
                            int dtype, float alpha, int epi);

/* Transposed convolution (paper Sec. 4.5: transpose convolutions are covered
 * by the same lowering).  x [N][H][W][Cin], w [KH][KW][Cin][Cout],
 * out [N][OH][OW][Cout] with OH = (H-1)*stride_h - 2*pad_h + dil_h*(KH-1) +
 * out_pad_h + 1: each input pixel scatters x*w to output rows
 * ih*stride_h - pad_h + kh*dil_h (the adjoint of the convolution with the same
 * filter and geometry).  out_pad must be smaller than the stride or the dilation. */
int oracle_conv2d_transpose_nhwc(const void* x, const void* w, const float* bias,
                                 double* out, double* preact,
                                 int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                 int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                 int64_t pad_h, int64_t pad_w, int64_t out_pad_h, int64_t out_pad_w,
                                 int64_t dil_h, int64_t dil_w,
                                 int dtype, float alpha, int epi);
int oracle_conv2d_transpose_nhwc_at(const void* x, const void* w, const float* bias,
                                    double* out, double* preact,
                                    int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                    int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                    int64_t pad_h, int64_t pad_w, int64_t out_pad_h, int64_t out_pad_w,
                                    int64_t dil_h, int64_t dil_w,
                                    int dtype, float alpha, int epi,
                                    int64_t nsamp, const int64_t* sn, const int64_t* soh,
                                    const int64_t* sow, const int64_t* sco);
int64_t oracle_conv_transpose_out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad,
                                      int64_t out_pad, int64_t dil);

/* int8 x int8 contraction, exact integer accumulation, and the quantised
 * epilogue of the paper's appendix on quantisation (figure of the fused
 * de-quantisation / quantisation nest).  The epilogue runs in binary32, one
 * rounding per operation, in this order:
 *   t = float(acc) * scale[j];  t += bias[j] (if bias);
 *   if mid_scale > 0: t = float(clamp(roundeven(t / mid_scale), -128, 127)) * mid_scale;
 *   t *= mul[j] (if mul);  t += add[j] (if add);  t = max(t, 0) (if relu);
 *   out_int8 ? int8(clamp(roundeven(t / out_scale), -128, 127)) : t.
 * out is int8_t or float accordingly; acc_out (may be NULL) receives the
 * integer sums.  B is K x N (ldb) or, if trans_b, N x K.  K <= 131071 keeps the
 * sum inside int32. */
int oracle_matmul_int8(const int8_t* A, const int8_t* B, void* out, int32_t* acc_out,
                       int64_t M, int64_t N, int64_t K,
                       int64_t lda, int64_t ldb, int64_t ldo, int trans_b,
                       const float* scale, const float* bias, float mid_scale,
                       const float* mul, const float* add, int relu, float out_scale,
                       int out_int8);

/* Same epilogue on the direct convolution (x NHWC, w HWIO, symmetric padding). */
int oracle_conv2d_nhwc_int8(const int8_t* x, const int8_t* w, void* out, int32_t* acc_out,
                            int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                            int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                            int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                            const float* scale, const float* bias, float mid_scale,
                            const float* mul, const float* add, int relu, float out_scale,
                            int out_int8);

/* The same two with the batch-norm step of the paper's figure unfolded: between the optional quantise /
 * de-quantise pair and the ReLU,
 *   r = 1 / sqrt(var[j] + eps);  t = t - mean[j];  t = t * r;  t = t * gamma[j];  t = t + beta[j]
 * each one binary32 operation (the square root and the division correctly rounded), in this order. */
int oracle_matmul_int8_bn(const int8_t* A, const int8_t* B, void* out, int32_t* acc_out,
                          int64_t M, int64_t N, int64_t K,
                          int64_t lda, int64_t ldb, int64_t ldo, int trans_b,
                          const float* scale, const float* bias, float mid_scale,
                          const float* mean, const float* var, float eps, const float* gamma, const float* beta,
                          int relu, float out_scale, int out_int8);
int oracle_conv2d_nhwc_int8_bn(const int8_t* x, const int8_t* w, void* out, int32_t* acc_out,
                               int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                               int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                               int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                               const float* scale, const float* bias, float mid_scale,
                               const float* mean, const float* var, float eps, const float* gamma, const float* beta,
                               int relu, float out_scale, int out_int8);

/* Residual-add epilogue: out = act(alpha * (A . B) + bias + beta * R), R of the
 * output's shape (row stride ldr), element type r_dtype (F32, BF16, F16),
 * widened exactly.  The convolution variant takes r [N][OH][OW][Cout]. */
int oracle_matmul_residual(const void* A, const void* B, const float* bias,
                           const void* R, double* out, double* preact,
                           int64_t M, int64_t N, int64_t K,
                           int64_t lda, int64_t ldb, int64_t ldo, int64_t ldr,
                           int dtype, int r_dtype, int trans_b, float alpha, float beta, int epi);
int oracle_conv2d_nhwc_residual(const void* x, const void* w, const float* bias,
                                const void* r, double* out, double* preact,
                                int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                                int dtype, int r_dtype, float alpha, float beta, int epi);

/* Attention layer (paper Sec. 4.4; the operator of its attention example):
 *   out[b][i][d] = sum_j P[b][i][j] * V[b][j][d],
 *   P[b][i][:]   = softmax_j( alpha * sum_c Q[b][i][c]*K[b][j][c] + bias[b][i][j] ).
 * Q [batch][Nq][D] (row stride ldq, batch stride stride_q), K, V [batch][Nk][D]
 * likewise, out [batch][Nq][D] doubles (ldo, stride_o), bias float
 * [batch][Nq][Nk] (ld_bias, stride_bias; stride 0 shares one matrix; NULL = no
 * bias).  dtype F32, BF16 or F16.  A bias of -inf removes a key from a row; a
 * row with every key removed is 0/0 and comes back NaN. */
int oracle_attention(const void* Q, const void* K, const void* V, const float* bias,
                     double* out,
                     int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                     int64_t ldq, int64_t ldk, int64_t ldv, int64_t ldo,
                     int64_t stride_q, int64_t stride_k, int64_t stride_v, int64_t stride_o,
                     int64_t ld_bias, int64_t stride_bias,
                     int dtype, float alpha);

/* Same definition for listed rows only: out[s][0..D) is row (sb[s], si[s]). */
int oracle_attention_rows(const void* Q, const void* K, const void* V, const float* bias,
                          double* out,
                          int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                          int64_t ldq, int64_t ldk, int64_t ldv,
                          int64_t stride_q, int64_t stride_k, int64_t stride_v,
                          int64_t ld_bias, int64_t stride_bias,
                          int dtype, float alpha,
                          int64_t nsamp, const int64_t* sb, const int64_t* si);

/* Causal attention: the same operator in which query row i attends to the keys
 * j <= i + (Nk - Nq) only (the mask of an autoregressive decoder; with Nq = Nk: j <= i;
 * with fewer queries than keys the queries are the LAST Nq positions).  No bias.  A row that
 * sees no key (possible only when Nq > Nk) is 0/0 and comes back NaN. */
int oracle_attention_causal(const void* Q, const void* K, const void* V,
                            double* out,
                            int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                            int64_t ldq, int64_t ldk, int64_t ldv, int64_t ldo,
                            int64_t stride_q, int64_t stride_k, int64_t stride_v, int64_t stride_o,
                            int dtype, float alpha);
int oracle_attention_causal_rows(const void* Q, const void* K, const void* V,
                                 double* out,
                                 int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                                 int64_t ldq, int64_t ldk, int64_t ldv,
                                 int64_t stride_q, int64_t stride_k, int64_t stride_v,
                                 int dtype, float alpha,
                                 int64_t nsamp, const int64_t* sb, const int64_t* si);

/* Output size of one spatial dimension, or -1 if empty/invalid. */
int64_t oracle_conv_out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad, int64_t dil);

/* scalar pieces, exported so that tests can pin them one by one */
double   oracle_epilogue(double s, double bias, float alpha, int epi);
double   oracle_gelu_tanh(double t);
double   oracle_widen(uint32_t bits, int dtype);       /* stored bits -> double */
uint16_t oracle_round_bf16(double v);                  /* round-to-nearest-even */
uint16_t oracle_round_f16(double v);

/* number of threads the loops will use (OpenMP) */
int oracle_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
