/*
 * libpbk: fused dense contractions for AMD MI355X (gfx950).
 *
 *     out = act(alpha * (A . B) + bias)
 *
 * as matmul, batched matmul, and 2-d convolution lowered as an implicit GEMM
 * (the tile of im2col rows is packed on the fly; the im2col matrix never
 * exists in memory).  This is the operator the paper's code generator targets:
 * a tiled matmul/convolution nest with its pointwise tail fused into the
 * output tile (paper Sec. 4.3, 4.5, 4.6).  Also the attention layer
 * softmax(alpha Q K^T + bias) V as one fused kernel (paper Sec. 4.4).
 *
 * Conventions shared by every entry point
 *  - All data pointers are DEVICE pointers valid on the device that `stream`
 *    belongs to.  The library never allocates, frees or keeps them.  The
 *    output must not alias any input.
 *  - Calls only enqueue work on `stream` (a hipStream_t; NULL = the default
 *    stream) and return; ordering is stream ordering.
 *  - Matrices are row-major with leading dimensions in ELEMENTS.
 *  - in_dtype is the element type of A and B (image and weights);
 *    out_dtype must be PBK_F32 or equal to in_dtype; for the FP8 input types it
 *    may be PBK_F32, PBK_BF16 or PBK_F16 (never FP8).  bias is always float.
 *    16-bit and 8-bit inputs are widened exactly, products are accumulated in
 *    fp32,
 *    the epilogue runs in fp32, and the result is rounded once to out_dtype
 *    (round-to-nearest-even).  PBK_F32 inputs use true fp32 multiply-add
 *    (VALU fma, or v_mfma_f32_32x32x2_f32 for large aligned problems; never a
 *    reduced-precision emulation).
 *  - Epilogue: t = alpha * acc (+ bias[n] for the BIAS variants);
 *    out = t | max(t,0) | 0.5*t*(1+tanh(sqrt(2/pi)*(t+0.044715*t^3))).
 *    bias must be non-NULL for the BIAS variants and is ignored otherwise.
 *    The ReLU keeps NaN (it selects t when t > 0 or t is NaN).
 *  - Every function returns a pbk_status.  On any status other than PBK_OK
 *    nothing was launched and the output is untouched.  A dimension of zero
 *    gives PBK_OK and does nothing (K == 0 still writes act(bias)).
 *  - Elements outside the M x K / K x N views (beyond K up to lda, etc.) are
 *    never allowed to influence the result, even if they hold NaN or Inf.
 *  - Re-entrant; no global mutable state besides a read-only cache of device
 *    properties.
 */
#ifndef PBK_H
#define PBK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The HIP stream handle, declared here exactly as the HIP runtime declares it, so that
 * this header needs no HIP header (a repeated identical typedef is valid C11 and C++). */
typedef struct ihipStream_t* hipStream_t;

typedef enum {
    PBK_OK = 0,
    PBK_ERR_NULL = 1,        /* a required pointer is NULL */
    PBK_ERR_SHAPE = 2,       /* negative dimension, empty conv output, size overflow */
    PBK_ERR_STRIDE = 3,      /* leading dimension or batch stride too small */
    PBK_ERR_ALIGN = 4,       /* pointer not aligned to its element size */
    PBK_ERR_DTYPE = 5,       /* unknown dtype or unsupported in/out pair */
    PBK_ERR_EPILOGUE = 6,    /* unknown epilogue, or bias missing */
    PBK_ERR_UNSUPPORTED = 7, /* valid request this build cannot run */
    PBK_ERR_HIP = 8          /* the HIP runtime reported an error at launch */
} pbk_status;

typedef enum {
    PBK_F32 = 0,
    PBK_BF16 = 1,
    PBK_F16 = 2,
    PBK_FP8_E4M3 = 3,   /* OCP FP8 E4M3 (bias 7, no infinities, max 448); input type only */
    PBK_FP8_E5M2 = 4,   /* OCP FP8 E5M2 (bias 15, max 57344); input type only */
    PBK_INT8 = 5        /* signed 8-bit integers; only through the *_int8 entry points */
} pbk_dtype;

typedef enum {
    PBK_EPI_NONE = 0,
    PBK_EPI_BIAS = 1,
    PBK_EPI_RELU = 2,
    PBK_EPI_BIAS_RELU = 3,
    PBK_EPI_BIAS_GELU_TANH = 4,
    PBK_EPI_GELU_TANH = 5
} pbk_epilogue;

/*
 * C[M][N] = act(alpha * A[M][K] . B[K][N] + bias[N])          (paper Sec. 4.3/4.6)
 * A: M x K, lda >= K.  B: K x N with ldb >= N, or if trans_b != 0 stored as
 * N x K with ldb >= K (B[k][n] = Bt[n][k]).  C: M x N, ldc >= N.
 */
pbk_status pbk_matmul(const void* A, const void* B, void* C, const float* bias,
                      int64_t M, int64_t N, int64_t K,
                      int64_t lda, int64_t ldb, int64_t ldc,
                      pbk_dtype in_dtype, pbk_dtype out_dtype, int trans_b,
                      float alpha, pbk_epilogue epi, hipStream_t stream);

/*
 * `batch` independent matmuls with one launch (paper Sec. 4.4: the two contractions of
 * the attention layer are batched over batch x heads; workload configuration
 * "attention scores" is the first of them).  Entry b uses A + b*stride_a, B + b*stride_b,
 * C + b*stride_c (strides in elements).  stride_a or stride_b may be 0 to
 * share one operand among all entries; stride_c must be >= (M-1)*ldc + N.
 * bias[N] is shared by all entries.
 */
pbk_status pbk_batched_matmul(const void* A, const void* B, void* C, const float* bias,
                              int64_t batch, int64_t M, int64_t N, int64_t K,
                              int64_t lda, int64_t ldb, int64_t ldc,
                              int64_t stride_a, int64_t stride_b, int64_t stride_c,
                              pbk_dtype in_dtype, pbk_dtype out_dtype, int trans_b,
                              float alpha, pbk_epilogue epi, hipStream_t stream);

/*
 * y[N][OH][OW][Cout] = act(alpha * conv(x, w) + bias[Cout])      (paper Sec. 4.5)
 * x: [N][H][W][Cin] (NHWC, dense).  w: [KH][KW][Cin][Cout] (dense).
 * Cross-correlation (no filter flip):
 *   y[n][oh][ow][co] = sum_{kh,kw,c} x[n][oh*stride_h - pad_h + kh*dil_h]
 *                                       [ow*stride_w - pad_w + kw*dil_w][c] * w[kh][kw][c][co]
 * with taps outside the image contributing zero, i.e. the GEMM with
 * M = N*OH*OW rows (n, oh, ow), N = Cout, K = KH*KW*Cin ordered (kh, kw, c).
 * OH = (H + 2*pad_h - dil_h*(KH-1) - 1) / stride_h + 1 (floor), OW likewise;
 * an empty output is PBK_ERR_SHAPE.
 */
pbk_status pbk_conv2d_nhwc(const void* x, const void* w, void* y, const float* bias,
                           int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                           int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                           int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                           pbk_dtype in_dtype, pbk_dtype out_dtype,
                           float alpha, pbk_epilogue epi, hipStream_t stream);

/*
 * The same convolution with separate padding on the four sides (the "same"-style
 * padding kinds; paper Sec. 4.5 lists padding kinds among the covered
 * configurations).  Row oh reads input rows oh*stride_h - pad_top + kh*dil_h;
 * OH = (H + pad_top + pad_bottom - dil_h*(KH-1) - 1) / stride_h + 1, OW likewise
 * with pad_left / pad_right.  pbk_conv2d_nhwc is this call with equal paddings.
 */
pbk_status pbk_conv2d_nhwc_pad4(const void* x, const void* w, void* y, const float* bias,
                                int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                int64_t pad_top, int64_t pad_bottom, int64_t pad_left, int64_t pad_right,
                                int64_t dil_h, int64_t dil_w,
                                pbk_dtype in_dtype, pbk_dtype out_dtype,
                                float alpha, pbk_epilogue epi, hipStream_t stream);

/*
 * Transposed convolution (paper Sec. 4.5: covered by the same lowering).
 * x: [N][H][W][Cin], w: [KH][KW][Cin][Cout], y: [N][OH][OW][Cout] with
 *   OH = (H-1)*stride_h - 2*pad_h + dil_h*(KH-1) + out_pad_h + 1   (OW likewise),
 *   y[n][oh][ow][co] = sum over (ih, kh) with ih*stride_h - pad_h + kh*dil_h == oh,
 *                      (iw, kw) likewise, and c, of x[n][ih][iw][c] * w[kh][kw][c][co]:
 * the adjoint of the convolution with the same filter and geometry.  out_pad must
 * be smaller than the stride or the dilation, OH and OW must be >= 1.  It runs as
 * the implicit GEMM with rows (n, oh, ow) and K = KH*KW*Cin in which the taps
 * that do not divide by the stride are zero; the epilogue is the usual one.
 */
pbk_status pbk_conv2d_transpose_nhwc(const void* x, const void* w, void* y, const float* bias,
                                     int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                     int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                     int64_t pad_h, int64_t pad_w, int64_t out_pad_h, int64_t out_pad_w,
                                     int64_t dil_h, int64_t dil_w,
                                     pbk_dtype in_dtype, pbk_dtype out_dtype,
                                     float alpha, pbk_epilogue epi, hipStream_t stream);

/*
 * Residual-add epilogue: C = act(alpha * A . B + bias + beta * R), the shortcut
 * branch of a residual block summed into the output tile before the activation
 * (paper Sec. 4.3: pointwise consumers fused into the tile).  R is M x N (row
 * stride ldr >= N) resp. [N][OH][OW][Cout], of type out_dtype, may alias nothing
 * that is written.  Everything else as pbk_matmul / pbk_conv2d_nhwc.
 */
pbk_status pbk_matmul_residual(const void* A, const void* B, void* C, const float* bias, const void* R,
                               int64_t M, int64_t N, int64_t K,
                               int64_t lda, int64_t ldb, int64_t ldc, int64_t ldr,
                               pbk_dtype in_dtype, pbk_dtype out_dtype, int trans_b,
                               float alpha, float beta, pbk_epilogue epi, hipStream_t stream);

pbk_status pbk_conv2d_nhwc_residual(const void* x, const void* w, void* y, const float* bias, const void* r,
                                    int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                    int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                    int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                                    pbk_dtype in_dtype, pbk_dtype out_dtype,
                                    float alpha, float beta, pbk_epilogue epi, hipStream_t stream);

/*
 * int8 x int8 contraction with exact 32-bit integer accumulation and a quantised
 * epilogue after the paper's appendix on quantisation (the fused de-quantisation /
 * quantisation nest at the output of a quantised convolution) with the batch norm
 * folded by the caller into a multiplier and a shift (the *_bn calls below take it
 * unfolded, as the figure has it), computed in
 * binary32, one rounding per operation, in this order, for output column j:
 *   t = float(acc) * scale[j];           de-quantise (scale is required)
 *   t = t + bias[j]                      if bias != NULL
 *   if mid_scale > 0:                    a quantise / de-quantise pair
 *       t = float(clamp(roundeven(t / mid_scale), -128, 127)) * mid_scale
 *   t = t * mul[j]                       if mul != NULL   (batch-norm scale, folded by the caller)
 *   t = t + add[j]                       if add != NULL   (batch-norm shift, folded by the caller)
 *   t = (t > 0 or t is NaN) ? t : 0      if relu != 0   (the figure's compare is "unordered or greater")
 *   out_dtype PBK_INT8: C = int8(clamp(roundeven(t / out_scale), -128, 127)), out_scale > 0
 *   out_dtype PBK_F32:  C = t
 * Results are bit-exact for a given input whatever kernel runs.  scale, bias, mul,
 * add are device float arrays of N entries.  K (KH*KW*Cin) must not exceed 131071
 * (PBK_ERR_UNSUPPORTED), which keeps every sum inside 32 bits.  A: M x K (lda);
 * B: K x N (ldb) or, if trans_b, N x K.  Convolution: x NHWC, w HWIO, symmetric
 * padding, OH/OW as pbk_conv2d_nhwc.  The matrix-unit kernel takes 16-byte aligned
 * operands with K, lda, ldb (and N for row-major B; Cin and Cout for the
 * convolution) multiples of 16; other calls run on the generic kernel with
 * integer accumulation.
 */
pbk_status pbk_matmul_int8(const int8_t* A, const int8_t* B, void* C,
                           int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb, int64_t ldc, int trans_b,
                           const float* scale, const float* bias, float mid_scale,
                           const float* mul, const float* add, int relu, float out_scale,
                           pbk_dtype out_dtype, hipStream_t stream);

pbk_status pbk_conv2d_nhwc_int8(const int8_t* x, const int8_t* w, void* y,
                                int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                                const float* scale, const float* bias, float mid_scale,
                                const float* mul, const float* add, int relu, float out_scale,
                                pbk_dtype out_dtype, hipStream_t stream);

/*
 * The same two with the batch-norm step exactly as the paper's fused nest has it (appendix on
 * quantisation, figure "IR after fusion of de-quantization and quantization"), unfolded: between the
 * optional quantise / de-quantise pair and the ReLU,
 *   r = 1 / sqrt(var[j] + eps)           an addition, a square root and a division (the last two
 *                                        correctly rounded)
 *   t = t - mean[j];  t = t * r;  t = t * gamma[j];  t = t + beta[j]
 * each one binary32 operation, in this order.  mean, var, gamma, beta: device float arrays of N (Cout)
 * entries, all required (PBK_ERR_EPILOGUE).  The caller-folded form above (mul = r * gamma,
 * add = beta - mean * mul) is cheaper by two operations and differs from this one in the last place.
 */
pbk_status pbk_matmul_int8_bn(const int8_t* A, const int8_t* B, void* C,
                              int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb, int64_t ldc, int trans_b,
                              const float* scale, const float* bias, float mid_scale,
                              const float* mean, const float* var, float eps, const float* gamma, const float* beta,
                              int relu, float out_scale, pbk_dtype out_dtype, hipStream_t stream);

pbk_status pbk_conv2d_nhwc_int8_bn(const int8_t* x, const int8_t* w, void* y,
                                   int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                   int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                   int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                                   const float* scale, const float* bias, float mid_scale,
                                   const float* mean, const float* var, float eps, const float* gamma, const float* beta,
                                   int relu, float out_scale, pbk_dtype out_dtype, hipStream_t stream);

/*
 * Attention layer, every operator fused into one kernel          (paper Sec. 4.4)
 *   O[b][i][:] = sum_j P[b][i][j] * V[b][j][:],
 *   P[b][i][:] = softmax over j of ( alpha * sum_c Q[b][i][c] * K[b][j][c] + bias[b][i][j] ).
 * `batch` independent entries (batch x heads flattened).  Q and O are Nq x D, K
 * and V are Nk x D, row-major with row strides ldq, ldk, ldv, ldo >= D and batch
 * strides stride_* (elements; 0 for K, V, Q shares one operand; stride_o must be
 * >= (Nq-1)*ldo + D when batch > 1).  bias is float, Nq x Nk with row stride
 * ld_bias >= Nk and batch stride stride_bias (0 = one matrix for all entries), or
 * NULL.  A bias of -inf removes a key from a row (masks); a row whose keys are all
 * removed has no defined result.  dtype (PBK_F32, PBK_BF16 or PBK_F16) is the
 * type of Q, K, V and O.  Scores and the softmax are computed in fp32; for the
 * 16-bit types the weights are rounded to dtype before they multiply V (fp32
 * accumulation), and O is rounded once.  The Nq x Nk score matrix never exists
 * in memory.  Nk must be >= 1 unless batch or Nq is 0; D must be >= 1 and, on
 * the generic path, <= 512 (else PBK_ERR_UNSUPPORTED).  The matrix-unit kernel
 * takes 16-bit types with D of 32, 64 or 128, 16-byte aligned Q, K, V, 8-byte
 * aligned O, row and batch strides that are multiples of 8 (4 for O); anything
 * else runs on the generic kernel.
 */
pbk_status pbk_attention(const void* Q, const void* K, const void* V, const float* bias, void* O,
                         int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                         int64_t ldq, int64_t ldk, int64_t ldv, int64_t ldo,
                         int64_t stride_q, int64_t stride_k, int64_t stride_v, int64_t stride_o,
                         int64_t ld_bias, int64_t stride_bias,
                         pbk_dtype dtype, float alpha, hipStream_t stream);

/*
 * Causal attention: the same operator in which query row i attends to the keys
 * j <= i + (Nk - Nq) only (the mask of an autoregressive decoder; Sec. 4.4 operator
 * with that mask; with Nq = Nk: j <= i; with fewer queries than keys the queries are
 * the last Nq positions).  No bias.  Key tiles that no query of a workgroup can see
 * are skipped, not masked: about half the work of the full operator for Nq = Nk.
 * Arguments, layouts, types and errors as for pbk_attention.  A row that sees no key
 * (possible only when Nq > Nk) has no defined result.  The matrix-unit kernel takes
 * the causal form for alpha > 0; otherwise the generic kernel runs it.
 */
pbk_status pbk_attention_causal(const void* Q, const void* K, const void* V, void* O,
                                int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                                int64_t ldq, int64_t ldk, int64_t ldv, int64_t ldo,
                                int64_t stride_q, int64_t stride_k, int64_t stride_v, int64_t stride_o,
                                pbk_dtype dtype, float alpha, hipStream_t stream);

/* Static, NUL-terminated description of a status code. */
const char* pbk_status_string(pbk_status s);

/* Library version: major*10000 + minor*100 + patch. */
int pbk_version(void);

/*
 * Name of the kernel configuration the most recent successful call ON THIS
 * THREAD dispatched to (for benchmarks and tests; e.g.
 * "mfma16_128x256x32_w1x4_s3_occ2", "generic_64x64x16_fma").  Never NULL; ""
 * before the first call.
 */
const char* pbk_last_kernel(void);

/*
 * Benchmarking and test aid, for the calls that follow ON THIS THREAD: "generic" forces
 * the fallback kernel, "mfma" the matrix-unit path with its automatic tile choice,
 * "mfma:<id>" one tile configuration (operands that the direct-to-LDS kernel cannot take
 * go to the gathering matrix-unit kernel instead), "gather" that kernel, "small" the
 * one-wave-per-tile fp32 kernel, "bstat" the B-stationary kernel for short contractions (K <= 256) over
 * many rows; a problem the choice cannot run gives PBK_ERR_UNSUPPORTED.  NULL or "" returns to the default.  The default is automatic
 * choice, or what the environment variable PBK_FORCE_KERNEL (same strings) held when the
 * process made its first call.  An unknown string is PBK_ERR_UNSUPPORTED and changes nothing.
 */
pbk_status pbk_force_kernel(const char* choice);

#ifdef __cplusplus
}
#endif
#endif /* PBK_H */
