// Internal description of one contraction, shared by the dispatcher and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pbk {

enum : int { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2, DT_FP8_E4M3 = 3, DT_FP8_E5M2 = 4, DT_INT8 = 5 };
enum : int { EPI_NONE = 0, EPI_BIAS = 1, EPI_RELU = 2, EPI_BIAS_RELU = 3,
             EPI_BIAS_GELU_TANH = 4, EPI_GELU_TANH = 5 };

// Geometry of the convolution whose im2col rows form the A operand
// (paper Sec. 4.5: row i = (n, oh, ow), column k = (kh, kw, c)).
struct ConvGeom {
    int H, W, Cin;
    int OH, OW;
    int KH, KW;
    int stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;   // pad: near side (top, left)
    // 0: row (n, oh, ow) reads input rows oh*stride - pad + kh*dil.
    // 1: transposed convolution in gather form: it reads input row (oh + pad - kh*dil)/stride
    //    for the taps where the division is exact.
    int transposed;
};

struct Problem {
    const void* A;        // M x K (lda), or the NHWC image when is_conv
    const void* B;        // K x N (ldb), or N x K (ldb) when trans_b
    void* C;              // M x N (ldc)
    const float* bias;    // [N] or nullptr
    int M, N, K, batch;
    int64_t lda, ldb, ldc;
    int64_t stride_a, stride_b, stride_c;   // elements between batch entries
    int in_dtype, out_dtype;
    int trans_b;
    int is_conv;
    int epi;
    float alpha;
    ConvGeom conv;
    // residual-add epilogue: out = act(alpha*acc + bias + beta*R), R of out_dtype, M x N (ldr); nullptr = none
    const void* R;
    int64_t ldr;
    float beta;
    // int8 operands (in_dtype DT_INT8): integer accumulation and the quantised epilogue
    //   t = float(acc)*q_scale[n] (+ bias[n]); optional requantise/dequantise with q_mid;
    //   unfolded batch norm if q_mean: t = (t - q_mean[n]) * (1 / sqrt(q_var[n] + q_eps)), q_mul = gamma, q_add = beta;
    //   t = t*q_mul[n] + q_add[n] (each if given); ReLU if q_relu;
    //   out = int8(clamp(roundeven(t/q_out))) for out_dtype DT_INT8, else t as fp32.
    const float* q_scale;
    const float* q_mul;
    const float* q_add;
    float q_mid, q_out;
    int q_relu;
    const float* q_mean;
    const float* q_var;
    float q_eps;
};

// One attention layer call (paper Sec. 4.4): O = softmax(alpha Q K^T + bias) V
// per batch entry; Q, O [Nq][D], K, V [Nk][D], bias float [Nq][Nk] or nullptr.
struct AttnProblem {
    const void* Q;
    const void* K;
    const void* V;
    const float* bias;
    void* O;
    int batch, Nq, Nk, D;
    int64_t ldq, ldk, ldv, ldo;                          // row strides, elements
    int64_t stride_q, stride_k, stride_v, stride_o;      // batch strides, elements
    int64_t ld_bias, stride_bias;
    int dtype;                                           // of Q, K, V and O
    float alpha;
    int causal;                                          // 1: row i attends to keys j <= i + (Nk - Nq) only (no bias then)
};

__host__ __device__ inline bool epi_has_bias(int epi) {
    return epi == EPI_BIAS || epi == EPI_BIAS_RELU || epi == EPI_BIAS_GELU_TANH;
}

// Launchers.  Each returns hipSuccess or the launch error; `name` receives a
// static string naming the configuration that ran.
hipError_t launch_generic(const Problem& p, hipStream_t stream, const char** name);
// small fp32 matmuls, one wave per 16 x 16 tile
bool small_f32_supported(const Problem& p);
bool small_f32_preferred(const Problem& p);
hipError_t launch_small_f32(const Problem& p, hipStream_t stream, const char** name);

// Returns false if this problem cannot take the MFMA path (alignment, dtype).
bool mfma_supported(const Problem& p);
// Returns false where the generic kernel is the better choice although the MFMA path could run.
bool mfma_preferred(const Problem& p);
hipError_t launch_mfma(const Problem& p, hipStream_t stream, int force_cfg, const char** name);

// The matrix-unit kernel that gathers its tiles element by element: 16-bit operands of any alignment, K, N
// and leading dimensions; convolutions with at least 8 input channels.
bool mfma_gather_supported(const Problem& p);
hipError_t launch_mfma_gather(const Problem& p, hipStream_t stream, const char** name);

// Short contractions (K <= 256) over many rows: B stationary in registers, the workgroup walks down M.
bool mfma_bstat_supported(const Problem& p);
bool mfma_bstat_preferred(const Problem& p);
hipError_t launch_mfma_bstat(const Problem& p, hipStream_t stream, const char** name);

// PBK_GROUP_M of the environment as read at the process's first call (0 = not set): tile rows
// per group of the block mapping, a benchmarking override.
int group_m_override();

// Attention: generic kernel (any dtype/alignment, D <= 512) and the fused MFMA kernel.
hipError_t launch_attention_generic(const AttnProblem& p, hipStream_t stream, const char** name);
bool attention_mfma_supported(const AttnProblem& p);
hipError_t launch_attention_mfma(const AttnProblem& p, hipStream_t stream, const char** name);

}  // namespace pbk
