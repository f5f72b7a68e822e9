// Generic attention kernel: any element type, any alignment, head size up to
// 512.  One wave per query row; keys are taken in chunks with the running
// maximum / running sum recurrence of the online softmax, so the row of
// scores never exists in memory (paper Sec. 4.4: all operators of the layer
// fused into one nest).  True fp32 arithmetic on widened inputs.  It is the
// fp32 path and the safety net for shapes the MFMA kernel declines.
#include <hip/hip_runtime.h>
#include <math.h>
#include "pbk_problem.h"
#include "pbk_epilogue.h"

namespace pbk {
namespace {

constexpr int AG_CHUNK = 256;      // keys per chunk
constexpr int AG_DREG = 8;         // output elements per lane: D <= 64 * AG_DREG

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

template <typename T> __device__ __forceinline__ void store_out(T* p, float v);
template <> __device__ __forceinline__ void store_out<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_out<bf16_t>(bf16_t* p, float v) { *p = (bf16_t)v; }
template <> __device__ __forceinline__ void store_out<f16_t>(f16_t* p, float v) { *p = (f16_t)v; }

template <typename T>
__global__ __launch_bounds__(64) void attention_generic_kernel(AttnProblem p) {
    __shared__ float w[AG_CHUNK];          // scores, then weights, of the current chunk
    const int lane = threadIdx.x;
    const int b = blockIdx.x / p.Nq, i = blockIdx.x % p.Nq;
    const T* q = (const T*)p.Q + (int64_t)b * p.stride_q + (int64_t)i * p.ldq;
    const T* K = (const T*)p.K + (int64_t)b * p.stride_k;
    const T* V = (const T*)p.V + (int64_t)b * p.stride_v;
    const float* bias = p.bias ? p.bias + (int64_t)b * p.stride_bias + (int64_t)i * p.ld_bias : nullptr;

    float o[AG_DREG];
#pragma unroll
    for (int e = 0; e < AG_DREG; ++e) o[e] = 0.0f;
    float m = -INFINITY, l = 0.0f;

    // causal: the row's keys are 0 .. i + (Nk - Nq); none at all gives 0 / 0
    int nk = p.Nk;
    if (p.causal) {
        const long long vis = (long long)i + p.Nk - p.Nq + 1;
        nk = vis < 0 ? 0 : vis < p.Nk ? (int)vis : p.Nk;
    }
    for (int j0 = 0; j0 < nk; j0 += AG_CHUNK) {
        const int n = nk - j0 < AG_CHUNK ? nk - j0 : AG_CHUNK;
        float cmax = -INFINITY;
        for (int t = lane; t < n; t += 64) {
            const T* k = K + (int64_t)(j0 + t) * p.ldk;
            float dot = 0.0f;
            for (int c = 0; c < p.D; ++c) dot = fmaf(widen<T>(q[c]), widen<T>(k[c]), dot);
            float s = p.alpha * dot;
            if (bias) s += bias[j0 + t];
            w[t] = s;
            cmax = fmaxf(cmax, s);
        }
        cmax = wave_max(cmax);
        const float m_new = fmaxf(m, cmax);
        const float m_use = m_new == -INFINITY ? 0.0f : m_new;     // every key so far removed by -inf bias
        const float corr = expf(m - m_use);
        __syncthreads();
        float csum = 0.0f;
        for (int t = lane; t < n; t += 64) {
            float e = expf(w[t] - m_use);
            w[t] = e;
            csum += e;
        }
        l = l * corr + wave_sum(csum);
        m = m_new;
        __syncthreads();
#pragma unroll
        for (int e = 0; e < AG_DREG; ++e) {
            const int d = lane + 64 * e;
            if (d < p.D) {
                float acc = 0.0f;
                for (int t = 0; t < n; ++t) acc = fmaf(w[t], widen<T>(V[(int64_t)(j0 + t) * p.ldv + d]), acc);
                o[e] = o[e] * corr + acc;
            }
        }
        __syncthreads();
    }
    T* out = (T*)p.O + (int64_t)b * p.stride_o + (int64_t)i * p.ldo;
#pragma unroll
    for (int e = 0; e < AG_DREG; ++e) {
        const int d = lane + 64 * e;
        if (d < p.D) store_out<T>(out + d, o[e] / l);
    }
}

template <typename T>
hipError_t launch_t(const AttnProblem& p, hipStream_t stream) {
    long long rows = (long long)p.batch * p.Nq;
    if (rows <= 0 || rows > 0x7FFFFFFFLL || p.D > 64 * AG_DREG) return hipErrorInvalidValue;
    AttnProblem pa = p;
    void* args[] = {&pa};
    return hipLaunchKernel((const void*)attention_generic_kernel<T>, dim3((unsigned)rows), dim3(64), args, 0, stream);
}

}  // namespace

hipError_t launch_attention_generic(const AttnProblem& p, hipStream_t stream, const char** name) {
    *name = "attn_generic_row_per_wave";
    switch (p.dtype) {
    case DT_F32: return launch_t<float>(p, stream);
    case DT_BF16: return launch_t<bf16_t>(p, stream);
    case DT_F16: return launch_t<f16_t>(p, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace pbk
