// Fused pointwise tail applied to fp32 accumulators in registers, and the
// single rounding to the output type (paper Sec. 4.3: pointwise consumers are
// fused into the copy-out of the tiled nest; here they run before any store).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "pbk_problem.h"

namespace pbk {

typedef __bf16 bf16_t;
typedef _Float16 f16_t;
// OCP FP8 operands (OFP8 specification); storage is one byte
struct fp8_e4m3_t { uint8_t v; };
struct fp8_e5m2_t { uint8_t v; };

__device__ __forceinline__ float gelu_tanh_f32(float t) {
    // 0.5 t (1 + tanh(u)), u = sqrt(2/pi) (t + 0.044715 t^3), written as t / (1 + exp(-2u)) (the same function:
    // 1 + tanh(u) = 2 / (1 + exp(-2u))); the exponential in base 2 with the constants folded:
    // -2u log2(e) = t (k1 + k2 t^2).  Hardware exp2 and reciprocal (1 ulp each); exp2 = inf gives -0, 0 gives t.
    const float k1 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;
    const float k2 = k1 * 0.044715f;
    const float w = t * fmaf(k2, t * t, k1);
    const float e = __builtin_amdgcn_exp2f(w);
    return t * __builtin_amdgcn_rcpf(1.0f + e);
}

// ReLU that keeps NaN: "greater than zero, or unordered" selects t (the compare of the paper's fused nest;
// the hardware maximum would turn NaN into 0)
__device__ __forceinline__ float relu_keep_nan(float t) { return !(t <= 0.0f) ? t : 0.0f; }

// t = alpha*acc + bias + beta*res ; act(t).  `bias` must be 0 when the epilogue has none.
__device__ __forceinline__ float apply_epilogue(float acc, float alpha, float bias, int epi,
                                                float beta = 0.0f, float res = 0.0f) {
    float t = fmaf(alpha, acc, bias);
    t = fmaf(beta, res, t);             // residual operand; beta is 0 when there is none
    switch (epi) {
    case EPI_RELU:
    case EPI_BIAS_RELU:
        return relu_keep_nan(t);
    case EPI_BIAS_GELU_TANH:
    case EPI_GELU_TANH:
        return gelu_tanh_f32(t);
    default:
        return t;
    }
}

// fp32 -> 16-bit storage, round to nearest even (hardware conversions).
template <typename T> __device__ __forceinline__ uint16_t to_bits16(float v);
template <> __device__ __forceinline__ uint16_t to_bits16<bf16_t>(float v) {
    return __builtin_bit_cast(uint16_t, (bf16_t)v);
}
template <> __device__ __forceinline__ uint16_t to_bits16<f16_t>(float v) {
    return __builtin_bit_cast(uint16_t, (f16_t)v);
}

template <typename T> __device__ __forceinline__ float widen(T v) { return (float)v; }
// E5M2 is the upper byte of a binary16
template <> __device__ __forceinline__ float widen<fp8_e5m2_t>(fp8_e5m2_t x) {
    return (float)__builtin_bit_cast(f16_t, (uint16_t)((uint16_t)x.v << 8));
}
// E4M3: bias 7, subnormals m/8 * 2^-6, S.1111.111 is NaN, no infinities
template <> __device__ __forceinline__ float widen<fp8_e4m3_t>(fp8_e4m3_t x) {
    uint32_t b = x.v, sign = (b & 0x80u) << 24, e = (b >> 3) & 0xFu, m = b & 7u;
    float mag;
    if (e == 0) mag = (float)m * 0.001953125f;                       // m * 2^-9
    else if (e == 15 && m == 7) mag = __builtin_nanf("");
    else mag = __builtin_bit_cast(float, ((e + 120u) << 23) | (m << 20));
    return __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, mag) | sign);
}

// ---- quantised epilogue of the int8 path (paper appendix on quantisation: de-quantise, bias,
// optional quantise/de-quantise pair, batch norm (unfolded as in the paper's figure, or folded by the
// caller into a multiplier and a shift), ReLU, output quantisation).
// Every step is a single binary32 operation in this order; contraction into fused
// multiply-adds is switched off so that the integer codes come out bit-exact.
// t / step as the IEEE quotient, for one divisor used many times.  With y = RN(1 / step) (one real division
// per kernel), q0 = RN(t y), r = t - step q0 (exact in a fused multiply-add) and q1 = RN(q0 + r y), q1 is the
// correctly rounded quotient (the final step of the classic FMA division sequences; it needs y correctly
// rounded, which fails only for a divisor whose significand is all ones) as long as nothing over- or
// underflows on the way.  fast: the divisor is a normal number in [2^-63, 2^63] without that significand;
// the dividend must be below 2^62 in magnitude, otherwise (and for NaN) the real division is taken.
// Quotients too small to be normal numbers are not exact, which the callers do not need: they round the
// quotient to an integer.
struct StepDiv {
    float step, rcp;
    bool fast;
};
__device__ __forceinline__ StepDiv make_step_div(float step) {
#pragma clang fp contract(off)
    StepDiv d;
    d.step = step;
    d.rcp = 1.0f / step;
    const uint32_t b = __builtin_bit_cast(uint32_t, step);
    const uint32_t e = (b >> 23) & 0xFFu;
    d.fast = e >= 64u && e <= 190u && (b & 0x7FFFFFu) != 0x7FFFFFu;
    return d;
}
__device__ __forceinline__ float step_quotient(float t, const StepDiv& d) {
#pragma clang fp contract(off)
    if (d.fast && __builtin_fabsf(t) < 0x1p62f) {
        const float q0 = t * d.rcp;
        const float r = __builtin_fmaf(-d.step, q0, t);
        return __builtin_fmaf(r, d.rcp, q0);
    }
    return t / d.step;
}

// The same for a divisor known to be `fast`, without the test of the dividend: the first product is kept
// within +-2^30 (v_med3_f32; a quotient that large saturates whatever its last bits are, and the correction
// still pushes it the right way), so that a huge or infinite dividend does not turn into NaN; a NaN dividend
// stays NaN through the remainder.
__device__ __forceinline__ float step_quotient_fast(float t, const StepDiv& d) {
#pragma clang fp contract(off)
    float q0 = t * d.rcp;
    q0 = __builtin_amdgcn_fmed3f(q0, -0x1p30f, 0x1p30f);
    const float r = __builtin_fmaf(-d.step, q0, t);
    return __builtin_fmaf(r, d.rcp, q0);
}

__device__ __forceinline__ float quantise_step(float t, const StepDiv& d) {
#pragma clang fp contract(off)
    float q = __builtin_rintf(step_quotient(t, d));  // v_rndne_f32: nearest, ties to even
    q = q < -128.0f ? -128.0f : q;
    q = q > 127.0f ? 127.0f : q;
    return q;
}

struct QuantParams {       // per-column values of one output element
    float scale, bias, mul, add;
    float mean, rinv;      // unfolded batch norm: subtract mean, multiply by rinv = 1 / sqrt(var + eps)
};

// 1 / sqrt(var + eps) as the paper's nest computes it: an addition, a correctly rounded square root and a
// correctly rounded division, one binary32 operation each
__device__ __forceinline__ float bn_rinv(float var, float eps) {
#pragma clang fp contract(off)
    float r = var + eps;
    r = __builtin_sqrtf(r);
    r = 1.0f / r;
    return r;
}

__device__ __forceinline__ float quant_value(int acc, const QuantParams& c, bool has_bias, bool has_bn, bool has_mul,
                                             bool has_add, const StepDiv& mid, int relu) {
#pragma clang fp contract(off)
    float t = (float)acc;                             // v_cvt_f32_i32: round to nearest even
    t = t * c.scale;
    if (has_bias) t = t + c.bias;
    if (mid.step > 0.0f) {
        float q = quantise_step(t, mid);
        t = q * mid.step;
    }
    if (has_bn) {                                     // then mul = gamma, add = beta
        t = t - c.mean;
        t = t * c.rinv;
    }
    if (has_mul) t = t * c.mul;
    if (has_add) t = t + c.add;
    if (relu) t = !(t <= 0.0f) ? t : 0.0f;            // greater than zero or unordered: NaN stays NaN
    return t;
}

// Branch-free form for the matrix-unit kernels: both steps `fast`; a part of the epilogue that is absent is
// given its neutral value in `c` (bias and add: -0.0f, which leaves every value and the sign of zero as they
// are; mul and rinv: 1.0f; mean: +0.0f).  Same operations in the same order as quant_value.
template <bool HAS_MID, bool HAS_BN>
__device__ __forceinline__ float quant_value_fast(int acc, const QuantParams& c, const StepDiv& mid, bool relu) {
#pragma clang fp contract(off)
    float t = (float)acc;
    t = t * c.scale;
    t = t + c.bias;
    if (HAS_MID) {
        float q = __builtin_rintf(step_quotient_fast(t, mid));
        q = q < -128.0f ? -128.0f : q;                // (compare and select: NaN stays NaN)
        q = q > 127.0f ? 127.0f : q;
        t = q * mid.step;
    }
    if (HAS_BN) {
        t = t - c.mean;
        t = t * c.rinv;
    }
    t = t * c.mul;
    t = t + c.add;
    const bool zero = (t <= 0.0f) & relu;
    return zero ? 0.0f : t;
}
// the output code; a NaN has no code that the method defines
__device__ __forceinline__ int quant_code_fast(float t, const StepDiv& out_scale) {
#pragma clang fp contract(off)
    float q = __builtin_rintf(step_quotient_fast(t, out_scale));
    q = __builtin_amdgcn_fmed3f(q, -128.0f, 127.0f);
    return (int)q;
}

__device__ __forceinline__ int8_t quant_code(float t, const StepDiv& out_scale) {
    return (int8_t)(int)quantise_step(t, out_scale);
}

template <> __device__ __forceinline__ float widen<int8_t>(int8_t v) { return (float)v; }

}  // namespace pbk
