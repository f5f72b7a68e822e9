// Small fp32 contractions (the 256^3 case of the paper's Sec. 4.3 walk-through and its kind): a few
// hundred output tiles at most, where the time is launch plus one memory latency and a tile-per-workgroup
// kernel of the usual size would leave most compute units idle.
//
// One wave per workgroup computes a 16 x 16 tile of C with v_mfma_f32_16x16x4_f32 (true binary32
// products and sums).  Nothing is staged in LDS: a lane loads its operand values straight into the
// registers the matrix instruction reads, 128 k at a time into one of two register sets, so that for
// K <= 256 every load of the tile is in flight at once.
//
// Operand layout of the instruction (k = 4 per issue): lane l supplies, for the operand whose tile index is
// l % 16, the value at k = l / 16.  The sum over k is order-free, so lane group q = l / 16 takes the k
// positions 16 J + 4 q + i (i = 0..3) of each block of 16: one 16-byte load per block from a k-major operand.
// The accumulator is computed transposed (B^T A^T), which leaves a lane with four neighbouring columns of
// one row of C: a 16-byte store.
#include <hip/hip_runtime.h>
#include "pbk_problem.h"
#include "pbk_epilogue.h"

namespace pbk {
namespace {

typedef float __attribute__((ext_vector_type(4))) f32x4s;

constexpr int SKC = 128;                 // k per register set
constexpr int SBLK = SKC / 16;           // blocks of 16 k per set

// four consecutive k of a k-major row, zero beyond kend; `vec`: the row allows 16-byte loads
__device__ __forceinline__ f32x4s ld_k4(const float* row, int k, int kend, bool ok, bool vec) {
    f32x4s v = {0.0f, 0.0f, 0.0f, 0.0f};
    if (!ok) return v;
    if (vec && k + 4 <= kend) return *(const f32x4s*)(row + k);
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (k + i < kend) v[i] = row[k + i];
    return v;
}

template <bool TRANS_B>
__global__ __launch_bounds__(64) void gemm_small_f32_kernel(Problem p, int tiles_m, int tiles_n) {
    const int lane = threadIdx.x, r = lane & 15, q = lane >> 4;
    int bid = blockIdx.x;
    const int tn = bid % tiles_n;
    bid /= tiles_n;
    const int tm = bid % tiles_m;
    const int b = bid / tiles_m;
    const int m0 = tm * 16, n0 = tn * 16;
    const float* A = (const float*)p.A + (int64_t)b * p.stride_a;
    const float* B = (const float*)p.B + (int64_t)b * p.stride_b;

    const bool a_ok = m0 + r < p.M, b_ok = n0 + r < p.N;
    const float* a_row = A + (int64_t)(a_ok ? m0 + r : 0) * p.lda;
    const bool a_vec = ((p.lda & 3) == 0) && (((uintptr_t)A & 15) == 0);      // (A includes the batch offset)
    // B: k-major (trans_b): row n of B like a row of A; otherwise column n0 + r of the k-rows
    const float* b_row = TRANS_B ? B + (int64_t)(b_ok ? n0 + r : 0) * p.ldb : B + (b_ok ? n0 + r : 0);
    const bool b_vec = TRANS_B && ((p.ldb & 3) == 0) && (((uintptr_t)B & 15) == 0);

    f32x4s av[2][SBLK], bv[2][SBLK];
    auto load = [&](int s, int kb) __attribute__((always_inline)) {
#pragma unroll
        for (int J = 0; J < SBLK; ++J) {
            const int k = kb + 16 * J + 4 * q;
            av[s][J] = ld_k4(a_row, k, p.K, a_ok, a_vec);
            if (TRANS_B) {
                bv[s][J] = ld_k4(b_row, k, p.K, b_ok, b_vec);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    bv[s][J][i] = (b_ok && k + i < p.K) ? b_row[(int64_t)(k + i) * p.ldb] : 0.0f;
            }
        }
    };
    f32x4s acc = {0.0f, 0.0f, 0.0f, 0.0f};
    auto multiply = [&](int s) __attribute__((always_inline)) {
#pragma unroll
        for (int J = 0; J < SBLK; ++J)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(bv[s][J][i], av[s][J][i], acc, 0, 0, 0);
    };
    load(0, 0);
    if (p.K > SKC) load(1, SKC);
    for (int kb = 0; kb < p.K; kb += 2 * SKC) {
        multiply(0);
        if (kb + 2 * SKC < p.K) load(0, kb + 2 * SKC);
        if (kb + SKC < p.K) {
            multiply(1);
            if (kb + 3 * SKC < p.K) load(1, kb + 3 * SKC);
        }
    }

    // lane: row m0 + r, columns n0 + 4 q .. + 3
    const int gm = m0 + r, gn = n0 + 4 * q;
    if (gm >= p.M || gn >= p.N) return;
    const bool has_bias = epi_has_bias(p.epi);
    float* c_row = (float*)p.C + (int64_t)b * p.stride_c + (int64_t)gm * p.ldc + gn;
    const float* r_row = p.R ? (const float*)p.R + (int64_t)b * p.stride_c + (int64_t)gm * p.ldr + gn : nullptr;
    f32x4s out;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const bool in = gn + e < p.N;
        const float bias = (has_bias && in) ? p.bias[gn + e] : 0.0f;
        const float res = (r_row && in) ? r_row[e] : 0.0f;
        out[e] = apply_epilogue(acc[e], p.alpha, bias, p.epi, p.beta, res);
    }
    if (gn + 4 <= p.N && (p.ldc & 3) == 0 && (((uintptr_t)p.C & 15) == 0) && ((p.stride_c & 3) == 0)) {
        *(f32x4s*)c_row = out;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (gn + e < p.N) c_row[e] = out[e];
    }
}

}  // namespace

// fp32 in and out, plain (batched) matmul with few enough 16 x 16 tiles that one wave each still beats
// larger tiles: above that the operand re-reads of so small a tile cost more than the idle units
bool small_f32_supported(const Problem& p) {
    if (p.in_dtype != DT_F32 || p.out_dtype != DT_F32 || p.is_conv) return false;
    if (p.M < 1 || p.N < 1 || p.K < 1) return false;
    const long long tiles = (long long)((p.M + 15) / 16) * ((p.N + 15) / 16) * p.batch;
    return tiles <= 0x7FFFFFFFLL;
}

bool small_f32_preferred(const Problem& p) {
    const long long tiles = (long long)((p.M + 15) / 16) * ((p.N + 15) / 16) * p.batch;
    return tiles <= 1024 && p.K <= 4096;
}

hipError_t launch_small_f32(const Problem& p, hipStream_t stream, const char** name) {
    *name = "small_f32_16x16_mfma4_wave_per_tile";
    int tiles_m = (p.M + 15) / 16, tiles_n = (p.N + 15) / 16;
    const long long blocks = (long long)tiles_m * tiles_n * p.batch;
    if (blocks <= 0 || blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    Problem pa = p;
    void* args[] = {&pa, &tiles_m, &tiles_n};
    const void* kern = p.trans_b ? (const void*)gemm_small_f32_kernel<true> : (const void*)gemm_small_f32_kernel<false>;
    return hipLaunchKernel(kern, dim3((unsigned)blocks), dim3(64), args, 0, stream);
}

}  // namespace pbk
