// Generic contraction kernel: any dtype, any alignment, any leading dimension,
// transposed B, and the implicit-GEMM view of a convolution.  True fp32
// multiply-add on widened inputs.  LDS-tiled 64x64x16, 4x4 outputs per lane.
// It is the fp32 path for small or unaligned problems and the safety net for shapes the MFMA path declines.
//
// Tiling and staging follow the paper's scheme (Sec. 4.3 tiling + fast
// buffers, Sec. 4.5 on-the-fly packing of the im2col tile, partial tiles
// zero-filled) at a tile size picked for VALU rather than matrix units.
#include <hip/hip_runtime.h>
#include <type_traits>
#include "pbk_problem.h"
#include "pbk_epilogue.h"

namespace pbk {
namespace {

constexpr int GT = 64;     // tile edge in M and N
constexpr int GK = 16;     // tile depth
constexpr int GLD = GT * GK / 256;   // elements of each operand tile a thread moves
constexpr int GPAD = 4;

template <typename T> __device__ __forceinline__ float ld_elem(const T* p, int64_t i) { return widen<T>(p[i]); }

// accumulator type: exact 32-bit integers for int8 operands, fp32 otherwise
template <typename T> struct AccOf { typedef float type; };
template <> struct AccOf<int8_t> { typedef int type; };
__device__ __forceinline__ float mad(float a, float b, float c) { return fmaf(a, b, c); }
__device__ __forceinline__ int mad(int a, int b, int c) { return a * b + c; }

// A(i, k) of the implicit GEMM: im2col element, zero outside the image.
template <typename T>
__device__ __forceinline__ float conv_a(const T* x, const ConvGeom& g, int i, int k) {
    int pix = g.OH * g.OW;
    int n = i / pix;
    int r = i - n * pix;
    int oh = r / g.OW;
    int ow = r - oh * g.OW;
    int tap = k / g.Cin;
    int c = k - tap * g.Cin;
    int kh = tap / g.KW;
    int kw = tap - kh * g.KW;
    int ih, iw;
    if (g.transposed) {
        int th = oh + g.pad_h - kh * g.dil_h, tw = ow + g.pad_w - kw * g.dil_w;
        if (th < 0 || tw < 0) return 0.0f;
        ih = th / g.stride_h; iw = tw / g.stride_w;
        if (ih * g.stride_h != th || iw * g.stride_w != tw) return 0.0f;
    } else {
        ih = oh * g.stride_h - g.pad_h + kh * g.dil_h;
        iw = ow * g.stride_w - g.pad_w + kw * g.dil_w;
    }
    if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) return 0.0f;
    return widen<T>(x[(((int64_t)n * g.H + ih) * g.W + iw) * g.Cin + c]);
}

template <typename T, bool CONV>
__global__ __launch_bounds__(256) void gemm_generic_kernel(Problem p, int tiles_m, int tiles_n) {
    typedef typename AccOf<T>::type acc_t;
    // rows are 16-byte aligned (68 values): a lane's four A values and four B values of one k are
    // one 16-byte LDS read each instead of four 4-byte ones
    typedef acc_t __attribute__((ext_vector_type(4))) acc4_t;
    __shared__ __attribute__((aligned(16))) acc_t As[GK][GT + GPAD];
    __shared__ __attribute__((aligned(16))) acc_t Bs[GK][GT + GPAD];

    int bid = blockIdx.x;
    int tn = bid % tiles_n;
    int rest = bid / tiles_n;
    int tm = rest % tiles_m;
    int b = rest / tiles_m;
    int m0 = tm * GT, n0 = tn * GT;

    const T* A = (const T*)p.A + (int64_t)b * p.stride_a;
    const T* B = (const T*)p.B + (int64_t)b * p.stride_b;

    int t = threadIdx.x;
    int tx = t % 16, ty = t / 16;
    acc_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0;

    // One k-tile ahead in registers: the global loads of tile t+1 are in flight while tile t is
    // multiplied out of LDS (their latency would otherwise be paid once per k-tile).
    float a_next[GLD], b_next[GLD];
    auto fetch = [&](int k0) {
        // A tile: 64 rows x GK k; lanes run along k (contiguous in memory)
#pragma unroll
        for (int r = 0; r < GLD; ++r) {
            int e = t + 256 * r;
            int mm = e / GK, kk = e % GK;
            int gm = m0 + mm, gk = k0 + kk;
            float v = 0.0f;
            if (gm < p.M && gk < p.K) {
                if (CONV) v = conv_a<T>(A, p.conv, gm, gk);
                else v = ld_elem<T>(A, (int64_t)gm * p.lda + gk);
            }
            a_next[r] = v;
        }
        // B tile: GK k x 64 n
#pragma unroll
        for (int r = 0; r < GLD; ++r) {
            int e = t + 256 * r;
            int kk, nn;
            if (p.trans_b) { nn = e / GK; kk = e % GK; }
            else { kk = e / GT; nn = e % GT; }
            int gk = k0 + kk, gn = n0 + nn;
            float v = 0.0f;
            if (gk < p.K && gn < p.N)
                v = p.trans_b ? ld_elem<T>(B, (int64_t)gn * p.ldb + gk)
                              : ld_elem<T>(B, (int64_t)gk * p.ldb + gn);
            b_next[r] = v;
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int r = 0; r < GLD; ++r) {
            int e = t + 256 * r;
            As[e % GK][e / GK] = (acc_t)a_next[r];
            if (p.trans_b) Bs[e % GK][e / GK] = (acc_t)b_next[r];
            else Bs[e / GT][e % GT] = (acc_t)b_next[r];
        }
    };
    if (p.K > 0) fetch(0);
    for (int k0 = 0; k0 < p.K; k0 += GK) {
        stash();
        __syncthreads();
        if (k0 + GK < p.K) fetch(k0 + GK);
#pragma unroll
        for (int kk = 0; kk < GK; ++kk) {
            const acc4_t a = *(const acc4_t*)&As[kk][ty * 4];
            const acc4_t bv = *(const acc4_t*)&Bs[kk][tx * 4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = mad(a[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }

    const bool has_bias = epi_has_bias(p.epi);
    StepDiv mid_div = {}, out_div = {};
    if constexpr (std::is_same<T, int8_t>::value) { mid_div = make_step_div(p.q_mid); out_div = make_step_div(p.q_out); }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int gm = m0 + ty * 4 + i;
        if (gm >= p.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int gn = n0 + tx * 4 + j;
            if (gn >= p.N) continue;
            int64_t o = (int64_t)b * p.stride_c + (int64_t)gm * p.ldc + gn;
            if constexpr (std::is_same<T, int8_t>::value) {
                QuantParams c = {p.q_scale[gn], p.bias ? p.bias[gn] : 0.0f, p.q_mul ? p.q_mul[gn] : 1.0f,
                                 p.q_add ? p.q_add[gn] : 0.0f, p.q_mean ? p.q_mean[gn] : 0.0f,
                                 p.q_mean ? bn_rinv(p.q_var[gn], p.q_eps) : 1.0f};
                float t = quant_value(acc[i][j], c, p.bias != nullptr, p.q_mean != nullptr, p.q_mul != nullptr,
                                      p.q_add != nullptr, mid_div, p.q_relu);
                if (p.out_dtype == DT_INT8) ((int8_t*)p.C)[o] = quant_code(t, out_div);
                else ((float*)p.C)[o] = t;
                continue;
            }
            float bias = has_bias ? p.bias[gn] : 0.0f;
            float res = 0.0f;
            if (p.R) {
                const int64_t ro = (int64_t)b * p.stride_c + (int64_t)gm * p.ldr + gn;
                res = p.out_dtype == DT_F32 ? ((const float*)p.R)[ro]
                    : p.out_dtype == DT_BF16 ? (float)((const bf16_t*)p.R)[ro] : (float)((const f16_t*)p.R)[ro];
            }
            float v = apply_epilogue((float)acc[i][j], p.alpha, bias, p.epi, p.beta, res);
            if (p.out_dtype == DT_F32) ((float*)p.C)[o] = v;
            else if (p.out_dtype == DT_BF16) ((uint16_t*)p.C)[o] = to_bits16<bf16_t>(v);
            else ((uint16_t*)p.C)[o] = to_bits16<f16_t>(v);
        }
    }
}

template <typename T>
hipError_t launch_t(const Problem& p, hipStream_t stream) {
    int tiles_m = (p.M + GT - 1) / GT, tiles_n = (p.N + GT - 1) / GT;
    long long blocks = (long long)tiles_m * tiles_n * p.batch;
    if (blocks <= 0 || blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    Problem pa = p;
    void* args[] = {&pa, &tiles_m, &tiles_n};
    const void* kern = p.is_conv ? (const void*)gemm_generic_kernel<T, true>
                                 : (const void*)gemm_generic_kernel<T, false>;
    return hipLaunchKernel(kern, dim3((unsigned)blocks), dim3(256), args, 0, stream);
}

}  // namespace

hipError_t launch_generic(const Problem& p, hipStream_t stream, const char** name) {
    *name = "generic_64x64x16_fma";
    switch (p.in_dtype) {
    case DT_F32: return launch_t<float>(p, stream);
    case DT_BF16: return launch_t<bf16_t>(p, stream);
    case DT_F16: return launch_t<f16_t>(p, stream);
    case DT_FP8_E4M3: return launch_t<fp8_e4m3_t>(p, stream);
    case DT_FP8_E5M2: return launch_t<fp8_e5m2_t>(p, stream);
    case DT_INT8: return launch_t<int8_t>(p, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace pbk
