// FP8 (OCP E4M3 / E5M2) instantiations of the MFMA contraction kernel.
// Both operands must be k-major (trans_b): the staging code then only moves
// bytes, so the problem is handed to the kernel in 2-byte units (two FP8 values
// per unit) and v_mfma_f32_32x32x64_f8f6f4 consumes 32 bytes per lane and operand.
#include "gemm_mfma_launch.h"

namespace pbk {
namespace {

template <typename T, typename TO>
hipError_t launch_fp8_cfg(const Problem& q, hipStream_t stream, int cfg, int group_m) {
    switch (cfg) {
    case 1: return launch_one<T, TO, 128, 128, 64, 2, 2, MODE_TRANS_B, 2, 1>(q, stream, group_m);
    case 4: return launch_one<T, TO, 256, 256, 64, 2, 4, MODE_TRANS_B, 2, 1>(q, stream, group_m);
    default: return hipErrorInvalidValue;
    }
}

template <typename T>
hipError_t launch_fp8_out(const Problem& q, hipStream_t stream, int cfg, int group_m) {
    // an F32 output does not use the 16-bit output type at all
    if (q.out_dtype == DT_F16) return launch_fp8_cfg<T, f16_t>(q, stream, cfg, group_m);
    return launch_fp8_cfg<T, bf16_t>(q, stream, cfg, group_m);
}

}  // namespace

hipError_t launch_mfma_fp8(const Problem& p, hipStream_t stream, int cfg, int group_m) {
    Problem q = p;
    q.K = p.K / 2;
    q.lda = p.lda / 2;
    q.ldb = p.ldb / 2;
    q.stride_a = p.stride_a / 2;
    q.stride_b = p.stride_b / 2;
    return p.in_dtype == DT_FP8_E4M3 ? launch_fp8_out<fp8_e4m3_t>(q, stream, cfg, group_m)
                                     : launch_fp8_out<fp8_e5m2_t>(q, stream, cfg, group_m);
}

}  // namespace pbk
