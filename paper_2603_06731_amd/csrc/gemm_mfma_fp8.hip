// FP8 operands: dispatch to the translation unit that holds the operand type and the 16-bit output type
// (gemm_mfma_fp8_tu.hip); an F32 output does not use the 16-bit output type at all and takes the bf16 unit.
#include "gemm_mfma_8bit.h"

namespace pbk {

hipError_t launch_mfma_fp8_e4m3_bf16(const Problem& q, hipStream_t stream, int cfg, int group_m);
hipError_t launch_mfma_fp8_e4m3_f16(const Problem& q, hipStream_t stream, int cfg, int group_m);
hipError_t launch_mfma_fp8_e5m2_bf16(const Problem& q, hipStream_t stream, int cfg, int group_m);
hipError_t launch_mfma_fp8_e5m2_f16(const Problem& q, hipStream_t stream, int cfg, int group_m);

hipError_t launch_mfma_fp8(const Problem& p, hipStream_t stream, int cfg, int group_m) {
    const Problem q = to_k_units(p);
    const bool f16_out = q.out_dtype == DT_F16;
    if (p.in_dtype == DT_FP8_E4M3)
        return f16_out ? launch_mfma_fp8_e4m3_f16(q, stream, cfg, group_m) : launch_mfma_fp8_e4m3_bf16(q, stream, cfg, group_m);
    return f16_out ? launch_mfma_fp8_e5m2_f16(q, stream, cfg, group_m) : launch_mfma_fp8_e5m2_bf16(q, stream, cfg, group_m);
}

}  // namespace pbk
