// FP8 instantiations of the MFMA contraction kernel for ONE operand type and ONE 16-bit output type
// (v_mfma_f32_32x32x64_f8f6f4, and v_mfma_f32_16x16x128_f8f6f4 in the pair pipeline).  Compiled four times
// (E4M3 / E5M2 x bf16 / f16 output) with PBK_FP8_TYPE, PBK_FP8_OUT and the two names set, so that the units
// build in parallel.
#include "gemm_mfma_8bit.h"

#define PBK_FP8_CAT2(a, b, c) launch_mfma_fp8_##a##_##b
#define PBK_FP8_CAT(a, b) PBK_FP8_CAT2(a, b, )

namespace pbk {

// q: the problem already in 2-byte units along k
hipError_t PBK_FP8_CAT(PBK_FP8_NAME, PBK_FP8_OUTNAME)(const Problem& q, hipStream_t stream, int cfg, int group_m) {
    return launch_fp8_cfg<PBK_FP8_TYPE, PBK_FP8_OUT>(q, stream, cfg, group_m);
}

}  // namespace pbk
