// FP8 E4M3 instantiations of the MFMA contraction kernel (v_mfma_f32_32x32x64_f8f6f4, 32 bytes
// per lane and operand), and the dispatch between the two FP8 types.
#include "gemm_mfma_8bit.h"

namespace pbk {

hipError_t launch_mfma_fp8_e4m3(const Problem& p, hipStream_t stream, int cfg, int group_m) {
    return launch_fp8_type<fp8_e4m3_t>(p, stream, cfg, group_m);
}

hipError_t launch_mfma_fp8(const Problem& p, hipStream_t stream, int cfg, int group_m) {
    return p.in_dtype == DT_FP8_E4M3 ? launch_mfma_fp8_e4m3(p, stream, cfg, group_m)
                                     : launch_mfma_fp8_e5m2(p, stream, cfg, group_m);
}

}  // namespace pbk
