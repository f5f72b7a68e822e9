// FP8 E5M2 instantiations of the MFMA contraction kernel.
#include "gemm_mfma_8bit.h"

namespace pbk {

hipError_t launch_mfma_fp8_e5m2(const Problem& p, hipStream_t stream, int cfg, int group_m) {
    return launch_fp8_type<fp8_e5m2_t>(p, stream, cfg, group_m);
}

}  // namespace pbk
