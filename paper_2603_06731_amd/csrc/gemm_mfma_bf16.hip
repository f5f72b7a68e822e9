// bf16 instantiations of the MFMA contraction kernel.
#include "gemm_mfma_launch.h"
namespace pbk {
hipError_t launch_mfma_bf16(const Problem& p, hipStream_t stream, int cfg, int group_m) {
    return launch_config<bf16_t>(p, stream, cfg, group_m);
}
}  // namespace pbk
