// bf16 / fp16 instantiations of the MFMA contraction kernel.  Compiled once per element type and group
// of tile configurations (-DPBK_16BIT_TYPE=bf16_t|f16_t -DPBK_16BIT_NAME=bf16|f16 -DPBK_GROUP=<n>), so
// that the instantiations build in parallel.
#include "gemm_mfma_launch.h"
#define PBK_CAT_(a, b, c) launch_mfma_##a##_g##b
#define PBK_CAT(a, b) PBK_CAT_(a, b, )
namespace pbk {
hipError_t PBK_CAT(PBK_16BIT_NAME, PBK_GROUP)(const Problem& p, hipStream_t stream, int cfg, int group_m) {
    return launch_config<PBK_16BIT_TYPE, kGroupMask16[PBK_GROUP]>(p, stream, cfg, group_m);
}
}  // namespace pbk
