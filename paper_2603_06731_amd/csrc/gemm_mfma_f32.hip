// fp32 instantiations of the MFMA contraction kernel (v_mfma_f32_32x32x2_f32: true fp32
// products and sums).  The kernel takes every size along k in 2-byte units, here half a value.
#include "gemm_mfma_8bit.h"

namespace pbk {

hipError_t launch_mfma_f32(const Problem& p, hipStream_t stream, int cfg, int group_m) {
    Problem q = p;
    q.K = p.K * 2;
    q.lda = p.lda * 2;
    q.ldb = p.ldb * 2;          // k-major: units; n-major: the kernel takes ldb * 2 bytes per k-row
    q.stride_a = p.stride_a * 2;
    q.stride_b = p.stride_b * 2;
    if (p.is_conv) q.conv.Cin = p.conv.Cin * 2;
    switch (cfg) {
    // (the 16-bit output type parameter is not used: fp32 operands give fp32 results)
    case 0: return launch_typed_modes<float, bf16_t, 128, 256, 32, 1, 4, 3, 2>(q, stream, group_m);
    default: return launch_typed_modes<float, bf16_t, 128, 128, 64, 2, 2, 2, 1>(q, stream, group_m);
    }
}

}  // namespace pbk
