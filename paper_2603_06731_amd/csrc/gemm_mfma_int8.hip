// int8 instantiations of the MFMA contraction kernel (v_mfma_i32_32x32x32_i8, exact 32-bit
// integer accumulation, quantised epilogue).  Both operands must be k-major (trans_b): the
// staging code then only moves bytes, and the problem is handed to the kernel in 2-byte units
// (two int8 values per unit), 16 bytes per lane and operand per MFMA as for the 16-bit types.
#include "gemm_mfma_launch.h"

namespace pbk {

hipError_t launch_mfma_int8(const Problem& p, hipStream_t stream, int cfg, int group_m) {
    Problem q = p;
    q.K = p.K / 2;
    q.lda = p.lda / 2;
    q.ldb = p.ldb / 2;
    q.stride_a = p.stride_a / 2;
    q.stride_b = p.stride_b / 2;
    switch (cfg) {
    case 0: return launch_one<int8_t, bf16_t, 128, 256, 32, 1, 4, MODE_TRANS_B, 3, 2>(q, stream, group_m);
    case 1: return launch_one<int8_t, bf16_t, 128, 128, 64, 2, 2, MODE_TRANS_B, 2, 1>(q, stream, group_m);
    case 4: return launch_one<int8_t, bf16_t, 256, 256, 64, 2, 4, MODE_TRANS_B, 2, 1>(q, stream, group_m);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace pbk
