// int8 instantiations of the MFMA contraction kernel (v_mfma_i32_32x32x32_i8, or
// v_mfma_i32_16x16x64_i8 when both operands are k-major; exact 32-bit integer accumulation,
// quantised epilogue); 16 bytes per lane and operand per MFMA, as for the 16-bit types.
#include "gemm_mfma_8bit.h"

namespace pbk {

hipError_t launch_mfma_int8(const Problem& p, hipStream_t stream, int cfg, int group_m) {
    const Problem q = to_k_units(p);
    switch (cfg) {
    case 0: return launch_typed_modes<int8_t, bf16_t, 128, 256, 32, 1, 4, 3, 2>(q, stream, group_m);
    case 1: return launch_typed_modes<int8_t, bf16_t, 128, 128, 64, 2, 2, 2, 1>(q, stream, group_m);
    case 4: return launch_typed_modes<int8_t, bf16_t, 256, 256, 64, 2, 4, 2, 1>(q, stream, group_m);
    case 8:     // 16x16x64 blocks: both operands k-major only
        if (q.trans_b && !q.is_conv)
            return launch_one<int8_t, bf16_t, 256, 256, 64, 2, 4, MODE_TRANS_B, 2, 1, 16>(q, stream, group_m);
        return launch_typed_modes<int8_t, bf16_t, 256, 256, 64, 2, 4, 2, 1>(q, stream, group_m);
    case 9:     // ... both staged 64 deep (128 values), one barrier per pair of k-tiles
        if (q.trans_b && !q.is_conv)
            return launch_one<int8_t, bf16_t, 256, 256, 32, 2, 4, MODE_TRANS_B, 5, 1, 16, 2>(q, stream, group_m);
        return launch_typed_modes<int8_t, bf16_t, 256, 256, 64, 2, 4, 2, 1>(q, stream, group_m);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace pbk
