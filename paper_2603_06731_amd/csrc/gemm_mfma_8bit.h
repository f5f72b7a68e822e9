// Launch of the MFMA kernel for 8-bit operand types (FP8, int8).  The kernel takes every size
// along k in 2-byte units (two values per unit): k-major tiles are then plain byte copies, and
// the n-major B tile (row-major B, convolution weights) is read with the 8-bit transposing
// LDS read.  Row strides of n-major operands stay byte counts (ldb * 2 units' worth).
#pragma once
#include "gemm_mfma_launch.h"

namespace pbk {

inline Problem to_k_units(const Problem& p) {
    Problem q = p;
    q.K = p.K / 2;
    q.lda = p.lda / 2;
    q.ldb = p.ldb / 2;          // k-major: units; n-major: the kernel multiplies by 2 again to get bytes
    q.stride_a = p.stride_a / 2;
    q.stride_b = p.stride_b / 2;
    if (p.is_conv) q.conv.Cin = p.conv.Cin / 2;
    return q;
}

template <typename T, typename TO, int BM, int BN, int BK, int WM, int WN, int NSTAGE, int OCC>
hipError_t launch_typed_modes(const Problem& q, hipStream_t stream, int group_m) {
    if (q.is_conv) return launch_one<T, TO, BM, BN, BK, WM, WN, MODE_CONV, NSTAGE, OCC>(q, stream, group_m);
    if (q.trans_b) return launch_one<T, TO, BM, BN, BK, WM, WN, MODE_TRANS_B, NSTAGE, OCC>(q, stream, group_m);
    return launch_one<T, TO, BM, BN, BK, WM, WN, MODE_DENSE, NSTAGE, OCC>(q, stream, group_m);
}

// The two tile configurations built for the FP8 types (a 64-unit k-tile = 128 values deep).
template <typename T, typename TO>
hipError_t launch_fp8_cfg(const Problem& q, hipStream_t stream, int cfg, int group_m) {
    switch (cfg) {
    case 1: return launch_typed_modes<T, TO, 128, 128, 64, 2, 2, 2, 1>(q, stream, group_m);
    case 4: return launch_typed_modes<T, TO, 256, 256, 64, 2, 4, 2, 1>(q, stream, group_m);
    case 9:     // both operands k-major: 16x16x128 blocks in the pair pipeline (one MFMA k-step per pair of k-tiles)
        if (q.trans_b && !q.is_conv)
            return launch_one<T, TO, 256, 256, 32, 2, 4, MODE_TRANS_B, 5, 1, 16, 2>(q, stream, group_m);
        return launch_typed_modes<T, TO, 256, 256, 64, 2, 4, 2, 1>(q, stream, group_m);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace pbk
