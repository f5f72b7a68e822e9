// Eligibility test and tile-configuration choice for the MFMA path.
#include <cstdlib>
#include "gemm_mfma_launch.h"

namespace pbk {

static bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// The MFMA path moves operands in whole 16-byte pieces (8 elements): bases,
// leading dimensions, batch strides and K must keep every piece aligned and
// entirely inside or outside the matrix; likewise N for row-major B and Cin
// for the convolution (a piece must not straddle two filter taps).
bool mfma_supported(const Problem& p) {
    // 8-bit operand types (FP8, int8): 16 values per 16-byte piece
    const bool e8 = p.in_dtype == DT_FP8_E4M3 || p.in_dtype == DT_FP8_E5M2 || p.in_dtype == DT_INT8;
    const bool f32 = p.in_dtype == DT_F32;
    if (p.in_dtype != DT_BF16 && p.in_dtype != DT_F16 && !e8 && !f32) return false;
    const int per16 = e8 ? 16 : f32 ? 4 : 8;         // elements per 16-byte piece
    const int esz = e8 ? 1 : f32 ? 4 : 2;
    if (f32 && p.K >= (1 << 29)) return false;        // k sizes are doubled for the kernel
    if (p.K < per16 || p.K % per16) return false;
    if (!al16(p.A) || !al16(p.B)) return false;
    if (p.stride_a % per16 || p.stride_b % per16) return false;
    // per-lane buffer offsets are 32-bit and must stay below 2^31
    const int64_t lim = (int64_t)1 << 31;
    if (p.is_conv) {
        if ((e8 || f32) && p.conv.transposed) return false;   // the transposed form is built for 16-bit types
        if (p.conv.Cin % per16 || p.N % per16) return false;
        int64_t img = (int64_t)(p.M / (p.conv.OH * p.conv.OW)) * p.conv.H * p.conv.W * p.conv.Cin * esz;
        int64_t halo = ((int64_t)p.conv.pad_h * p.conv.W + p.conv.pad_w + p.conv.W) * p.conv.Cin * esz;
        if (img + halo >= lim) return false;
    } else {
        if (p.lda % per16 || p.ldb % per16) return false;
        if (!p.trans_b && p.N % per16) return false;
        if (256 * p.lda * esz + 256 >= lim) return false;
    }
    if (256 * p.ldb * esz + 1024 >= lim) return false;
    return true;
}

// fp32 operands take the matrix units only when there is enough work to fill the chip with
// 128-row tiles; small problems (cfg1-sized) are quicker on the generic kernel's 64x64 tiles.
bool mfma_preferred(const Problem& p) {
    if (p.in_dtype != DT_F32) return true;
    long long t = (long long)((p.M + 127) / 128) * ((p.N + 127) / 128) * p.batch;
    return p.M >= 128 && p.N >= 128 && t >= 64;
}

// 16-bit operands.  Configurations 5-7 use the 16x16x32 MFMA blocks (measured against their
// 32x32x16 twins 3, 0: 8192^3 786 against 816 us, 3x3 convolution 144 against 151 us, the
// store-bound attention-score product equal); 7 also stages A 64 deep (762 us).
static int choose_config(const Problem& p) {
    long long t = (long long)((p.M + 127) / 128) * ((p.N + 255) / 256) * p.batch;
    long long t256 = (long long)((p.M + 255) / 256) * ((p.N + 255) / 256) * p.batch;
    if (p.trans_b && !p.is_conv && p.K >= 1024) {
        // k-major B, long contraction: the 128x256 configurations are slow there (1044 us against
        // 874 us for 256x256x32 on 8192^3); short ones (K = 128) follow the general rule below
        // (9: both operands staged 64 deep, one barrier per pair of k-tiles: 715 against 800 us on 8192^3,
        // 5-7 % ahead of 5 from K = 1024 up and down to 4096^2 outputs)
        if (p.M >= 256 && p.N >= 256 && t256 >= 128) return 9;
        return 1;
    }
    // Long contractions over many tiles: one 256x256x32 workgroup per CU with a 4-stage ring.
    // Short contractions (store-dominated) and convolutions: two 128x256 workgroups per CU, whose
    // two barrier domains fill each other's bubbles.
    // (K = 1024 / 2048: the two 128x256 workgroups are 2-5 % ahead; K = 4096 and 8192: 10 % behind)
    // (9 = 7 with one barrier per two k-tiles: 8192^3 739 against 757 us, the MLP shape 711 against 726 us,
    // interleaved runs; 6 % on a 24-tile problem that is not power limited)
    // (a sweep of 6 against 9 over 256- to 4096-tile problems: 9 is 5-13 % ahead from K = 2048 up, also on one
    // round of 256 tiles (4096^2 x 3072: 78 against 86 us, 8192 x 2048 x 8192: 186 against 212 us); K = 1024
    // is a tie, below that 6 wins by up to 17 % unless the output is far larger than the last-level cache)
    if (!p.is_conv && !p.trans_b && p.M >= 256 && p.N >= 256 && t256 >= 256 && p.K >= 2048) return 9;
    // convolutions whose channel count is a multiple of 64 (the image is then staged in 64-deep pieces): 9 from one
    // round of 256x256 tiles and K = 1024 up (32x56x56x256 -> 256, 3x3: 131 against 151 us; 64x28x28x256 -> 512: 121
    // against 133 us; K = 576 equal; 1x1 filters and fewer than 100 tiles: 6 or 1 stay ahead by 10-15 %)
    if (p.is_conv && !p.conv.transposed && p.conv.Cin % 64 == 0 && p.M >= 256 && p.N >= 256 && t256 >= 256 && p.K >= 1024)
        return 9;
    if (p.M >= 128 && p.N >= 256 && t >= 256) return 6;
    return 1;
}

// 16-bit types: the translation unit (group) that holds a configuration
typedef hipError_t GroupFn(const Problem&, hipStream_t, int, int);
static hipError_t launch_group16(int cfg, GroupFn* const (&groups)[kNumGroups16], const Problem& p, hipStream_t stream, int group_m) {
    if (cfg < 0 || cfg > 31) return hipErrorInvalidValue;
    for (int g = 0; g < kNumGroups16; ++g)
        if ((kGroupMask16[g] >> cfg) & 1u) return groups[g](p, stream, cfg, group_m);
    return hipErrorInvalidValue;
}
hipError_t launch_mfma_bf16(const Problem& p, hipStream_t stream, int cfg, int group_m) {
    static GroupFn* const g[kNumGroups16] = {launch_mfma_bf16_g0, launch_mfma_bf16_g1, launch_mfma_bf16_g2,
                                             launch_mfma_bf16_g3, launch_mfma_bf16_g4};
    return launch_group16(cfg, g, p, stream, group_m);
}
hipError_t launch_mfma_f16(const Problem& p, hipStream_t stream, int cfg, int group_m) {
    static GroupFn* const g[kNumGroups16] = {launch_mfma_f16_g0, launch_mfma_f16_g1, launch_mfma_f16_g2,
                                             launch_mfma_f16_g3, launch_mfma_f16_g4};
    return launch_group16(cfg, g, p, stream, group_m);
}

hipError_t launch_mfma(const Problem& p, hipStream_t stream, int force_cfg, const char** name) {
    const bool fp8 = p.in_dtype == DT_FP8_E4M3 || p.in_dtype == DT_FP8_E5M2;
    if (p.in_dtype == DT_F32) {
        long long t = (long long)((p.M + 127) / 128) * ((p.N + 255) / 256) * p.batch;
        int c = (force_cfg == 0 || force_cfg == 1) ? force_cfg : (p.M >= 128 && p.N >= 256 && t >= 256) ? 0 : 1;
        *name = c == 0 ? "mfma_f32_128x256x16_w1x4_s3_occ2" : "mfma_f32_128x128x32_w2x2_s2";
        return launch_mfma_f32(p, stream, c, 8);
    }
    if (p.in_dtype == DT_INT8) {
        // measured: the 256x256 tile with the deep k-tile is the fastest of the three built for int8
        long long t256 = (long long)((p.M + 255) / 256) * ((p.N + 255) / 256) * p.batch;
        // (with both operands k-major the 16x16x64 blocks: 0.54 against 0.59 ms on 8192^3)
        const bool kmajor = p.trans_b && !p.is_conv;
        int c = (force_cfg == 0 || force_cfg == 1 || force_cfg == 4 || force_cfg == 8 || force_cfg == 9) ? force_cfg
                : (p.M >= 256 && p.N >= 256 && t256 >= 128) ? (kmajor ? 9 : 4) : 1;
        if ((c == 8 || c == 9) && !kmajor) c = 4;       // the 16x16 blocks are built for k-major operands only
        *name = kMfmaConfigs[c].name;
        const int gm = group_m_override() > 0 ? group_m_override() : 8;
        return launch_mfma_int8(p, stream, c, gm);
    }
    int cfg = (force_cfg >= 0 && force_cfg < kNumMfmaConfigs) ? force_cfg : choose_config(p);
    if (p.is_conv && p.conv.transposed && cfg != 0 && cfg != 1 && cfg != 6) cfg = choose_config(p);   // the ones built
    if (!fp8 && ((cfg >= 2 && cfg <= 4) || cfg == 8)) cfg = choose_config(p);   // 16-bit types: 0, 1, 5, 6, 7, 9 are built
    // 9 takes a convolution whose channel count is a multiple of 64 (not the transposed form)
    if (cfg == 9 && p.is_conv && (p.conv.transposed || p.conv.Cin % 64 != 0)) cfg = 7;
    if (fp8) {
        // the FP8 instruction consumes a 64-deep k-tile (in 2-byte units) in two steps:
        // only the 64-deep configurations are built for it
        const bool kmajor = p.trans_b && !p.is_conv;
        if (force_cfg != 1 && force_cfg != 4 && !(force_cfg == 9 && kmajor)) {       // (also a forced 5-8)
            long long t256 = (long long)((p.M + 255) / 256) * ((p.N + 255) / 256) * p.batch;
            cfg = (p.M >= 256 && p.N >= 256 && t256 >= 128) ? (kmajor ? 9 : 4) : 1;
        } else {
            cfg = force_cfg;
        }
    }
    const int group_m = group_m_override() > 0 ? group_m_override() : 8;
    *name = kMfmaConfigs[cfg].name;
    if (fp8) return launch_mfma_fp8(p, stream, cfg, group_m);
    return p.in_dtype == DT_BF16 ? launch_mfma_bf16(p, stream, cfg, group_m)
                                 : launch_mfma_f16(p, stream, cfg, group_m);
}

}  // namespace pbk
