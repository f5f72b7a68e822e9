// Instantiation and launch of the MFMA kernel for one element type.
// Included by one translation unit per dtype so they compile in parallel.
#pragma once
#include <atomic>
#include <cstdlib>
#include "gemm_mfma_kernel.h"

namespace pbk {

struct MfmaConfig {
    int id;
    int bm, bn, bk, wm, wn, stages;
    const char* name;
};

// Tile configurations (the static stand-in for the paper's analytical tile
// size model, Sec. 4.3): id -> workgroup tile and wave grid.
static const MfmaConfig kMfmaConfigs[] = {
    {0, 128, 256, 32, 1, 4, 3, "mfma_128x256x32_w1x4_s3_occ2"},
    {1, 128, 128, 64, 2, 2, 2, "mfma_128x128x64_w2x2_s2"},
    {2, 128, 128, 32, 2, 2, 3, "mfma_128x128x32_w2x2_s3_occ3"},     // 2, 3: measured and retired, not built
    {3, 256, 256, 32, 2, 4, 4, "mfma_256x256x32_w2x4_s4"},
    {4, 256, 256, 64, 2, 4, 2, "mfma_256x256x64_w2x4_s2"},          // 8-bit types only
    {5, 256, 256, 32, 2, 4, 4, "mfma16_256x256x32_w2x4_s4"},        // 16x16x32 MFMA blocks (16-bit types)
    {6, 128, 256, 32, 1, 4, 3, "mfma16_128x256x32_w1x4_s3_occ2"},
    {7, 256, 256, 32, 2, 4, 4, "mfma16_256x256x32_w2x4_s4_a64"},    // A staged 64 deep (plain matrices)
    {8, 256, 256, 64, 2, 4, 2, "mfma16_256x256x64_w2x4_s2"},        // int8, both operands k-major (16x16x64 blocks)
    {9, 256, 256, 32, 2, 4, 5, "mfma16_256x256x32_w2x4_a64_b6_pair"},   // as 7 with six B stages, one barrier per two k-tiles
};
static const int kNumMfmaConfigs = sizeof(kMfmaConfigs) / sizeof(kMfmaConfigs[0]);

// XCD (accelerator complex die, each with its own L2) and compute unit counts of a device,
// asked once per device.  Workgroup ids are dealt round-robin to the XCDs, which the block
// mapping undoes.
struct DeviceShape { int xcds, cus; };
inline hipError_t device_shape(int dev, DeviceShape* out) {
    static std::atomic<unsigned> cache[32];          // xcds << 16 | cus; 0 = not asked yet
    const int slot = dev & 31;
    unsigned v = cache[slot].load(std::memory_order_acquire);
    if (!v) {
        int x = 0, c = 0;
        hipError_t e = hipDeviceGetAttribute(&x, hipDeviceAttributeNumberOfXccs, dev);
        if (e != hipSuccess || x < 1) { (void)hipGetLastError(); x = 1; }
        e = hipDeviceGetAttribute(&c, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        v = ((unsigned)x << 16) | (unsigned)(c & 0xFFFF);
        cache[slot].store(v, std::memory_order_release);
    }
    out->xcds = (int)(v >> 16);
    out->cus = (int)(v & 0xFFFF);
    return hipSuccess;
}

template <typename T, typename TO, int BM, int BN, int BK, int WM, int WN, int MODE, int NSTAGE, int OCC, int MI = 32,
          int ASTG = 0>
hipError_t launch_one(const Problem& p, hipStream_t stream, int group_m) {
    constexpr int LDS_BYTES = NSTAGE * (BM * BK * 2 + BN * BK * 2);
    auto kern = gemm_mfma_kernel<T, TO, BM, BN, BK, WM, WN, MODE, NSTAGE, OCC, MI, ASTG>;
    static std::atomic<unsigned> attr_done{0};      // bit per device
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    unsigned bit = 1u << (dev & 31);
    if (!(attr_done.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done.fetch_or(bit, std::memory_order_release);
    }
    TileMap tm;
    tm.tiles_m = (p.M + BM - 1) / BM;
    tm.tiles_n = (p.N + BN - 1) / BN;
    tm.tiles_per_batch = tm.tiles_m * tm.tiles_n;
    long long total = (long long)tm.tiles_per_batch * p.batch;
    if (total <= 0 || total > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    tm.total = (int)total;
    tm.group_m = group_m < 1 ? 1 : group_m;
    DeviceShape ds;
    e = device_shape(dev, &ds);
    if (e != hipSuccess) return e;
    tm.xcds = ds.xcds;
    // hipLaunchKernel reports this launch's own status; the per-thread "last error"
    // may hold an unrelated earlier failure of another library
    Problem pa = p;
    void* args[] = {&pa, &tm};
    return hipLaunchKernel((const void*)kern, dim3((unsigned)total), dim3(WM * WN * 64), args, LDS_BYTES, stream);
}

template <typename T, int BM, int BN, int BK, int WM, int WN, int NSTAGE, int OCC = 1, int MI = 32, int ASTG = 0>
hipError_t launch_modes(const Problem& p, hipStream_t stream, int group_m) {
    if constexpr (ASTG == 2) {            // built for plain matrices (B row-major or k-major) only
        if (p.is_conv) {          // the image in 64-deep pieces: each must lie inside one filter tap
            if (p.conv.transposed || p.conv.Cin % 64 != 0) return hipErrorInvalidValue;
            return launch_one<T, T, BM, BN, BK, WM, WN, MODE_CONV, NSTAGE, OCC, MI, ASTG>(p, stream, group_m);
        }
        if (p.trans_b) return launch_one<T, T, BM, BN, BK, WM, WN, MODE_TRANS_B, NSTAGE, OCC, MI, ASTG>(p, stream, group_m);
        return launch_one<T, T, BM, BN, BK, WM, WN, MODE_DENSE, NSTAGE, OCC, MI, ASTG>(p, stream, group_m);
    } else {
    if (p.is_conv && p.conv.transposed) {
        // the transposed form is built for the two configurations the dispatcher picks
        if constexpr ((BM == 128 && BN == 256 && BK == 32) || (BM == 128 && BN == 128 && BK == 64))
            return launch_one<T, T, BM, BN, BK, WM, WN, MODE_CONVT, NSTAGE, OCC, MI>(p, stream, group_m);
        else
            return hipErrorInvalidValue;
    }
    if (p.is_conv) return launch_one<T, T, BM, BN, BK, WM, WN, MODE_CONV, NSTAGE, OCC, MI>(p, stream, group_m);
    if (p.trans_b) return launch_one<T, T, BM, BN, BK, WM, WN, MODE_TRANS_B, NSTAGE, OCC, MI>(p, stream, group_m);
    return launch_one<T, T, BM, BN, BK, WM, WN, MODE_DENSE, NSTAGE, OCC, MI, ASTG>(p, stream, group_m);
    }
}

// The 16-bit instantiations are split over several translation units (groups of configurations) so
// that they compile in parallel: MASK has bit i set where this unit builds configuration i.
// PBK_DEV_MASK (build-time, development only) removes configurations from every group.
#ifndef PBK_DEV_MASK
#define PBK_DEV_MASK 0xFFFFFFFFu
#endif
#define PBK_CASE(ID, ...) case ID: if constexpr (((MASK & (PBK_DEV_MASK)) >> ID) & 1u) return launch_modes<T, __VA_ARGS__>(p, stream, group_m); else return hipErrorInvalidValue;

template <typename T, unsigned MASK>
hipError_t launch_config(const Problem& p, hipStream_t stream, int cfg, int group_m) {
    switch (cfg) {
    PBK_CASE(0, 128, 256, 32, 1, 4, 3, 2)
    PBK_CASE(1, 128, 128, 64, 2, 2, 2)
    // 2-4 (32x32 blocks) are not built for the 16-bit types: their 16x16 twins 5-7 replaced them
    PBK_CASE(5, 256, 256, 32, 2, 4, 4, 1, 16)
    PBK_CASE(6, 128, 256, 32, 1, 4, 3, 2, 16)
    PBK_CASE(7, 256, 256, 32, 2, 4, 4, 1, 16, 1)
    PBK_CASE(9, 256, 256, 32, 2, 4, 5, 1, 16, 2)
    default: return hipErrorInvalidValue;
    }
}

// configuration groups of the 16-bit translation units (gemm_mfma_16bit.hip, once per type and group)
constexpr unsigned kGroupMask16[] = {
    (1u << 0) | (1u << 1),            // 0: the 32x32-block configurations
    (1u << 5),                        // 1: 256x256x32, plain ring
    (1u << 6),                        // 2: 128x256x32, two workgroups per compute unit
    (1u << 7),                        // 3: A staged 64 deep
    (1u << 9),                        // 4: ... with six B stages and one barrier per pair of k-tiles
};
constexpr int kNumGroups16 = sizeof(kGroupMask16) / sizeof(kGroupMask16[0]);
#define PBK_DECLARE_GROUP16(NAME, G) hipError_t launch_mfma_##NAME##_g##G(const Problem& p, hipStream_t stream, int cfg, int group_m);
PBK_DECLARE_GROUP16(bf16, 0) PBK_DECLARE_GROUP16(bf16, 1) PBK_DECLARE_GROUP16(bf16, 2) PBK_DECLARE_GROUP16(bf16, 3) PBK_DECLARE_GROUP16(bf16, 4)
PBK_DECLARE_GROUP16(f16, 0) PBK_DECLARE_GROUP16(f16, 1) PBK_DECLARE_GROUP16(f16, 2) PBK_DECLARE_GROUP16(f16, 3) PBK_DECLARE_GROUP16(f16, 4)

hipError_t launch_mfma_bf16(const Problem& p, hipStream_t stream, int cfg, int group_m);
hipError_t launch_mfma_fp8(const Problem& p, hipStream_t stream, int cfg, int group_m);
hipError_t launch_mfma_int8(const Problem& p, hipStream_t stream, int cfg, int group_m);
hipError_t launch_mfma_f32(const Problem& p, hipStream_t stream, int cfg, int group_m);
hipError_t launch_mfma_f16(const Problem& p, hipStream_t stream, int cfg, int group_m);

}  // namespace pbk
