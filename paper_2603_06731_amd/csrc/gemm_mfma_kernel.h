// MFMA contraction kernel for gfx950: 16-bit, 8-bit or fp32 inputs, fp32 (int32) accumulation.
//
// Structure (paper Sec. 4.3 multi-level tiling and fast buffers, Sec. 4.5
// on-the-fly packing, Sec. 4.6 mapping to matrix units, App. A.2 overlap of
// copy and compute), re-designed for CDNA4:
//   workgroup tile BM x BN x BK  ->  WM x WN waves, each a (BM/WM) x (BN/WN)
//   register tile of MFMA blocks: 16x16 (v_mfma_f32_16x16x32, 16-bit types, the
//   configurations the dispatcher picks) or 32x32 (v_mfma_f32_32x32x16 for 16-bit
//   types, v_mfma_f32_32x32x64_f8f6f4 for FP8, v_mfma_i32_32x32x32_i8,
//   v_mfma_f32_32x32x2_f32); accumulators live in registers for the whole K loop.
//   Global -> LDS staging without passing through registers: every wave issues
//   buffer_load_dwordx4 ... lds, each writing 64 x 16 bytes to 1 KiB of LDS.
//   A ring of NSTAGE LDS stages: the loads of k-tiles t+1 .. t+NSTAGE-1 are in
//   flight while k-tile t is multiplied; one barrier per k-tile; a wave's loads
//   are spread between its MFMAs.  One configuration stages A 64 deep every
//   other k-tile instead, so that its loads move whole 128-byte lines.  Pieces that lie outside the matrix
//   (rows beyond M, columns beyond N, k beyond K, convolution taps in the
//   padding) are given an out-of-range buffer offset, for which the hardware
//   writes zeros to LDS: partial tiles are zero-filled for free.
//   A tile in LDS: [BM][BK] with the 16-byte chunk index XOR-swizzled by the
//   row so that the ds_read_b128 fragment reads hit distinct banks; since a
//   direct-to-LDS load writes lane i to byte 16*i, the swizzle is applied to
//   the global address each lane fetches from.
//   B tile in LDS: [BK][BN] as in memory (n contiguous); the k-contiguous
//   MFMA operand is produced by the transposing LDS read ds_read_b64_tr_b16,
//   with the 64-byte chunk index XOR-swizzled by k.  With trans_b the B tile
//   is [BN][BK] and is handled exactly like A.
//   The MFMA is issued with the operands swapped (B fragment as srcA, A
//   fragment as srcB) so each lane ends up with 4 consecutive n of one row m:
//   the epilogue (scale, bias, activation, rounding) works on 4-wide pieces in
//   registers; the rounded tile passes through the wave's LDS slice once to
//   change lane ownership and leaves as 16-byte stores along rows.
//   Rows/columns beyond M/N are never stored.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include "pbk_problem.h"
#include "pbk_epilogue.h"

namespace pbk {

typedef __attribute__((ext_vector_type(4))) int int4v;
typedef __attribute__((ext_vector_type(2))) int int2v;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(8))) short short8v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

#define PBK_LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

enum : int { MODE_DENSE = 0, MODE_TRANS_B = 1, MODE_CONV = 2, MODE_CONVT = 3 };

// buffer offsets at or above this are out of range for every descriptor we
// build (num_records = 2^31): the load returns zeros
constexpr unsigned kOob = 0x80000000u;

// One MFMA operand fragment of a lane: CH 16-byte pieces that are consecutive
// along k in memory.  16-bit types: 8 elements (v_mfma_f32_32x32x16);
// FP8: 32 elements (v_mfma_f32_32x32x64_f8f6f4).  Lanes 0-31 hold the first
// half of the instruction's k range, lanes 32-63 the second.
template <int CH> struct Frag { short8v c[CH]; };

typedef __attribute__((ext_vector_type(8))) int int8v;

template <typename T> struct MfmaOp;
template <> struct MfmaOp<bf16_t> {
    static constexpr int kChunks = 1;
    static __device__ __forceinline__ f32x16 run(const Frag<1>& a, const Frag<1>& b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a.c[0]),
                                                       __builtin_bit_cast(bf16x8, b.c[0]), c, 0, 0, 0);
    }
};
template <> struct MfmaOp<f16_t> {
    static constexpr int kChunks = 1;
    static __device__ __forceinline__ f32x16 run(const Frag<1>& a, const Frag<1>& b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a.c[0]),
                                                      __builtin_bit_cast(f16x8, b.c[0]), c, 0, 0, 0);
    }
};
// 16-bit types, 16x16 blocks: v_mfma_f32_16x16x32.  Lane l holds, of either operand, index l%16
// and the 8 consecutive k values 8 (l/16) .. 8 (l/16) + 7; of the result, column l%16 of srcB's
// index and rows 4 (l/16) + 0..3 of srcA's.  Half the accumulator traffic per flop of the 32x32
// instruction: measured 10 % faster at full clock and 17 % faster under the power cap.
template <typename T> struct MfmaOp16;
template <> struct MfmaOp16<bf16_t> {
    static __device__ __forceinline__ f32x4 run(short8v a, short8v b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct MfmaOp16<f16_t> {
    static __device__ __forceinline__ f32x4 run(short8v a, short8v b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
// int8, 16x16 blocks: v_mfma_i32_16x16x64_i8, the same 16 bytes per lane and operand (16 values)
typedef __attribute__((ext_vector_type(4))) int i32x4;
template <> struct MfmaOp16<int8_t> {
    static __device__ __forceinline__ f32x4 run(short8v a, short8v b, f32x4 c) {
        i32x4 r = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(int4v, a), __builtin_bit_cast(int4v, b),
                                                        __builtin_bit_cast(i32x4, c), 0, 0, 0);
        return __builtin_bit_cast(f32x4, r);
    }
};
__device__ __forceinline__ int8v frag_bytes32(const Frag<2>& f) {
    return __builtin_shufflevector(__builtin_bit_cast(int4v, f.c[0]), __builtin_bit_cast(int4v, f.c[1]),
                                   0, 1, 2, 3, 4, 5, 6, 7);
}
// FP8: format selectors cbsz / blgp: 0 = E4M3, 1 = E5M2; all block scales zero (= unscaled instruction)
template <> struct MfmaOp<fp8_e4m3_t> {
    static constexpr int kChunks = 2;
    static __device__ __forceinline__ f32x16 run(const Frag<2>& a, const Frag<2>& b, f32x16 c) {
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(frag_bytes32(a), frag_bytes32(b), c, 0, 0, 0, 0, 0, 0);
    }
};
template <> struct MfmaOp<fp8_e5m2_t> {
    static constexpr int kChunks = 2;
    static __device__ __forceinline__ f32x16 run(const Frag<2>& a, const Frag<2>& b, f32x16 c) {
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(frag_bytes32(a), frag_bytes32(b), c, 1, 1, 0, 0, 0, 0);
    }
};

// (FP8 has no 16-byte-fragment 16x16 instruction at its full rate; these exist so that the 16-bit pipelines
// still parse for an FP8 type: the FP8 form of the pair pipeline issues MfmaOp16x128 instead)
template <> struct MfmaOp16<fp8_e4m3_t> { static __device__ __forceinline__ f32x4 run(short8v, short8v, f32x4 c) { return c; } };
template <> struct MfmaOp16<fp8_e5m2_t> { static __device__ __forceinline__ f32x4 run(short8v, short8v, f32x4 c) { return c; } };
// FP8, 16x16 blocks: v_mfma_f32_16x16x128_f8f6f4, 32 bytes (32 values) per lane and operand: lane l supplies 32
// values of the operand row l % 16; which k they are is free as long as both operands are loaded alike
template <typename T> struct MfmaOp16x128;
template <> struct MfmaOp16x128<fp8_e4m3_t> {
    static __device__ __forceinline__ f32x4 run(int8v a, int8v b, f32x4 c) {
        return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
    }
};
template <> struct MfmaOp16x128<fp8_e5m2_t> {
    static __device__ __forceinline__ f32x4 run(int8v a, int8v b, f32x4 c) {
        return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 1, 1, 0, 0, 0, 0);
    }
};

// int8: v_mfma_i32_32x32x32_i8, 16 bytes (16 values) per lane and operand; the 32-bit integer
// accumulators travel in the same registers, typed as floats only in name
typedef __attribute__((ext_vector_type(16))) int i32x16;
template <> struct MfmaOp<int8_t> {
    static constexpr int kChunks = 1;
    static __device__ __forceinline__ f32x16 run(const Frag<1>& a, const Frag<1>& b, f32x16 c) {
        i32x16 r = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(int4v, a.c[0]), __builtin_bit_cast(int4v, b.c[0]),
                                                         __builtin_bit_cast(i32x16, c), 0, 0, 0);
        return __builtin_bit_cast(f32x16, r);
    }
};

// fp32: v_mfma_f32_32x32x2_f32 (true fp32 products and sums), one k value per lane and
// instruction: the 16-byte fragment (4 consecutive k) feeds four of them.  Lanes 0-31 hold
// k0..k0+3 and lanes 32-63 k0+4..k0+7, so instruction e contracts k0+e with k0+4+e; any
// pairing is as good as another as long as both operands use the same one.
template <> struct MfmaOp<float> {
    static constexpr int kChunks = 1;
    static __device__ __forceinline__ f32x16 run(const Frag<1>& a, const Frag<1>& b, f32x16 c) {
        const f32x4 av = __builtin_bit_cast(f32x4, a.c[0]), bv = __builtin_bit_cast(f32x4, b.c[0]);
#pragma unroll
        for (int e = 0; e < 4; ++e) c = __builtin_amdgcn_mfma_f32_32x32x2f32(av[e], bv[e], c, 0, 0, 0);
        return c;
    }
};

// How linear workgroup ids are turned into (batch, tile_m, tile_n).
// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2; ids
// are first regrouped so that every XCD owns a contiguous run, then runs are
// walked in column-major groups of `group_m` tile rows so that the tiles in
// flight on one XCD share A rows and B columns.
struct TileMap {
    int tiles_m, tiles_n, tiles_per_batch, total;
    int group_m;
    int xcds;
};

__device__ __forceinline__ void map_tile(const TileMap& tm, int bid, int& b, int& tile_m, int& tile_n) {
    int q = tm.total / tm.xcds, r = tm.total % tm.xcds;
    int xcd = bid % tm.xcds, local = bid / tm.xcds;
    int id = xcd * q + (xcd < r ? xcd : r) + local;
    b = id / tm.tiles_per_batch;
    int t = id - b * tm.tiles_per_batch;
    int per_group = tm.group_m * tm.tiles_n;
    int g = t / per_group;
    int first_m = g * tm.group_m;
    int rows = tm.tiles_m - first_m < tm.group_m ? tm.tiles_m - first_m : tm.group_m;
    int in_g = t - g * per_group;
    tile_m = first_m + in_g % rows;
    tile_n = in_g / rows;
}

// 16-byte-chunk swizzle for a [rows][BK] 16-bit tile (row = BK*2 bytes).  The term that is
// XORed into the chunk index steps every RP rows; which RP keeps a wave-wide ds_read_b128 free of
// bank conflicts depends on how the fragment spreads its lanes over rows and chunks (measured with
// the bank-conflict counter): 32-row fragments (row lane%32, chunk lane/32) need 256 bytes' worth
// of rows per step, 16-row fragments (row lane%16, chunk lane/16) half of that.
template <int BK, bool S16 = false>
__device__ __forceinline__ int kmajor_swz(int row) {
    constexpr int CPR = BK / 8;            // chunks per row
    constexpr int RP = (S16 ? 128 : 256) / (BK * 2);
    return (row / RP) % CPR;
}
template <int BK, bool S16 = false>
__device__ __forceinline__ int kmajor_offset(int row, int chunk) {
    return row * (BK * 2) + ((chunk ^ kmajor_swz<BK, S16>(row)) << 4);
}

// Byte offset inside a [BK][BN] 16-bit tile (row = BN*2 bytes) of byte `nbyte`
// of row k: 64-byte chunks XOR-swizzled by k%4, and the two 32-byte halves of a
// chunk swapped in rows with bit 3 of k set (a transposing read of the 16x16
// blocks touches rows k..k+3 and k+8..k+11 of one 32-byte column in one pass).
__device__ __forceinline__ int nmajor_half(int k) { return ((k >> 3) & 1) << 5; }
template <int BN>
__device__ __forceinline__ int nmajor_offset(int k, int nbyte) {
    return k * (BN * 2) + ((((nbyte >> 6) ^ (k & 3)) << 6) | ((nbyte & 63) ^ nmajor_half(k)));
}

// Raw buffer descriptor over [base, base + 2^31): stride 0, 32-bit data format.
__device__ __forceinline__ int4v make_rsrc(const void* base) {
    // the base is wave-uniform; readfirstlane makes that visible to the register allocator
    uint64_t a = (uint64_t)base;
    int4v r = {__builtin_amdgcn_readfirstlane((int)(uint32_t)a),
               __builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32)), (int)kOob, 0x00020000};
    return r;
}

// One wave-wide 1 KiB direct-to-LDS load: lane i -> LDS bytes [16 i, 16 i + 16)
// of the block at LDS byte address lds_addr (wave-uniform, carried in M0).
// Written as inline assembly so that the compiler does not serialise later LDS
// reads of the OTHER stage behind it; completion is awaited explicitly with
// s_waitcnt vmcnt(n) before the barrier that publishes the stage.  M0 is declared
// clobbered, so whatever else the compiler keeps there is saved around the statement.
__device__ __forceinline__ void dma16(int4v rsrc, unsigned lds_addr, unsigned voff) {
    // descriptor and LDS address are wave-uniform by construction; readfirstlane pins
    // them to scalar registers whatever the compiler's divergence analysis concluded
    rsrc[0] = __builtin_amdgcn_readfirstlane(rsrc[0]);
    rsrc[1] = __builtin_amdgcn_readfirstlane(rsrc[1]);
    rsrc[2] = __builtin_amdgcn_readfirstlane(rsrc[2]);
    rsrc[3] = __builtin_amdgcn_readfirstlane(rsrc[3]);
    lds_addr = (unsigned)__builtin_amdgcn_readfirstlane((int)lds_addr);
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_addr), "v"(voff), "s"(rsrc) : "memory", "m0");
}

__device__ __forceinline__ unsigned lds_addr_of(const char* p) {
    return (unsigned)(uintptr_t)PBK_LDS_PTR(const char, p);
}

template <int V> struct IntTag { static constexpr int value = V; };
template <bool V> struct BoolTag { static constexpr bool value = V; };
struct TailYes { static constexpr bool value = true; };
struct TailNo { static constexpr bool value = false; };

// Two floats -> two 16-bit values packed in one dword (round to nearest even).
template <typename T> __device__ __forceinline__ uint32_t pack2(float a, float b);
template <> __device__ __forceinline__ uint32_t pack2<bf16_t>(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
template <> __device__ __forceinline__ uint32_t pack2<f16_t>(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

// Epilogue of one wave: its WTM x WTN register tile -> global memory.
// AV is the accumulator vector of one MFMA block and fixes the block layout:
//   f32x16 (32x32 block): lane holds row lane%32, columns 8 g + 4 (lane/32) + 0..3 for g = 0..3;
//   f32x4  (16x16 block): lane holds row lane%16, columns 4 (lane/16) + 0..3.
template <typename T, typename AV, int FM, int FN, int WTM, int WTN, int LDS_PER_WAVE>
struct EpiCtx {
    static constexpr bool S16 = sizeof(AV) == 16;
    static constexpr int RB = S16 ? 16 : 32;       // rows (and columns) of one block
    static constexpr int G = S16 ? 1 : 4;          // 4-column pieces a lane holds per block
    static_assert(FM * RB == WTM && FN * RB == WTN, "blocks must tile the wave tile");
    const Problem& p;
    AV (&acc)[FM][FN];
    char* wlds;            // this wave's private LDS slice
    int row0, col0;        // global coordinates of the wave tile's corner
    int lane;
    int64_t c_batch;

    __device__ __forceinline__ int lrow_of(int i) const { return i * RB + (lane & (RB - 1)); }
    __device__ __forceinline__ int lcol_of(int j, int g) const {
        return S16 ? j * 16 + ((lane >> 4) << 2) : j * 32 + g * 8 + ((lane >> 5) << 2);
    }
    __device__ __forceinline__ float val(int i, int j, int g, int e) const { return acc[i][j][S16 ? e : g * 4 + e]; }

    template <int ACT, bool HAS_RES = true> __device__ __forceinline__ float act_of(float acc_v, float bias_v, float res_v = 0.0f) const {
        float t = fmaf(p.alpha, acc_v, bias_v);
        if (HAS_RES) t = fmaf(p.beta, res_v, t);
        if (ACT == 1) t = relu_keep_nan(t);
        if (ACT == 2) t = gelu_tanh_f32(t);
        return t;
    }

    // residual values R[gm][gn..gn+3] widened to float (zero where there is no residual operand);
    // vec: whole aligned 4-element pieces may be loaded at once
    template <bool OUT_F32> __device__ __forceinline__ void res4(int gm, int gn, bool vec, float (&rv)[4]) const {
        rv[0] = rv[1] = rv[2] = rv[3] = 0.0f;
        if (!p.R || gm >= p.M || gn >= p.N) return;
        const int64_t o = c_batch + (int64_t)gm * p.ldr + gn;
        if (OUT_F32) {
            if (vec) { f32x4 q = *(const f32x4*)((const float*)p.R + o); rv[0] = q[0]; rv[1] = q[1]; rv[2] = q[2]; rv[3] = q[3]; }
            else {
#pragma unroll
                for (int e = 0; e < 4; ++e) if (gn + e < p.N) rv[e] = ((const float*)p.R)[o + e];
            }
        } else {
            T h[4] = {(T)0.0f, (T)0.0f, (T)0.0f, (T)0.0f};
            if (vec) { int2v q = *(const int2v*)((const uint16_t*)p.R + o); __builtin_memcpy(h, &q, 8); }
            else {
#pragma unroll
                for (int e = 0; e < 4; ++e) if (gn + e < p.N) h[e] = ((const T*)p.R)[o + e];
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) rv[e] = (float)h[e];
        }
    }

    // bias for columns gn..gn+3 (zero where there is none)
    __device__ __forceinline__ void bias4(int gn, bool vec, float (&bv)[4]) const {
        bv[0] = bv[1] = bv[2] = bv[3] = 0.0f;
        if (!epi_has_bias(p.epi)) return;
        if (vec && gn + 3 < p.N) {
            f32x4 q = *(const f32x4*)(p.bias + gn);
            bv[0] = q[0]; bv[1] = q[1]; bv[2] = q[2]; bv[3] = q[3];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (gn + e < p.N) bv[e] = p.bias[gn + e];
        }
    }

    template <int ACT, bool OUT_F32> __device__ __forceinline__ void run() {
        constexpr int ESZ = OUT_F32 ? 4 : 2;
        constexpr int EPC = 16 / ESZ;                       // elements per 16-byte chunk
        // the coalesced path needs whole, aligned 16-byte chunks of C
        const bool fast = (p.N % EPC == 0) && (p.ldc % EPC == 0) &&
                          (((uintptr_t)p.C + (uintptr_t)c_batch * ESZ) % 16 == 0);
        const bool bias_vec = ((uintptr_t)p.bias % 16) == 0;
        // the residual operand is a compile-time property of the staged path: its loads and bounds tests
        // would otherwise sit, as branches, in front of every 4-wide piece of every epilogue
        if (!fast) run_direct<OUT_F32>(bias_vec, ACT);
        else if (p.R) run_staged<ACT, OUT_F32, true>(bias_vec);
        else run_staged<ACT, OUT_F32, false>(bias_vec);
    }

    // ---- fast path: registers -> (epilogue) -> LDS slice -> 16-byte row stores
    template <int ACT, bool OUT_F32, bool HAS_RES> __device__ __forceinline__ void run_staged(bool bias_vec) {
        constexpr int ESZ = OUT_F32 ? 4 : 2;
        constexpr int EPC = 16 / ESZ;                       // elements per 16-byte chunk
        constexpr int ROW_BYTES = WTN * ESZ;
        constexpr int CPR = ROW_BYTES / 16;                 // 16-byte chunks per row
        constexpr int RP = ROW_BYTES >= 256 ? 1 : 256 / ROW_BYTES;   // rows per 256 bytes
        constexpr int MAX_ROWS = LDS_PER_WAVE / ROW_BYTES;
        constexpr int PASS_BLOCKS = (MAX_ROWS / RB) < FM ? (MAX_ROWS / RB) : FM;   // row blocks per pass
        static_assert(PASS_BLOCKS >= 1, "LDS slice too small for one row block");
        static_assert(CPR <= 64 && 64 % CPR == 0, "row chunks must divide the wave");
        constexpr int ROWS_PER_LD = 64 / CPR;               // rows covered by one wave-wide 16-byte read
        static_assert((RB % ROWS_PER_LD) == 0, "reads must tile a row block");
        const int ld_row = lane / CPR, ld_chunk = lane % CPR;
        const bool res_vec = HAS_RES && (p.ldr % 4 == 0) &&
                             (((uintptr_t)p.R + (uintptr_t)c_batch * ESZ) % (4 * ESZ) == 0);

        // every bias value this lane needs, loaded once and together
        float bias_r[FN][G][4];
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int g = 0; g < G; ++g)
                bias4(col0 + lcol_of(j, g), bias_vec, bias_r[j][g]);

#pragma unroll
        for (int i0 = 0; i0 < FM; i0 += PASS_BLOCKS) {
            // registers -> LDS (row-major [rows][WTN], 16-byte chunks XOR-swizzled by row)
#pragma unroll
            for (int ii = 0; ii < PASS_BLOCKS; ++ii) {
                const int i = i0 + ii;
                if (i >= FM) break;
                const int lrow = lrow_of(ii);
                const int sw = (lrow / RP) % CPR;
#pragma unroll
                for (int j = 0; j < FN; ++j) {
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        const int lcol = lcol_of(j, g);
                        float v[4], rv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                        if (HAS_RES) res4<OUT_F32>(row0 + lrow_of(i), col0 + lcol, res_vec, rv);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = act_of<ACT, HAS_RES>(val(i, j, g, e), bias_r[j][g][e], rv[e]);
                        const int cbyte = lcol * ESZ;
                        char* dst = wlds + lrow * ROW_BYTES + ((((cbyte >> 4) ^ sw)) << 4) + (cbyte & 15);
                        if (OUT_F32) {
                            f32x4 w = {v[0], v[1], v[2], v[3]};
                            *(f32x4*)dst = w;
                        } else {
                            int2v w;
                            w[0] = (int)pack2<T>(v[0], v[1]);
                            w[1] = (int)pack2<T>(v[2], v[3]);
                            *(int2v*)dst = w;
                        }
                    }
                }
            }
            // LDS -> global, 16 bytes per lane, lanes running along rows; reads are
            // batched ahead of the stores so their latency is paid once per batch
            constexpr int PASS_ROWS = PASS_BLOCKS * RB;
            constexpr int NLD = PASS_ROWS / ROWS_PER_LD;
            constexpr int BATCH = NLD < 8 ? NLD : 8;
            const int gn = col0 + ld_chunk * EPC;
            const int lrow0 = i0 * RB + ld_row;                     // row inside the wave tile
            char* cptr = (char*)p.C + (c_batch + (int64_t)(row0 + lrow0) * p.ldc + gn) * ESZ;
            const int64_t cstep = (int64_t)ROWS_PER_LD * p.ldc * ESZ;
            const int rows_left = (p.M - row0 < WTM ? p.M - row0 : WTM) - lrow0;   // valid rows from lrow0 on
#pragma unroll
            for (int q0 = 0; q0 < NLD; q0 += BATCH) {
                int4v w[BATCH];
#pragma unroll
                for (int q = 0; q < BATCH; ++q) {
                    const int lrow = (q0 + q) * ROWS_PER_LD + ld_row;
                    const int sw = (lrow / RP) % CPR;
                    w[q] = *(const int4v*)(wlds + lrow * ROW_BYTES + ((ld_chunk ^ sw) << 4));
                }
#pragma unroll
                for (int q = 0; q < BATCH; ++q) {
                    if ((q0 + q) * ROWS_PER_LD < rows_left && gn < p.N)
                        *(int4v*)(cptr + (q0 + q) * cstep) = w[q];
                }
            }
        }
    }

    // ---- int8 path: the accumulators are 32-bit integers; quantised epilogue, stores straight
    // from registers (4 consecutive columns per lane: one dword of int8 codes, or 16 bytes of fp32)
    // WM_ x WN_ waves form the workgroup tile; lds_all: the workgroup's LDS (free after the k loop, at least
    // one byte per element of the tile); wm, wn: this wave's place
    // PATH 0: any parameters (a division per element and step); 1 + HAS_MID + 2 HAS_BN: both steps allow the
    // reciprocal sequence, the element code is free of branches
    template <int WM_, int WN_, int PATH> __device__ __forceinline__ void run_quant(char* lds_all, int wm, int wn) {
        constexpr bool FAST = PATH > 0, F_MID = ((PATH - 1) & 1) != 0, F_BN = ((PATH - 1) & 2) != 0;
        const bool out_i8 = p.out_dtype == DT_INT8;
        const bool has_bias = p.bias != nullptr, has_mul = p.q_mul != nullptr, has_add = p.q_add != nullptr;
        const bool has_bn = p.q_mean != nullptr;
        const StepDiv mid_div = make_step_div(p.q_mid), out_div = make_step_div(p.q_out);
        const bool relu = p.q_relu != 0;
        const int esz = out_i8 ? 1 : 4;
        const bool vec = (p.N % 4 == 0) && (p.ldc % 4 == 0) &&
                         (((uintptr_t)p.C + (uintptr_t)c_batch * esz) % (4 * esz) == 0);
        // int8 codes of the whole WORKGROUP tile pass through LDS once, so that a store instruction writes whole
        // rows of the tile (128 or 256 bytes; a wave tile alone is 64 bytes wide: half a cache line, and stores
        // of half lines ran at a fraction of the memory rate).  Needs whole aligned 16-byte chunks of C.
        constexpr int BM_ = WM_ * WTM, ROW_BYTES = WN_ * WTN;
        constexpr int CPR = ROW_BYTES / 16;
        constexpr bool CAN_STAGE = BM_ * ROW_BYTES <= WM_ * WN_ * LDS_PER_WAVE && CPR <= 64 && 64 % CPR == 0;
        const bool staged = CAN_STAGE && out_i8 && (p.N % 16 == 0) && (p.ldc % 16 == 0) &&
                            (((uintptr_t)p.C + (uintptr_t)c_batch) % 16 == 0);
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int lcol = lcol_of(j, g);
                const int gn = col0 + lcol;
                QuantParams c[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool in = gn + e < p.N;
                    c[e].scale = in ? p.q_scale[gn + e] : 0.0f;
                    c[e].bias = (in && has_bias) ? p.bias[gn + e] : (FAST ? -0.0f : 0.0f);
                    c[e].mul = (in && has_mul) ? p.q_mul[gn + e] : 1.0f;
                    c[e].add = (in && has_add) ? p.q_add[gn + e] : (FAST ? -0.0f : 0.0f);
                    c[e].mean = (in && has_bn) ? p.q_mean[gn + e] : 0.0f;
                    c[e].rinv = (in && has_bn) ? bn_rinv(p.q_var[gn + e], p.q_eps) : 1.0f;
                }
#pragma unroll
                for (int i = 0; i < FM; ++i) {
                    const int lrow = lrow_of(i);
                    const int gm = row0 + lrow;
                    if (!staged && (gm >= p.M || gn >= p.N)) continue;
                    const int64_t o = c_batch + (int64_t)gm * p.ldc + gn;
                    float t[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int a = __float_as_int(val(i, j, g, e));
                        t[e] = FAST ? quant_value_fast<F_MID, F_BN>(a, c[e], mid_div, relu)
                                    : quant_value(a, c[e], has_bias, has_bn, has_mul, has_add, mid_div, p.q_relu);
                    }
                    if (out_i8) {
                        int8_t q[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) q[e] = FAST ? (int8_t)quant_code_fast(t[e], out_div) : quant_code(t[e], out_div);
                        const unsigned w = (unsigned)(uint8_t)q[0] | ((unsigned)(uint8_t)q[1] << 8) |
                                           ((unsigned)(uint8_t)q[2] << 16) | ((unsigned)(uint8_t)q[3] << 24);
                        if (staged) {
                            const int trow = wm * WTM + lrow, tcol = wn * WTN + lcol;       // place in the workgroup tile
                            *(unsigned*)(lds_all + trow * ROW_BYTES + ((((tcol >> 4) ^ (trow % CPR))) << 4) + (tcol & 15)) = w;
                        } else if (vec) {
                            *(unsigned*)((int8_t*)p.C + o) = w;
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (gn + e < p.N) ((int8_t*)p.C)[o + e] = q[e];
                        }
                    } else if (vec) {
                        f32x4 w = {t[0], t[1], t[2], t[3]};
                        *(f32x4*)((float*)p.C + o) = w;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (gn + e < p.N) ((float*)p.C)[o + e] = t[e];
                    }
                }
            }
        }
        if constexpr (CAN_STAGE) {
            if (staged) {
                __syncthreads();              // the tile's codes are complete
                constexpr int ROWS_PER_ST = 64 / CPR;                    // tile rows per store instruction
                constexpr int ROWS_PER_WAVE = BM_ / (WM_ * WN_);
                static_assert(ROWS_PER_WAVE % ROWS_PER_ST == 0, "rows of the tile split evenly over the waves' stores");
                const int st_row = lane / CPR, st_chunk = lane % CPR;
                const int m_tile = row0 - wm * WTM, n_tile = col0 - wn * WTN;
                const int gn = n_tile + st_chunk * 16;
                const int wave_rows = (wm * WN_ + wn) * ROWS_PER_WAVE;
#pragma unroll
                for (int q = 0; q < ROWS_PER_WAVE / ROWS_PER_ST; ++q) {
                    const int trow = wave_rows + q * ROWS_PER_ST + st_row;
                    const int4v w = *(const int4v*)(lds_all + trow * ROW_BYTES + ((st_chunk ^ (trow % CPR)) << 4));
                    if (m_tile + trow < p.M && gn < p.N)
                        *(int4v*)((int8_t*)p.C + c_batch + (int64_t)(m_tile + trow) * p.ldc + gn) = w;
                }
            }
        }
    }

    // ---- general path (ragged N, unaligned C): stores straight from registers
    template <bool OUT_F32> __device__ __forceinline__ void run_direct(bool bias_vec, int act) {
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int gn = col0 + lcol_of(j, g);
                float bv[4];
                bias4(gn, bias_vec, bv);
#pragma unroll
                for (int i = 0; i < FM; ++i) {
                    const int gm = row0 + lrow_of(i);
                    if (gm >= p.M || gn >= p.N) continue;
                    const int64_t o = c_batch + (int64_t)gm * p.ldc + gn;
                    float rv[4];
                    res4<OUT_F32>(gm, gn, false, rv);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (gn + e >= p.N) break;
                        float v = fmaf(p.alpha, val(i, j, g, e), bv[e]);
                        v = fmaf(p.beta, rv[e], v);
                        if (act == 1) v = relu_keep_nan(v);
                        else if (act == 2) v = gelu_tanh_f32(v);
                        if (OUT_F32) ((float*)p.C)[o + e] = v;
                        else ((uint16_t*)p.C)[o + e] = to_bits16<T>(v);
                    }
                }
            }
        }
    }
};

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    // s_waitcnt vmcnt(N) only: vmcnt is split over bits [3:0] and [15:14]; lgkmcnt/expcnt left at maximum
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// OCC: workgroups of this kernel meant to share a CU (bounds the register budget)
// T: operand type fed to the MFMA; TO: 16-bit output type (used when out_dtype is not F32).
// Sizes BK, lda, ldb, K and the batch strides are in 2-byte units whatever T is: for the FP8
// types the host halves them (two FP8 values per unit), the staging code only moves bytes.
// MI: edge of the MFMA block, 32 (every type) or 16 (16-bit types: v_mfma_f32_16x16x32).
// ASTG 1 (16x16 blocks, plain matrices, BK = 32, four stages): A is staged 64 k deep, every other
// k-tile, so that each direct-to-LDS load moves whole 128-byte lines of A.  With 64-byte row
// pieces every line of A is requested from L2 twice (once per k-tile; measured: 1.5 times the
// L1->L2 read requests of the 64-deep configurations), and that path is as loaded as the MFMA pipe.
// ASTG 2: the same staging of A with SIX stages of B (NSTAGE = 5 sizes the LDS: 2 x 32 + 6 x 16 KiB of the 160)
// and one barrier per PAIR of k-tiles.  With a k-major B (MODE_TRANS_B) the six stages are three pieces of
// B staged 64 deep like A.  A convolution (MODE_CONV) takes the pair pipeline when Cin is a multiple of 64: a 64-deep
// piece of the image then lies inside one filter tap.
template <typename T, typename TO, int BM, int BN, int BK, int WM, int WN, int MODE, int NSTAGE, int OCC, int MI = 32,
          int ASTG = 0>
__global__ __launch_bounds__(WM * WN * 64, (OCC * WM * WN + 3) / 4) void gemm_mfma_kernel(Problem p, TileMap tmap) {
    constexpr bool S16 = MI == 16;
    constexpr bool ADBL = ASTG != 0;          // A staged 64 deep
    constexpr bool PAIRB = ASTG == 2;         // ... with one barrier per pair of k-tiles
    static_assert(!ADBL || (MI == 16 && (MODE == MODE_DENSE || (PAIRB && (MODE == MODE_TRANS_B || MODE == MODE_CONV))) &&
                            BK == 32 && NSTAGE == (PAIRB ? 5 : 4)), "ASTG: see above");
    constexpr int BKA = ADBL ? 64 : BK;          // depth of one staged piece of A
    // raised wave priority around the MFMA groups: measured +1..2.5 % for one 256x256 workgroup per CU
    // and for the convolution, -1 % for two 128x256 workgroups per CU on plain matrices
    constexpr bool PRIO = BM == 256 || MODE == MODE_CONV;
    // FP8 in the pair pipeline: one v_mfma_f32_16x16x128 per 64-deep piece of both (k-major) operands
    constexpr bool F8PAIR = PAIRB && MfmaOp<T>::kChunks == 2;
    static_assert(MI == 32 || (MI == 16 && (sizeof(T) == 2 || (std::is_same<T, int8_t>::value && MODE == MODE_TRANS_B) ||
                                            (F8PAIR && MODE == MODE_TRANS_B))),
                  "16x16 blocks are built for the 16-bit types and for 8-bit types with both operands k-major");
    constexpr bool CONVT = MODE == MODE_CONVT;               // transposed convolution: gather form
    constexpr bool CONV = MODE == MODE_CONV || CONVT;        // A is an image, rows are output pixels
    constexpr bool TRANS_B = MODE == MODE_TRANS_B;
    constexpr int NW = WM * WN;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int FM = WTM / MI, FN = WTN / MI;     // MFMA blocks of the wave tile
    constexpr int CH = MfmaOp<T>::kChunks;         // 16-byte pieces per lane per MFMA operand
    constexpr int KSUB = BK / (16 * CH);           // MFMA k-steps per k-tile
    // 8-bit element types: sizes along k are in 2-byte units, a k-row of the n-major B tile is one
    // k VALUE (so the tile has 2*BK rows of BN bytes) and is read with the 8-bit transposing LDS read
    constexpr bool E8 = sizeof(T) == 1;
    // fp32: a unit is half a value; the n-major B tile has BK/2 rows of BN floats and is read with
    // plain 4-byte LDS reads (32 lanes along n)
    constexpr bool E4 = sizeof(T) == 4;
    static_assert(sizeof(T) == 2 || MODE != MODE_CONVT, "transposed convolution is built for 16-bit types only");
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int A_BLKS = BM * BKA * 2 / 1024, B_BLKS = B_BYTES / 1024;     // 1 KiB per wave-load
    constexpr int CA = A_BLKS / NW, CB = B_BLKS / NW;
    static_assert(A_BLKS % NW == 0 && B_BLKS % NW == 0, "tile must split evenly over waves");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32x32");
    static_assert(BK == 32 || BK == 64, "BK");
    static_assert(NSTAGE >= 2 && NSTAGE <= 5, "LDS stages");
    constexpr int LOADS = CA + CB;             // direct-to-LDS loads per wave per k-tile
    static_assert((NSTAGE - 2) * LOADS < 64, "vmcnt range");
    static_assert(TRANS_B || BN == 128 || BN == 256, "n-major B tile needs BN of 128 or 256");

    extern __shared__ __attribute__((aligned(1024))) char lds[];   // NSTAGE x (A tile | B tile)

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / WN, wn = wave % WN;

    int b, tile_m, tile_n;
    map_tile(tmap, blockIdx.x, b, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // ---- per-lane source offsets of the direct-to-LDS loads -----------------
    // k-major tile ([rows][BK]): 1 KiB block = KM_ROWS rows; lane -> (row, slot)
    constexpr int KM_CPR = BK / 8;
    constexpr int KM_ROWS = 64 / KM_CPR;
    const int km_row = lane / KM_CPR, km_slot = lane % KM_CPR;
    constexpr int KMA_CPR = BKA / 8;              // the same for the staged piece of A
    constexpr int KMA_ROWS = 64 / KMA_CPR;
    const int kma_row = lane / KMA_CPR, kma_slot = lane % KMA_CPR;
    // n-major tile ([BK][BN]): 1 KiB block = NM_ROWS k-rows
    constexpr int NM_CPR = BN / 8;
    constexpr int NM_ROWS = 64 / NM_CPR;
    const int nm_row = lane / NM_CPR, nm_slot = lane % NM_CPR;
    // 8-bit n-major tile ([2 BK][BN] bytes): 1 KiB block = NM8_ROWS k-rows of BN/16 slots
    constexpr int NM8_CPR = BN / 16;
    constexpr int NM8_ROWS = 64 / NM8_CPR;
    // fp32 n-major tile ([BK/2][BN] floats): BN/4 slots per k-row
    constexpr int NM4_CPR = BN / 4;
    constexpr int NM4_ROWS = 64 / NM4_CPR;

    const char* Abase = (const char*)p.A + (int64_t)b * p.stride_a * 2;
    const char* Bbase = (const char*)p.B + (int64_t)b * p.stride_b * 2;

    unsigned a_voff[CA];       // dense / trans: byte offset from the tile's row block at k0; conv: pixel base
    int a_kofs[CA];            // k offset (elements) of the piece inside the k-tile
    int a_ih0[CA], a_iw0[CA];  // conv: top-left tap coordinates
    bool a_ok[CA];
#pragma unroll
    for (int r = 0; r < CA; ++r) {
        int blk = wave * CA + r;
        int row = blk * KMA_ROWS + kma_row;
        int chunk = kma_slot ^ kmajor_swz<BKA, S16>(row);
        a_kofs[r] = chunk * 8;
        int gm = m0 + row;
        a_ok[r] = gm < p.M;
        if (CONV) {
            int pix = p.conv.OH * p.conv.OW;
            int gmc = a_ok[r] ? gm : 0;
            int n = gmc / pix;
            int rem = gmc - n * pix;
            int oh = rem / p.conv.OW;
            int ow = rem - oh * p.conv.OW;
            if (CONVT) {
                // output row oh receives tap kh from input row (oh + pad - kh*dil) / stride, if that divides
                a_ih0[r] = oh + p.conv.pad_h;
                a_iw0[r] = ow + p.conv.pad_w;
                a_voff[r] = (unsigned)(n * p.conv.H * p.conv.W * p.conv.Cin * 2);    // image base
            } else {
                a_ih0[r] = oh * p.conv.stride_h - p.conv.pad_h;
                a_iw0[r] = ow * p.conv.stride_w - p.conv.pad_w;
                // byte offset of pixel (n, ih0, iw0), channel 0; may be "negative" (wraps), fixed up per tap
                a_voff[r] = (unsigned)(((n * p.conv.H + a_ih0[r]) * p.conv.W + a_iw0[r]) * p.conv.Cin * 2);
            }
        } else {
            a_voff[r] = a_ok[r] ? (unsigned)(row * (int)p.lda * 2 + chunk * 16) : kOob;
        }
    }
    // (pair pipeline with a k-major B: the pieces of B are 64 deep like A's, 2 CB loads per wave and PAIR)
    constexpr bool BDBL = PAIRB && MODE == MODE_TRANS_B;
    constexpr int CBP = BDBL ? 2 * CB : CB;
    unsigned b_voff[CBP];
    int b_kofs[CBP];
#pragma unroll
    for (int r = 0; r < CBP; ++r) {
        int blk = wave * CBP + r;
        if (BDBL) {
            int row = blk * KMA_ROWS + kma_row;
            int chunk = kma_slot ^ kmajor_swz<BKA, S16>(row);
            b_kofs[r] = chunk * 8;
            b_voff[r] = (n0 + row < p.N) ? (unsigned)(row * (int)p.ldb * 2 + chunk * 16) : kOob;
        } else if (TRANS_B) {
            int row = blk * KM_ROWS + km_row;
            int chunk = km_slot ^ kmajor_swz<BK, S16>(row);
            b_kofs[r] = chunk * 8;
            b_voff[r] = (n0 + row < p.N) ? (unsigned)(row * (int)p.ldb * 2 + chunk * 16) : kOob;
        } else {
            if (E8) {
                // 16-byte chunk index XOR-swizzled by the k-row (8 rows of one transposing read
                // land in 8 different bank groups); b_kofs in 2-byte units like every k size
                const int krow = blk * NM8_ROWS + lane / NM8_CPR;
                const int chunk = (lane % NM8_CPR) ^ (krow & 7);
                b_kofs[r] = krow >> 1;
                b_voff[r] = (n0 + chunk * 16 < p.N) ? (unsigned)(krow * (int)p.ldb * 2 + chunk * 16) : kOob;
                continue;
            }
            if (E4) {
                // 128-byte chunks XOR-swizzled by bit 2 of the k-row: the two rows a 4-byte read
                // touches (k and k+4, lanes 0-31 and 32-63) fall into different bank halves
                const int krow = blk * NM4_ROWS + lane / NM4_CPR;
                const int slot = lane % NM4_CPR;
                const int sslot = ((((slot >> 3) ^ ((krow >> 2) & 1))) << 3) | (slot & 7);
                b_kofs[r] = krow * 2;
                b_voff[r] = (n0 + sslot * 4 < p.N) ? (unsigned)(krow * (int)p.ldb * 2 + sslot * 16) : kOob;
                continue;
            }
            int krow = blk * NM_ROWS + nm_row;
            int c64 = (nm_slot >> 2) ^ (krow & 3);
            int nbyte = (c64 << 6) | (((nm_slot & 3) << 4) ^ nmajor_half(krow));
            b_kofs[r] = krow;
            b_voff[r] = (n0 + (nbyte >> 1) < p.N) ? (unsigned)(krow * (int)p.ldb * 2 + nbyte) : kOob;
        }
    }

    // Descriptor bases: A at (m0, 0), B at (0, n0) resp. (n0, 0); advanced by k0 per k-tile.
    const char* a_tile = CONV ? Abase : Abase + (int64_t)m0 * p.lda * 2;
    const char* b_tile = TRANS_B ? Bbase + (int64_t)n0 * p.ldb * 2 : Bbase + (int64_t)n0 * (E8 ? 1 : E4 ? 4 : 2);

    const unsigned lds_base = (unsigned)__builtin_amdgcn_readfirstlane((int)lds_addr_of(lds));

    // Convolution: filter tap (kh, kw) and first channel of the current k-tile,
    // advanced incrementally (uniform) when a k-tile lies inside one tap.
    const bool one_tap = CONV && (p.conv.Cin % BK) == 0;
    int tap_kh = 0, tap_kw = 0, tap_c = 0;

    // State of the k-tile whose loads are being issued (uniform across the wave).
    int ld_k0 = 0;
    unsigned ld_sa = 0, ld_sb = 0;
    int4v ld_ra = make_rsrc(a_tile), ld_rb = make_rsrc(b_tile);
    int ld_dh = 0, ld_dw = 0;
    unsigned ld_delta = 0;
    int ld_c = 0;              // transposed convolution, one tap per k-tile: first channel of the tile

    // Start issuing the k-tile at k0 into `stage`: descriptors rebased to k0.
    auto begin_tile = [&](int k0, int stage) {
        ld_k0 = k0;
        ld_sa = lds_base + stage * STAGE;
        ld_sb = ld_sa + A_BYTES;
        if (CONV) {
            ld_dh = tap_kh * p.conv.dil_h; ld_dw = tap_kw * p.conv.dil_w;
            ld_delta = (unsigned)(((ld_dh * p.conv.W + ld_dw) * p.conv.Cin + tap_c) * 2);
            ld_c = tap_c;
            if (one_tap) {              // advance the uniform tap state to the next k-tile
                tap_c += BK;
                if (tap_c >= p.conv.Cin) {
                    tap_c = 0;
                    if (++tap_kw == p.conv.KW) { tap_kw = 0; ++tap_kh; }
                }
            }
        } else {
            ld_ra = make_rsrc(a_tile + (int64_t)k0 * 2);
        }
        ld_rb = make_rsrc(TRANS_B ? b_tile + (int64_t)k0 * 2 : b_tile + (int64_t)k0 * p.ldb * (E8 ? 4 : E4 ? 1 : 2));
    };

    // Issue load number r (0 .. LOADS-1) of the current tile: first this wave's
    // CA pieces of A, then its CB pieces of B.  TAIL: the k-tile may reach
    // beyond K (only the last one can).
    auto issue_piece = [&](int r, auto tail_tag) {
        constexpr bool TAIL = decltype(tail_tag)::value;
        if (r < CA) {
            unsigned off;
            if (CONVT) {
                int dh, dw, c;
                if (one_tap) {
                    dh = ld_dh; dw = ld_dw; c = ld_c + a_kofs[r];
                } else {
                    int k = ld_k0 + a_kofs[r];
                    int tap = k / p.conv.Cin;
                    c = k - tap * p.conv.Cin;
                    int kh = tap / p.conv.KW;
                    int kw = tap - kh * p.conv.KW;
                    dh = kh * p.conv.dil_h; dw = kw * p.conv.dil_w;
                }
                const int th = a_ih0[r] - dh, tw = a_iw0[r] - dw;
                const int ih = th / p.conv.stride_h, iw = tw / p.conv.stride_w;
                bool ok = a_ok[r] && th >= 0 && tw >= 0 && ih * p.conv.stride_h == th && iw * p.conv.stride_w == tw &&
                          ih < p.conv.H && iw < p.conv.W;
                if (TAIL) ok = ok && (ld_k0 + a_kofs[r] < p.K);
                off = ok ? a_voff[r] + (unsigned)(((ih * p.conv.W + iw) * p.conv.Cin + c) * 2) : kOob;
            } else if (CONV) {
                int dh, dw;
                if (one_tap) {
                    dh = ld_dh; dw = ld_dw;
                    off = a_voff[r] + ld_delta + (unsigned)(a_kofs[r] * 2);
                } else {
                    int k = ld_k0 + a_kofs[r];
                    int tap = k / p.conv.Cin;
                    int c = k - tap * p.conv.Cin;
                    int kh = tap / p.conv.KW;
                    int kw = tap - kh * p.conv.KW;
                    dh = kh * p.conv.dil_h; dw = kw * p.conv.dil_w;
                    off = a_voff[r] + (unsigned)(((dh * p.conv.W + dw) * p.conv.Cin + c) * 2);
                }
                int ih = a_ih0[r] + dh, iw = a_iw0[r] + dw;
                bool ok = a_ok[r] && ih >= 0 && ih < p.conv.H && iw >= 0 && iw < p.conv.W;
                if (TAIL) ok = ok && (ld_k0 + a_kofs[r] < p.K);
                off = ok ? off : kOob;
            } else {
                off = a_voff[r];
                if (TAIL && ld_k0 + a_kofs[r] >= p.K) off = kOob;
            }
            dma16(ld_ra, ld_sa + (wave * CA + r) * 1024, off);
        } else {
            const int rb = r - CA;
            unsigned off = b_voff[rb];
            if (TAIL && ld_k0 + b_kofs[rb] >= p.K) off = kOob;
            dma16(ld_rb, ld_sb + (wave * CB + rb) * 1024, off);
        }
    };
    auto issue_loads = [&](int k0, int stage, auto tail_tag) {
        begin_tile(k0, stage);
#pragma unroll
        for (int r = 0; r < CA + CB; ++r) issue_piece(r, tail_tag);
    };

    // ---- per-lane fragment read offsets -----------------------------------
    // A fragment (32 rows x 16 k): lane -> row lane%32, k-chunk lane/32 of the 2 in the k16 step
    const int frag_row = lane & 31, frag_kc = lane >> 5;
    // B via transposing read: 16-lane block -> 16 n; lane -> k row (lane%16)/4, n piece lane%4
    const int tr_k = ((lane & 15) >> 2) + ((lane >> 5) << 3);
    const int tr_nbyte = ((((lane >> 4) & 1) << 4) + ((lane & 3) << 2)) * 2;
    // 8-bit transposing read (ds_read_b64_tr_b8): within a 16-lane block, lane i addresses 8 bytes of
    // k-row i/2 at n-piece i%2 and receives, for n = i, the 8 consecutive k of the block's 8 rows
    const int tr8_row = (lane & 15) >> 1;                                   // k-row within the 8 (= swizzle term)
    const int tr8_n = (((lane >> 4) & 1) << 4) + ((lane & 1) << 3);         // n offset within the 32 of a fragment
    const int tr8_half = lane >> 5;

    typedef typename std::conditional<S16, f32x4, f32x16>::type AccV;
    AccV acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < (S16 ? 4 : 16); ++e) acc[i][j][e] = 0.0f;

    // Wait until at most `newer` whole k-tiles of this wave's loads are still in
    // flight (loads complete in order, so everything older has landed).
    auto wait_newer = [&](int newer) {
        switch (newer) {
        case 0: wait_vmcnt<0>(); break;
        case 1: wait_vmcnt<LOADS>(); break;
        case 2: wait_vmcnt<(NSTAGE > 3 ? 2 : 0) * LOADS>(); break;
        default: wait_vmcnt<(NSTAGE > 4 ? 3 : 0) * LOADS>(); break;
        }
    };

    // ---- main loop: NSTAGE LDS stages; the loads of k-tiles t+1 .. t+NSTAGE-1
    // are in flight while k-tile t is multiplied; one barrier per k-tile.
    // prime(): first fragment reads of k-tile 0; run_tile(...): one k-tile (see tile_body).
    const int KT = (p.K + BK - 1) / BK;       // k-tiles
    const int KF = p.K / BK;                  // of which full
    // pairs_tag true: the steady state runs k-tiles in pairs and tells run_tile which of the pair
    // it is (phase 1, 2; 0 = a tile on its own), for pipelines whose register buffers alternate
    // from one tile to the next.
    auto main_loop = [&](auto&& prime, auto&& run_tile, auto pairs_tag) {
        constexpr bool PAIRS = decltype(pairs_tag)::value;
        if (KT <= 0) return;
        int issued = 0;                        // k-tiles whose loads have been issued
        int slot_in = 0;                       // stage the next issued tile goes to
        auto issue_next = [&](auto tail_tag) {
            issue_loads(issued * BK, slot_in, tail_tag);
            ++issued;
            slot_in = (slot_in + 1 == NSTAGE) ? 0 : slot_in + 1;
        };
        while (issued < NSTAGE - 1 && issued < KT) {
            if (issued < KF) issue_next(TailNo{}); else issue_next(TailYes{});
        }
        wait_newer(issued - 1);
        __syncthreads();
        prime();
        int kt = 0, slot = 0;
        // steady state: every issued tile is full, NSTAGE-2 younger tiles stay in flight
        auto steady_tile = [&](auto phase_tag) {
            begin_tile(issued * BK, slot_in);          // its loads are issued between the MFMAs
            ++issued;
            slot_in = (slot_in + 1 == NSTAGE) ? 0 : slot_in + 1;
            const int nslot = (slot + 1 == NSTAGE) ? 0 : slot + 1;
            run_tile(slot, nslot, true, IntTag<NSTAGE - 2>{}, 0, BoolTag<true>{}, phase_tag);
            slot = nslot;
            ++kt;
        };
        if (PAIRS) {
            while (issued + 1 < KF) {
                steady_tile(IntTag<1>{});
                steady_tile(IntTag<2>{});
            }
        }
        while (issued < KF) steady_tile(IntTag<0>{});
        // drain: a possibly ragged last tile, then nothing left to issue
        for (; kt < KT; ++kt) {
            if (issued < KT) issue_next(TailYes{});
            const int nslot = (slot + 1 == NSTAGE) ? 0 : slot + 1;
            run_tile(slot, nslot, kt + 1 < KT, IntTag<-1>{}, issued - (kt + 2), BoolTag<false>{}, IntTag<0>{});
            slot = nslot;
        }
    };

    if constexpr (!S16) {
        // one fragment: A rows block i, B columns block j of k16 step ks
        auto read_a1 = [&](const char* sa, int ks, int i) -> Frag<CH> {
            Frag<CH> f;
            int row = wm * WTM + i * 32 + frag_row;
    #pragma unroll
            for (int c = 0; c < CH; ++c)
                f.c[c] = *(const short8v*)(sa + kmajor_offset<BK>(row, (ks * 2 + frag_kc) * CH + c));
            return f;
        };
        auto read_b1 = [&](const char* sb, int ks, int j) -> Frag<CH> {
            Frag<CH> f;
            if (TRANS_B) {
                int row = wn * WTN + j * 32 + frag_row;
    #pragma unroll
                for (int c = 0; c < CH; ++c)
                    f.c[c] = *(const short8v*)(sb + kmajor_offset<BK>(row, (ks * 2 + frag_kc) * CH + c));
            } else if (E4) {
                // column n = lane%32, k = 8 ks + 4 (lane/32) + e for e = 0..3: four 4-byte reads
                const int nbyte = (wn * WTN + j * 32 + frag_row) * 4;
                const char* r0 = sb + (ks * 8 + frag_kc * 4) * (BN * 4) + ((((nbyte >> 7) ^ frag_kc)) << 7) + (nbyte & 127);
                int4v w;
    #pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = *(const int*)(r0 + e * (BN * 4));
                f.c[0] = __builtin_bit_cast(short8v, w);
            } else if (E8) {
                // a lane's fragment: 16*CH consecutive k of column n = lane%32, half lane/32 of the step
                const int nb = wn * WTN + j * 32 + tr8_n;
                const int kbase = (ks * 2 + tr8_half) * (16 * CH) + tr8_row;
    #pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const char* r0 = sb + (kbase + c * 16) * BN + ((((nb >> 4) ^ tr8_row)) << 4) + (nb & 15);
                    int2v lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32(PBK_LDS_PTR(int2v, r0));
                    int2v hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32(PBK_LDS_PTR(int2v, r0 + 8 * BN));
                    int4v w = {lo[0], lo[1], hi[0], hi[1]};
                    f.c[c] = __builtin_bit_cast(short8v, w);
                }
            } else {
                int nbyte = (wn * WTN + j * 32) * 2 + tr_nbyte;
                int k = ks * 16 + tr_k;
                short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    PBK_LDS_PTR(short4v, sb + nmajor_offset<BN>(k, nbyte)));
                short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    PBK_LDS_PTR(short4v, sb + nmajor_offset<BN>(k + 4, nbyte)));
                f.c[0] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
            return f;
        };
        auto read_a = [&](const char* sa, int ks, Frag<CH> (&af)[FM]) {
    #pragma unroll
            for (int i = 0; i < FM; ++i) af[i] = read_a1(sa, ks, i);
        };
        auto read_b = [&](const char* sb, int ks, Frag<CH> (&bf)[FN]) {
    #pragma unroll
            for (int j = 0; j < FN; ++j) bf[j] = read_b1(sb, ks, j);
        };
        static_assert(FM + FN <= FM * FN, "a step has at least as many MFMA groups as fragments to read under it");

        // Fragments are double-buffered in registers across k16 steps AND across
        // k-tiles: the reads of step ks+1 go, one fragment at a time, between the MFMAs
        // of step ks (mid(k) runs after MFMA group k), and the first fragments of the
        // next k-tile are read (after the barrier that publishes its stage) between the
        // MFMAs of this tile's last step: the matrix pipe restarts right after the
        // barrier instead of after a burst of reads.
        Frag<CH> af[2][FM], bf[2][FN];
        auto mfma_step = [&](int cur, auto&& mid) {
    #pragma unroll
            for (int i = 0; i < FM; ++i)
    #pragma unroll
                for (int j = 0; j < FN; ++j) {
                    acc[i][j] = MfmaOp<T>::run(bf[cur][j], af[cur][i], acc[i][j]);
                    mid(i * FN + j);
                }
        };
        // Same, with this wave's loads of the tile being fetched spread evenly between
        // the MFMAs of the whole k-tile (one every GAP MFMAs) instead of issued in one
        // burst: a burst fills the memory pipeline's queue and stalls the wave in front
        // of its MFMAs.  EARLY of the LOADS pieces are issued before the wait+barrier of
        // the k-tile, the rest under its last MFMA group.
        constexpr int MFMA_PER_TILE = KSUB * FM * FN;
        constexpr int MFMA_BEFORE_WAIT = (KSUB - 1) * FM * FN;
        // with two stages the tile being fetched is the very next one: everything goes before the wait
        constexpr int SPAN = NSTAGE >= 3 ? MFMA_PER_TILE : MFMA_BEFORE_WAIT;
        // piece r is issued right after MFMA number r*SPAN/LOADS of the k-tile
        constexpr int EARLY = (MFMA_BEFORE_WAIT * LOADS + SPAN - 1) / SPAN < LOADS
                                  ? (MFMA_BEFORE_WAIT * LOADS + SPAN - 1) / SPAN : LOADS;
        static_assert(NSTAGE >= 3 || EARLY == LOADS, "two stages: all pieces must precede the wait");
        auto mfma_step_loading = [&](int cur, int ks, auto&& mid) {
    #pragma unroll
            for (int i = 0; i < FM; ++i)
    #pragma unroll
                for (int j = 0; j < FN; ++j) {
                    acc[i][j] = MfmaOp<T>::run(bf[cur][j], af[cur][i], acc[i][j]);
                    mid(i * FN + j);
                    const int idx = (ks * FM + i) * FN + j;         // MFMA number within the k-tile
    #pragma unroll
                    for (int r = 0; r < LOADS; ++r) {
                        if ((r * SPAN) / LOADS == idx) {
                            issue_piece(r, TailNo{});
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                }
        };
        static_assert(KSUB % 2 == 0, "fragment buffer parity assumes an even number of k16 steps");

        // One k-tile.  have_next: publish the next tile's stage (wait for this
        // wave's pieces, barrier) and start reading it under the last MFMA group.
        // NEWER >= 0: compile-time count of younger k-tiles in flight; -1: `newer_rt`.
        auto tile_body = [&](int stage, int next_stage, bool have_next, auto newer_tag, int newer_rt, auto spread_tag) {
            constexpr int NEWER = decltype(newer_tag)::value;
            constexpr bool SPREAD = decltype(spread_tag)::value;
            const char* sa = lds + stage * STAGE;
            const char* sb = sa + A_BYTES;
    #pragma unroll
            for (int ks = 0; ks < KSUB - 1; ++ks) {
                auto mid = [&](int k) {
                    if (k < FM) af[(ks + 1) & 1][k] = read_a1(sa, ks + 1, k);
                    else if (k < FM + FN) bf[(ks + 1) & 1][k - FM] = read_b1(sb, ks + 1, k - FM);
                    if (k < FM + FN) __builtin_amdgcn_sched_barrier(0);
                };
                if (PRIO) __builtin_amdgcn_s_setprio(2);
                if (SPREAD) mfma_step_loading(ks & 1, ks, mid); else mfma_step(ks & 1, mid);
                if (PRIO) __builtin_amdgcn_s_setprio(0);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (have_next) {
                // steady state: NEWER-1 whole younger tiles plus the EARLY pieces just issued may stay in flight
                if (NEWER >= 0) wait_vmcnt<(SPREAD && NSTAGE >= 3 ? (NEWER >= 1 ? NEWER - 1 : 0) * LOADS + EARLY : (NEWER >= 0 ? NEWER : 0) * LOADS)>();
                else wait_newer(newer_rt);
                __syncthreads();          // everyone's pieces landed; everyone is done reading `stage`
            }
            const char* na = lds + next_stage * STAGE;
            auto mid_next = [&](int k) {
                if (!have_next) return;
                if (k < FM) af[0][k] = read_a1(na, 0, k);
                else if (k < FM + FN) bf[0][k - FM] = read_b1(na + A_BYTES, 0, k - FM);
                if (k < FM + FN) __builtin_amdgcn_sched_barrier(0);
            };
            if (PRIO) __builtin_amdgcn_s_setprio(2);
            if (SPREAD) mfma_step_loading((KSUB - 1) & 1, KSUB - 1, mid_next); else mfma_step((KSUB - 1) & 1, mid_next);
            if (PRIO) __builtin_amdgcn_s_setprio(0);
            __builtin_amdgcn_sched_barrier(0);
        };

        main_loop([&]() { read_a(lds, 0, af[0]); read_b(lds + A_BYTES, 0, bf[0]); },
                  [&](int stage, int next_stage, bool have_next, auto newer_tag, int newer_rt, auto spread_tag, auto) {
                      tile_body(stage, next_stage, have_next, newer_tag, newer_rt, spread_tag);
                  }, BoolTag<false>{});
    } else {
        // ---- 16x16 blocks.  A k32 step of the wave tile is split into two halves of its rows: the
        // pipeline step s = 2 kq + h multiplies rows half h of k32-step kq.  A fragments are
        // double-buffered per step, B fragments per k32 step (both halves use them), so only
        // half of the A fragments of a step are live at a time.
        constexpr int KQ = BK / 32;                // k32 steps per k-tile
        constexpr int NSTEP = 2 * KQ;
        constexpr int FMH = FM / 2;                // A fragments (16 rows each) per half
        static_assert(FM % 2 == 0, "wave tile rows must split into two halves of 16-row blocks");
        const int f16_row = lane & 15, f16_kc = lane >> 4;
        // transposing read: 16-lane block q covers k rows 8q..8q+3 (second read: +4); lane -> row (lane%16)/4, n piece lane%4
        const int t16_k = ((lane & 15) >> 2) + ((lane >> 4) << 3);
        const int t16_nbyte = (lane & 3) * 8;
        short8v af[2][FMH], bf[2][FN];
        // byte offset of this lane's first transposing read for B block j of k32 step 0; the second
        // read (k + 4) and further k32 steps (k + 32 kq) keep the swizzle terms: constant offsets
        int b_off[FN];
#pragma unroll
        for (int j = 0; j < FN; ++j) b_off[j] = nmajor_offset<BN>(t16_k, (wn * WTN + j * 16) * 2 + t16_nbyte);
        // one fragment: A rows block i of step s; B columns block j of k32 step kq
        auto read_a1 = [&](const char* sa, int s, int i) -> short8v {
            const int kq = s >> 1, h = s & 1;
            const int row = wm * WTM + (h * FMH + i) * 16 + f16_row;
            return *(const short8v*)(sa + kmajor_offset<BK, true>(row, kq * 4 + f16_kc));
        };
        auto read_b1 = [&](const char* sb, int kq, int j) -> short8v {
            if (TRANS_B) {
                const int row = wn * WTN + j * 16 + f16_row;
                return *(const short8v*)(sb + kmajor_offset<BK, true>(row, kq * 4 + f16_kc));
            } else {
                const char* r0 = sb + b_off[j] + kq * 32 * (BN * 2);
                short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PBK_LDS_PTR(short4v, r0));
                short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PBK_LDS_PTR(short4v, r0 + 4 * (BN * 2)));
                return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        };
        auto read_a = [&](const char* sa, int s, short8v (&dst)[FMH]) {
#pragma unroll
            for (int i = 0; i < FMH; ++i) dst[i] = read_a1(sa, s, i);
        };
        auto read_b = [&](const char* sb, int kq, short8v (&dst)[FN]) {
#pragma unroll
            for (int j = 0; j < FN; ++j) dst[j] = read_b1(sb, kq, j);
        };
        static_assert(FMH + FN <= FMH * FN, "a step has at least as many MFMAs as fragments to read under it");
        constexpr int MFMA_PER_TILE = NSTEP * FMH * FN;
        constexpr int MFMA_BEFORE_WAIT = (NSTEP - 1) * FMH * FN;
        constexpr int SPAN = NSTAGE >= 3 ? MFMA_PER_TILE : MFMA_BEFORE_WAIT;
        constexpr int EARLY = (MFMA_BEFORE_WAIT * LOADS + SPAN - 1) / SPAN < LOADS
                                  ? (MFMA_BEFORE_WAIT * LOADS + SPAN - 1) / SPAN : LOADS;
        static_assert(NSTAGE >= 3 || EARLY == LOADS, "two stages: all pieces must precede the wait");
        // the MFMAs of step s; mid(k) runs after MFMA number k of the step (the fragment reads of the next
        // step go there, one at a time: nothing waits for them before the next step, and the matrix pipe
        // restarts right after a barrier instead of after a burst of reads; measured 3.6-4 % on 8192^3);
        // SPREAD: this wave's loads of the tile being fetched are issued between the MFMAs as well
        auto mfma_step = [&](int s, int bcur, auto spread_tag, auto&& mid) {
            constexpr bool SPREAD = decltype(spread_tag)::value;
            const int h = s & 1;
#pragma unroll
            for (int i = 0; i < FMH; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    acc[h * FMH + i][j] = MfmaOp16<T>::run(bf[bcur][j], af[s & 1][i], acc[h * FMH + i][j]);
                    mid(i * FN + j);
                    if (SPREAD) {
                        const int idx = (s * FMH + i) * FN + j;         // MFMA number within the k-tile
#pragma unroll
                        for (int r = 0; r < LOADS; ++r) {
                            if ((r * SPAN) / LOADS == idx) {
                                issue_piece(r, TailNo{});
                                __builtin_amdgcn_sched_barrier(0);
                            }
                        }
                    }
                }
        };
        if constexpr (ADBL) {
            // ---- A staged 64 deep.  LDS: two pieces of A ([BM][64 k], the 64-deep k-major layout), then
            // four stages of B.  k-tile t reads half t%2 of A piece (t/2)%2 and B stage t%4.  While an even
            // tile t is multiplied the wave issues A(t+2, t+3) (its piece was last read by tile t-1) and
            // B(t+3); while an odd tile, B(t+3) only.  The A loads of a tile come first in issue order.
            constexpr int AP_BYTES = BM * 128;
            constexpr int B_REGION = 2 * AP_BYTES;
            static_assert(B_REGION + (PAIRB ? 6 : 4) * B_BYTES == NSTAGE * STAGE, "LDS footprint: NSTAGE plain stages");
            auto a_lds = [&](int t) { return ((t >> 1) & 1) * AP_BYTES; };
            auto b_lds = [&](int t) { return B_REGION + (t & 3) * B_BYTES; };
            int4v ad_ra = make_rsrc(a_tile), ad_rb = make_rsrc(b_tile);
            unsigned ad_sa = 0, ad_sb = 0;
            int ad_ka = 0, ad_kb = 0;
            // convolution: tap offsets of the piece being issued (uniform: the whole 64-deep piece lies in one tap)
            int ad_dh = 0, ad_dw = 0;
            unsigned ad_delta = 0;
            auto begin_a = [&](int k0, int dst) {
                ad_ka = k0; ad_sa = lds_base + dst;
                if (CONV) {
                    const int tap = k0 / p.conv.Cin, c = k0 - tap * p.conv.Cin;
                    const int kh = tap / p.conv.KW, kw = tap - kh * p.conv.KW;
                    ad_dh = kh * p.conv.dil_h; ad_dw = kw * p.conv.dil_w;
                    ad_delta = (unsigned)(((ad_dh * p.conv.W + ad_dw) * p.conv.Cin + c) * 2);
                } else {
                    ad_ra = make_rsrc(a_tile + (int64_t)k0 * 2);
                }
            };
            auto begin_b = [&](int k0, int dst) {
                ad_kb = k0; ad_sb = lds_base + dst;
                ad_rb = make_rsrc(TRANS_B ? b_tile + (int64_t)k0 * 2 : b_tile + (int64_t)k0 * p.ldb * 2);
            };
            auto issue_a = [&](int r, auto tail_tag) {
                unsigned off = a_voff[r];
                if (CONV) {
                    off = a_voff[r] + ad_delta + (unsigned)(a_kofs[r] * 2);
                    const int ih = a_ih0[r] + ad_dh, iw = a_iw0[r] + ad_dw;
                    const bool ok = a_ok[r] && ih >= 0 && ih < p.conv.H && iw >= 0 && iw < p.conv.W;
                    off = ok ? off : kOob;
                }
                if (decltype(tail_tag)::value && ad_ka + a_kofs[r] >= p.K) off = kOob;
                dma16(ad_ra, ad_sa + (wave * CA + r) * 1024, off);
            };
            auto issue_b = [&](int rb, auto tail_tag) {
                unsigned off = b_voff[rb];
                if (decltype(tail_tag)::value && ad_kb + b_kofs[rb] >= p.K) off = kOob;
                dma16(ad_rb, ad_sb + (wave * CBP + rb) * 1024, off);
            };
            // A fragments of rows half `rh` from half `h` of the piece at sa
            auto read_a2 = [&](const char* sa, int h, int rh, short8v (&dst)[FMH]) {
#pragma unroll
                for (int i = 0; i < FMH; ++i) {
                    const int row = wm * WTM + (rh * FMH + i) * 16 + f16_row;
                    dst[i] = *(const short8v*)(sa + kmajor_offset<64, true>(row, h * 4 + f16_kc));
                }
            };
            if constexpr (PAIRB) {
                // ---- one barrier per PAIR of k-tiles.  LDS: the two pieces of A, then six stages of B; k-tile t
                // reads half t%2 of A piece (t/2)%2 and B stage t%6.  A pair is four quarters of QM MFMAs (tile,
                // rows half).  Its barrier stands in front of the LAST quarter, when every LDS read of the pair has
                // been issued; the next pair's first fragments are read under that last quarter.  Loads: B of pair
                // p+2 (its stages were last read by pair p-1, which ended at the previous barrier) goes out during
                // the first three quarters of pair p, A of pair p+2 (into the piece pair p has just finished with)
                // during the last quarter.  A wave's loads complete in issue order -- B(p+1), A(p+1), B(p+2),
                // A(p+2), ... -- so at the barrier of pair p all but the 2 CB loads of B(p+2) must have landed.
                constexpr int NBS = 6;
                constexpr int QM = FMH * FN;
                static_assert(QM % CA == 0 && (3 * QM) % (4 * CB) == 0, "load positions");
                auto stage_add = [](int sidx, int d) { const int r = sidx + d; return r >= NBS ? r - NBS : r; };
                // (k-major B: stages 2i and 2i+1 are the halves of the 64-deep piece i)
                auto b_at = [&](int sidx) { return BDBL ? B_REGION + (sidx >> 1) * 2 * B_BYTES : B_REGION + sidx * B_BYTES; };
                // B fragment j of the k-tile in stage sidx
                auto read_bs = [&](int sidx, int j) -> short8v {
                    if (BDBL) {
                        const int row = wn * WTN + j * 16 + f16_row;
                        return *(const short8v*)(lds + b_at(sidx) + kmajor_offset<64, true>(row, (sidx & 1) * 4 + f16_kc));
                    } else {
                        return read_b1(lds + b_at(sidx), 0, j);
                    }
                };
                int bstage = 0;                  // B stage of the even tile of the current pair
                int pair_burst = 0;              // drain: loads issued at the start of the current pair
                auto a_frag = [&](const char* sa, int h, int rh, int i) -> short8v {
                    const int row = wm * WTM + (rh * FMH + i) * 16 + f16_row;
                    return *(const short8v*)(sa + kmajor_offset<64, true>(row, h * 4 + f16_kc));
                };
                auto prio_up = [&]() { if (PRIO) __builtin_amdgcn_s_setprio(2); };
                auto prio_down = [&]() { if (PRIO) __builtin_amdgcn_s_setprio(0); __builtin_amdgcn_sched_barrier(0); };
                if constexpr (F8PAIR) {
                    // ---- FP8: a pair of k-tiles (128 values) is ONE k-step of v_mfma_f32_16x16x128.  A pair is two
                    // halves of QM MFMAs (rows half 0, rows half 1); the barrier stands between them, when the A
                    // fragments of rows half 1 have been read.  B of pair p+2 goes out during the first half, A of pair
                    // p+2 during the second; the next pair's fragments are read under the second half: its A
                    // fragments of rows half 0 into af8[0] (free after the first half), its B fragment j into bf8[j]
                    // right after the MFMAs of column j (the second half runs column by column for that).
                    int8v af8[2][FMH], bf8[FN];
                    auto frag8 = [&](const char* piece, int row) __attribute__((always_inline)) -> int8v {
                        // the lane's 32 values are chunks kc and 4 + kc of the row's eight (the sum over k is order-free
                        // and both operands are read alike): each read is then the bank-conflict-free pattern of the
                        // 16-bit fragments (chunks 2 kc, 2 kc + 1: every second LDS cycle a conflict, by the counter)
                        const int4v lo = *(const int4v*)(piece + kmajor_offset<64, true>(row, f16_kc));
                        const int4v hi = *(const int4v*)(piece + kmajor_offset<64, true>(row, 4 + f16_kc));
                        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    };
                    auto a8 = [&](int t, int rh, int i) __attribute__((always_inline)) -> int8v {
                        return frag8(lds + a_lds(t), wm * WTM + (rh * FMH + i) * 16 + f16_row);
                    };
                    auto b8 = [&](int sidx, int j) __attribute__((always_inline)) -> int8v {
                        return frag8(lds + b_at(sidx), wn * WTN + j * 16 + f16_row);
                    };
                    // first half: rows half 0, MFMA (i, j) in row order; mid(k) after MFMA k; STEADY: B load r after MFMA 4 r + 2
                    auto half0 = [&](auto steady_tag, auto&& mid) __attribute__((always_inline)) {
                        constexpr bool STEADY = decltype(steady_tag)::value;
#pragma unroll
                        for (int i = 0; i < FMH; ++i)
#pragma unroll
                            for (int j = 0; j < FN; ++j) {
                                acc[i][j] = MfmaOp16x128<T>::run(bf8[j], af8[0][i], acc[i][j]);
                                mid(i * FN + j);
                                if (STEADY) {
#pragma unroll
                                    for (int r = 0; r < CBP; ++r)
                                        if ((2 * r + 1) * QM / (2 * CBP) == i * FN + j) { issue_b(r, TailNo{}); __builtin_amdgcn_sched_barrier(0); }
                                }
                            }
                    };
                    // second half: rows half 1, column by column; mid(k) after MFMA k; STEADY: A load r after MFMA r QM / CA
                    auto half1 = [&](auto steady_tag, auto&& mid) __attribute__((always_inline)) {
                        constexpr bool STEADY = decltype(steady_tag)::value;
#pragma unroll
                        for (int j = 0; j < FN; ++j)
#pragma unroll
                            for (int i = 0; i < FMH; ++i) {
                                acc[FMH + i][j] = MfmaOp16x128<T>::run(bf8[j], af8[1][i], acc[FMH + i][j]);
                                mid(j * FMH + i);
                                if (STEADY) {
#pragma unroll
                                    for (int r = 0; r < CA; ++r)
                                        if (r * (QM / CA) == j * FMH + i) { issue_a(r, TailNo{}); __builtin_amdgcn_sched_barrier(0); }
                                }
                            }
                    };
                    // reads of the next pair (even tile tn, B stage sn) under the second half: B column j after its
                    // last MFMA (k = j FMH + FMH - 1), A fragment i of rows half 0 after MFMA j FMH + i of column 0 .. 
                    auto next_reads = [&](int k, int tn, int sn) __attribute__((always_inline)) {
                        if (k < FMH) { af8[0][k] = a8(tn, 0, k); __builtin_amdgcn_sched_barrier(0); }
                        if ((k % FMH) == FMH - 1) { bf8[k / FMH] = b8(sn, k / FMH); __builtin_amdgcn_sched_barrier(0); }
                    };
                    auto pair_steady8 = [&](int t) __attribute__((always_inline)) {
                        begin_b((t + 4) * BK, b_at(stage_add(bstage, 4)));
                        begin_a((t + 4) * BK, a_lds(t + 4));
                        prio_up();
                        half0(BoolTag<true>{}, [&](int k) {
                            if (k < FMH) { af8[1][k] = a8(t, 1, k); __builtin_amdgcn_sched_barrier(0); }
                        });
                        prio_down();
                        wait_vmcnt<CBP>();
                        __syncthreads();          // also: everyone is done reading what the next loads overwrite
                        const int sn = stage_add(bstage, 2);
                        prio_up();
                        half1(BoolTag<true>{}, [&](int k) { next_reads(k, t + 2, sn); });
                        prio_down();
                        bstage = sn;
                    };
                    // drain: the pair of tiles t, t+1 (t+1 may lie beyond K: zeros), loads in bursts and only where tiles exist
                    auto drain_pair8 = [&](int t, bool have_next) __attribute__((always_inline)) {
                        int burst = 0;
                        if (t + 4 < KT) {
                            begin_b((t + 4) * BK, b_at(stage_add(bstage, 4)));
#pragma unroll
                            for (int r = 0; r < CBP; ++r) issue_b(r, TailYes{});
                            burst = CBP;
                        }
                        prio_up();
                        half0(BoolTag<false>{}, [&](int k) {
                            if (k < FMH) { af8[1][k] = a8(t, 1, k); __builtin_amdgcn_sched_barrier(0); }
                        });
                        prio_down();
                        if (have_next) {
                            if (burst) wait_vmcnt<CBP>(); else wait_vmcnt<0>();
                            __syncthreads();
                            if (t + 4 < KT) {
                                begin_a((t + 4) * BK, a_lds(t + 4));
#pragma unroll
                                for (int r = 0; r < CA; ++r) issue_a(r, TailYes{});
                            }
                        }
                        const int sn = stage_add(bstage, 2);
                        prio_up();
                        half1(BoolTag<false>{}, [&](int k) { if (have_next) next_reads(k, t + 2, sn); });
                        prio_down();
                        bstage = sn;
                    };
                    if (KT > 0) {
                        begin_a(0, a_lds(0));
#pragma unroll
                        for (int r = 0; r < CA; ++r) issue_a(r, TailYes{});
                        begin_b(0, b_at(0));
#pragma unroll
                        for (int r = 0; r < CBP; ++r) issue_b(r, TailYes{});
                        if (2 < KT) {
                            begin_a(2 * BK, a_lds(2));
#pragma unroll
                            for (int r = 0; r < CA; ++r) issue_a(r, TailYes{});
                            begin_b(2 * BK, b_at(2));
#pragma unroll
                            for (int r = 0; r < CBP; ++r) issue_b(r, TailYes{});
                            wait_vmcnt<CA + CBP>();
                        } else {
                            wait_vmcnt<0>();
                        }
                        __syncthreads();
#pragma unroll
                        for (int i = 0; i < FMH; ++i) af8[0][i] = a8(0, 0, i);
#pragma unroll
                        for (int j = 0; j < FN; ++j) bf8[j] = b8(0, j);
                        int t = 0;
                        for (; t + 6 <= KF; t += 2) pair_steady8(t);
                        for (; t < KT; t += 2) drain_pair8(t, t + 2 < KT);
                    }
                } else {
                // quarter Q of the pair whose even tile is t: tile Q/2, rows half Q%2, B fragments in bf[Q/2].
                // STEADY: B load r of the pair goes after MFMA (2r+1) 3QM/(4CB) of the pair, A load r after
                // MFMA 3QM + r QM/CA.
                auto quarter = [&](auto q_tag, auto steady_tag, int t, auto&& mid) {
                    constexpr int Q = decltype(q_tag)::value;
                    constexpr bool STEADY = decltype(steady_tag)::value;
                    constexpr int st = Q & 1, P = Q >> 1;
#pragma unroll
                    for (int i = 0; i < FMH; ++i)
#pragma unroll
                        for (int j = 0; j < FN; ++j) {
                            acc[st * FMH + i][j] = MfmaOp16<T>::run(bf[P][j], af[st][i], acc[st * FMH + i][j]);
                            mid(i * FN + j);
                            if (STEADY) {
                                const int idx = Q * QM + i * FN + j;
#pragma unroll
                                for (int r = 0; r < 2 * CB; ++r) {
                                    if ((2 * r + 1) * (3 * QM) / (4 * CB) == idx) {
                                        if (!BDBL && r == CB) begin_b((t + 5) * BK, b_at(stage_add(bstage, 5)));
                                        issue_b(BDBL ? r : r % CB, TailNo{});
                                        __builtin_amdgcn_sched_barrier(0);
                                    }
                                }
#pragma unroll
                                for (int r = 0; r < CA; ++r) {
                                    if (3 * QM + r * (QM / CA) == idx) {
                                        issue_a(r, TailNo{});
                                        __builtin_amdgcn_sched_barrier(0);
                                    }
                                }
                            }
                        }
                };
                // steady pair: tiles t, t+1; tiles t+4, t+5 are full
                auto pair_steady = [&](int t) {
                    begin_b((t + 4) * BK, b_at(stage_add(bstage, 4)));
                    begin_a((t + 4) * BK, a_lds(t + 4));
                    const char* sa = lds + a_lds(t);
                    const int s1 = stage_add(bstage, 1), s2 = stage_add(bstage, 2);
                    prio_up();
                    quarter(IntTag<0>{}, BoolTag<true>{}, t, [&](int k) {
                        if (k < FMH) { af[1][k] = a_frag(sa, 0, 1, k); __builtin_amdgcn_sched_barrier(0); }
                    });
                    prio_down();
                    prio_up();
                    quarter(IntTag<1>{}, BoolTag<true>{}, t, [&](int k) {
                        if (k < FMH) { af[0][k] = a_frag(sa, 1, 0, k); __builtin_amdgcn_sched_barrier(0); }
                        else if (k < FMH + FN) { bf[1][k - FMH] = read_bs(s1, k - FMH); __builtin_amdgcn_sched_barrier(0); }
                    });
                    prio_down();
                    prio_up();
                    quarter(IntTag<2>{}, BoolTag<true>{}, t, [&](int k) {
                        if (k < FMH) { af[1][k] = a_frag(sa, 1, 1, k); __builtin_amdgcn_sched_barrier(0); }
                    });
                    prio_down();
                    wait_vmcnt<2 * CB>();
                    __syncthreads();          // also: everyone is done reading what the next loads overwrite
                    const char* na = lds + a_lds(t + 2);
                    prio_up();
                    quarter(IntTag<3>{}, BoolTag<true>{}, t, [&](int k) {
                        if (k < FMH) { af[0][k] = a_frag(na, 0, 0, k); __builtin_amdgcn_sched_barrier(0); }
                        else if (k < FMH + FN) { bf[0][k - FMH] = read_bs(s2, k - FMH); __builtin_amdgcn_sched_barrier(0); }
                    });
                    prio_down();
                    bstage = stage_add(bstage, 2);
                };
                // drain: one tile t of parity PAR, loads issued in bursts and only where tiles exist
                auto drain_tile = [&](auto par_tag, int t, bool have_next) {
                    constexpr int PAR = decltype(par_tag)::value;
                    if (PAR == 0) {
                        pair_burst = 0;
                        if (BDBL) {
                            if (t + 4 < KT) {                 // one 64-deep piece: k-tiles t+4 and t+5 (zeros beyond K)
                                begin_b((t + 4) * BK, b_at(stage_add(bstage, 4)));
#pragma unroll
                                for (int r = 0; r < CBP; ++r) issue_b(r, TailYes{});
                                pair_burst += CBP;
                            }
                        } else {
                            for (int d = 4; d <= 5; ++d) {
                                if (t + d < KT) {
                                    begin_b((t + d) * BK, b_at(stage_add(bstage, d)));
#pragma unroll
                                    for (int r = 0; r < CB; ++r) issue_b(r, TailYes{});
                                    pair_burst += CB;
                                }
                            }
                        }
                    }
                    const char* sa = lds + a_lds(t);
                    prio_up();
                    quarter(IntTag<2 * PAR>{}, BoolTag<false>{}, t, [&](int k) {
                        if (k < FMH) { af[1][k] = a_frag(sa, PAR, 1, k); __builtin_amdgcn_sched_barrier(0); }
                    });
                    prio_down();
                    if (PAR == 1 && have_next) {
                        if (pair_burst >= 2 * CB) wait_vmcnt<2 * CB>(); else if (pair_burst >= CB) wait_vmcnt<CB>();
                        else wait_vmcnt<0>();
                        __syncthreads();
                        if (t + 3 < KT) {
                            begin_a((t + 3) * BK, a_lds(t + 3));
#pragma unroll
                            for (int r = 0; r < CA; ++r) issue_a(r, TailYes{});
                        }
                    }
                    const char* na = lds + a_lds(t + 1);
                    const int sn = stage_add(bstage, PAR + 1);
                    prio_up();
                    quarter(IntTag<2 * PAR + 1>{}, BoolTag<false>{}, t, [&](int k) {
                        if (!have_next) return;
                        if (k < FMH) { af[0][k] = a_frag(na, PAR ^ 1, 0, k); __builtin_amdgcn_sched_barrier(0); }
                        else if (k < FMH + FN) { bf[PAR ^ 1][k - FMH] = read_bs(sn, k - FMH); __builtin_amdgcn_sched_barrier(0); }
                    });
                    prio_down();
                    if (PAR == 1) bstage = stage_add(bstage, 2);
                };
                if (KT > 0) {
                    // what pair 0 reads first, then what pair 1 reads; the first barrier waits for the former only
                    begin_a(0, a_lds(0));
#pragma unroll
                    for (int r = 0; r < CA; ++r) issue_a(r, TailYes{});
                    if (BDBL) {
                        begin_b(0, b_at(0));
#pragma unroll
                        for (int r = 0; r < CBP; ++r) issue_b(r, TailYes{});
                    } else {
                        for (int t = 0; t < 2 && t < KT; ++t) {
                            begin_b(t * BK, b_at(t));
#pragma unroll
                            for (int r = 0; r < CB; ++r) issue_b(r, TailYes{});
                        }
                    }
                    int later = 0;
                    if (2 < KT) {
                        begin_a(2 * BK, a_lds(2));
#pragma unroll
                        for (int r = 0; r < CA; ++r) issue_a(r, TailYes{});
                        later += CA;
                    }
                    if (BDBL) {
                        if (2 < KT) {
                            begin_b(2 * BK, b_at(2));
#pragma unroll
                            for (int r = 0; r < CBP; ++r) issue_b(r, TailYes{});
                            later += CBP;
                        }
                    } else {
                        for (int t = 2; t < 4 && t < KT; ++t) {
                            begin_b(t * BK, b_at(t));
#pragma unroll
                            for (int r = 0; r < CB; ++r) issue_b(r, TailYes{});
                            later += CB;
                        }
                    }
                    if (later >= CA + 2 * CB) wait_vmcnt<CA + 2 * CB>(); else if (later >= CA + CB) wait_vmcnt<CA + CB>();
                    else wait_vmcnt<0>();
                    __syncthreads();
                    read_a2(lds + a_lds(0), 0, 0, af[0]);
#pragma unroll
                    for (int j = 0; j < FN; ++j) bf[0][j] = read_bs(0, j);
                    int t = 0;
                    for (; t + 6 <= KF; t += 2) pair_steady(t);
                    for (; t < KT; t += 2) {
                        drain_tile(IntTag<0>{}, t, t + 1 < KT);
                        if (t + 1 < KT) drain_tile(IntTag<1>{}, t + 1, t + 2 < KT);
                    }
                }
                }   // !F8PAIR
            } else {
                constexpr int NT = 2 * FMH * FN;           // MFMAs per k-tile
                constexpr int NB = FMH * FN;               // of which before the barrier
                // L loads are spread over the tile: load r right after MFMA number r NT / L; pieces before the barrier:
                auto early_of = [](int L) { return L == 0 ? 0 : ((NB * L + NT - 1) / NT < L ? (NB * L + NT - 1) / NT : L); };
                auto mfma2 = [&](int st, int bcur, auto l_tag, auto&& mid) {
                    constexpr int L = decltype(l_tag)::value;     // CA + CB: A pieces then B pieces; CB: B pieces; 0: none
    #pragma unroll
                    for (int i = 0; i < FMH; ++i)
    #pragma unroll
                        for (int j = 0; j < FN; ++j) {
                            acc[st * FMH + i][j] = MfmaOp16<T>::run(bf[bcur][j], af[st][i], acc[st * FMH + i][j]);
                            mid(i * FN + j);
                            const int idx = (st * FMH + i) * FN + j;
    #pragma unroll
                            for (int r = 0; r < L; ++r) {
                                if ((r * NT) / (L > 0 ? L : 1) == idx) {      // (L = 0: the loop is empty)
                                    if (L > CB && r < CA) issue_a(r, TailNo{}); else issue_b(L > CB ? r - CA : r, TailNo{});
                                    __builtin_amdgcn_sched_barrier(0);
                                }
                            }
                        }
                };
                auto wait_rt = [&](int n) {
                    if (n >= CA + CB) wait_vmcnt<CA + CB>(); else if (n >= CA) wait_vmcnt<CA>();
                    else if (n >= CB) wait_vmcnt<CB>(); else wait_vmcnt<0>();
                };
                // one k-tile t (half h = t % 2).  PHASE as above; L > 0: steady state with L loads spread; else
                // `burst` loads were issued at the start of the tile.  The fragment reads (second rows half of
                // this tile, then the first fragments of the next one after the barrier) go one at a time
                // between the MFMAs, like in the plain pipeline below.
                auto tile2 = [&](int t, int h, bool have_next, auto phase_tag, auto l_tag, int burst) {
                    constexpr int PHASE = decltype(phase_tag)::value;
                    constexpr int L = decltype(l_tag)::value;
                    constexpr int P = PHASE == 2 ? 1 : 0;
                    const char* sa = lds + a_lds(t);
                    if (PRIO) __builtin_amdgcn_s_setprio(2);
                    mfma2(0, P, l_tag, [&](int k) {
                        if (k < FMH) {
                            const int row = wm * WTM + (FMH + k) * 16 + f16_row;
                            af[1][k] = *(const short8v*)(sa + kmajor_offset<64, true>(row, h * 4 + f16_kc));
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    });
                    if (PRIO) __builtin_amdgcn_s_setprio(0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (have_next) {
                        // What tile t+1 reads must have landed; a wave's loads complete in issue order, so it
                        // waits until only the loads issued after those are outstanding.  Steady state, even t:
                        // A(t, t+1) and B(t+1) were issued during tile t-2; younger are B(t+2) from tile t-1
                        // (CB loads) and the early_of(CA + CB) pieces of this tile issued so far.  Odd t:
                        // A(t+1, t+2) are the first CA loads of tile t-1 and B(t+1) is older; younger are the
                        // CB loads of B(t+2) that followed them and the early_of(CB) pieces of this tile.
                        // Drain: everything but this tile's own burst.
                        if (L > 0) wait_vmcnt<CB + early_of(L)>(); else wait_rt(burst);
                        __syncthreads();      // also: everyone is done reading what the next loads overwrite
                    }
                    const char* na = lds + a_lds(t + 1);
                    const char* nb = lds + b_lds(t + 1);
                    if (PRIO) __builtin_amdgcn_s_setprio(2);
                    mfma2(1, P, l_tag, [&](int k) {
                        if (!have_next) return;
                        if (k < FMH) {
                            const int row = wm * WTM + k * 16 + f16_row;
                            af[0][k] = *(const short8v*)(na + kmajor_offset<64, true>(row, (h ^ 1) * 4 + f16_kc));
                            __builtin_amdgcn_sched_barrier(0);
                        } else if (k < FMH + FN) {
                            bf[P ^ 1][k - FMH] = read_b1(nb, 0, k - FMH);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    });
                    if (PRIO) __builtin_amdgcn_s_setprio(0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (PHASE == 0 && have_next) {
    #pragma unroll
                        for (int j = 0; j < FN; ++j) bf[0][j] = bf[1][j];
                    }
                };
                if (KT > 0) {
                    begin_a(0, a_lds(0));
    #pragma unroll
                    for (int r = 0; r < CA; ++r) issue_a(r, TailYes{});
                    for (int t = 0; t < 3 && t < KT; ++t) {
                        begin_b(t * BK, b_lds(t));
    #pragma unroll
                        for (int r = 0; r < CB; ++r) issue_b(r, TailYes{});
                    }
                    wait_vmcnt<0>();
                    __syncthreads();
                    read_a2(lds + a_lds(0), 0, 0, af[0]);
                    read_b(lds + b_lds(0), 0, bf[0]);
                    int t = 0;
                    for (; t + 4 < KF; t += 2) {
                        begin_a((t + 2) * BK, a_lds(t + 2));
                        begin_b((t + 3) * BK, b_lds(t + 3));
                        tile2(t, 0, true, IntTag<1>{}, IntTag<CA + CB>{}, 0);
                        begin_b((t + 4) * BK, b_lds(t + 4));
                        tile2(t + 1, 1, true, IntTag<2>{}, IntTag<CB>{}, 0);
                    }
                    for (; t < KT; ++t) {
                        int burst = 0;
                        if (!(t & 1) && t + 2 < KT) {
                            begin_a((t + 2) * BK, a_lds(t + 2));
    #pragma unroll
                            for (int r = 0; r < CA; ++r) issue_a(r, TailYes{});
                            burst += CA;
                        }
                        if (t + 3 < KT) {
                            begin_b((t + 3) * BK, b_lds(t + 3));
    #pragma unroll
                            for (int r = 0; r < CB; ++r) issue_b(r, TailYes{});
                            burst += CB;
                        }
                        tile2(t, t & 1, t + 1 < KT, IntTag<0>{}, IntTag<0>{}, burst);
                    }
                }
            }
        } else {
            // B fragments of k32 step kq of a tile that starts from buffer P live in bf[(P + kq) % 2]; the
            // next tile's first ones are read into bf[(P + KQ) % 2] while this tile's last step still
            // multiplies.  With an odd number of k32 steps per tile the buffers swap roles from tile to
            // tile: the steady state runs tiles in pairs (PHASE 1 starts from buffer 0, PHASE 2 from
            // buffer 1); a tile on its own (PHASE 0) starts from buffer 0 and moves the next tile's
            // fragments back there (register copies) once its last MFMAs have been issued.
            auto tile_body = [&](int stage, int next_stage, bool have_next, auto newer_tag, int newer_rt, auto spread_tag,
                                 auto phase_tag) {
                constexpr int NEWER = decltype(newer_tag)::value;
                constexpr bool SPREAD = decltype(spread_tag)::value;
                constexpr int PHASE = decltype(phase_tag)::value;
                constexpr int P = (PHASE == 2 && (KQ & 1)) ? 1 : 0;
                const char* sa = lds + stage * STAGE;
                const char* sb = sa + A_BYTES;
    #pragma unroll
                for (int s = 0; s < NSTEP - 1; ++s) {
                    if (PRIO) __builtin_amdgcn_s_setprio(2);
                    mfma_step(s, (P + (s >> 1)) & 1, spread_tag, [&](int k) {
                        if (k < FMH) {
                            af[(s + 1) & 1][k] = read_a1(sa, s + 1, k);
                            __builtin_amdgcn_sched_barrier(0);
                        } else if (((s + 1) & 1) == 0 && k < FMH + FN) {
                            bf[(P + ((s + 1) >> 1)) & 1][k - FMH] = read_b1(sb, (s + 1) >> 1, k - FMH);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    });
                    if (PRIO) __builtin_amdgcn_s_setprio(0);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (have_next) {
                    if (NEWER >= 0) wait_vmcnt<(SPREAD && NSTAGE >= 3 ? (NEWER >= 1 ? NEWER - 1 : 0) * LOADS + EARLY : (NEWER >= 0 ? NEWER : 0) * LOADS)>();
                    else wait_newer(newer_rt);
                    __syncthreads();          // everyone's pieces landed; everyone is done reading `stage`
                }
                const char* na = lds + next_stage * STAGE;
                if (PRIO) __builtin_amdgcn_s_setprio(2);
                mfma_step(NSTEP - 1, (P + KQ - 1) & 1, spread_tag, [&](int k) {
                    if (!have_next) return;
                    if (k < FMH) {
                        af[0][k] = read_a1(na, 0, k);
                        __builtin_amdgcn_sched_barrier(0);
                    } else if (k < FMH + FN) {
                        bf[(P + KQ) & 1][k - FMH] = read_b1(na + A_BYTES, 0, k - FMH);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                });
                if (PRIO) __builtin_amdgcn_s_setprio(0);
                __builtin_amdgcn_sched_barrier(0);
                if (PHASE == 0 && (KQ & 1) && have_next) {
    #pragma unroll
                    for (int j = 0; j < FN; ++j) bf[0][j] = bf[1][j];
                }
            };
            main_loop([&]() { read_a(lds, 0, af[0]); read_b(lds + A_BYTES, 0, bf[0]); }, tile_body, BoolTag<(KQ & 1) != 0>{});
        }
    }

    // ---- epilogue in registers, then one coalesced store ---------------------
    // Lane holds, for 32x32 block (i,j): row m = lane%32, columns 8*g + 4*(lane/32) + 0..3
    // (16x16 blocks: row lane%16, columns 4*(lane/16) + 0..3).
    // alpha/bias/activation and the rounding to the output type happen on the
    // accumulator registers.  The rounded pieces then take one trip through this
    // wave's own slice of LDS (free after the k loop) purely to change which lane
    // holds what, so that the global stores are 16 bytes per lane along rows:
    // every store instruction writes whole 128-byte (or longer) row segments.
    __syncthreads();                           // all waves are done reading the last stage
    const int act = (p.epi == EPI_RELU || p.epi == EPI_BIAS_RELU) ? 1
                  : (p.epi == EPI_GELU_TANH || p.epi == EPI_BIAS_GELU_TANH) ? 2 : 0;
    const bool out_f32 = p.out_dtype == DT_F32;
    char* wlds = lds + wave * ((NSTAGE * STAGE) / NW);
    EpiCtx<TO, AccV, FM, FN, WTM, WTN, (NSTAGE * STAGE) / NW> ctx{p, acc, wlds, m0 + wm * WTM, n0 + wn * WTN, lane,
                                                         (int64_t)b * p.stride_c};
    if constexpr (sizeof(T) == 1 && MfmaOp<T>::kChunks == 1) {      // int8 operands
        const bool has_mid = p.q_mid > 0.0f, has_bn = p.q_mean != nullptr;
        const bool fast = (!has_mid || make_step_div(p.q_mid).fast) && (p.out_dtype != DT_INT8 || make_step_div(p.q_out).fast);
        if (!fast) ctx.template run_quant<WM, WN, 0>(lds, wm, wn);
        else if (!has_mid && !has_bn) ctx.template run_quant<WM, WN, 1>(lds, wm, wn);
        else if (has_mid && !has_bn) ctx.template run_quant<WM, WN, 2>(lds, wm, wn);
        else if (!has_mid) ctx.template run_quant<WM, WN, 3>(lds, wm, wn);
        else ctx.template run_quant<WM, WN, 4>(lds, wm, wn);
    } else if (out_f32) {
        if (act == 0) ctx.template run<0, true>(); else if (act == 1) ctx.template run<1, true>();
        else ctx.template run<2, true>();
    } else {
        if (act == 0) ctx.template run<0, false>(); else if (act == 1) ctx.template run<1, false>();
        else ctx.template run<2, false>();
    }
}

}  // namespace pbk
