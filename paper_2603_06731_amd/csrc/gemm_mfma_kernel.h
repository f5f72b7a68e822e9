// MFMA contraction kernel for gfx950: 16-bit inputs, fp32 accumulation.
//
// Structure (paper Sec. 4.3 multi-level tiling and fast buffers, Sec. 4.5
// on-the-fly packing, Sec. 4.6 mapping to matrix units, App. A.2 overlap of
// copy and compute), re-designed for CDNA4:
//   workgroup tile BM x BN x BK  ->  WM x WN waves, each a (BM/WM) x (BN/WN)
//   register tile of 32x32 MFMA blocks (v_mfma_f32_32x32x16), accumulators
//   live in registers for the whole K loop.
//   Global -> LDS staging in 16-byte pieces, double-buffered: the loads of
//   k-tile t+1 are in flight while k-tile t is multiplied.
//   A tile in LDS: [BM][BK] with the 16-byte chunk index XOR-swizzled by the
//   row so that the ds_read_b128 fragment reads hit distinct banks.
//   B tile in LDS: [BK][BN] as in memory (n contiguous); the k-contiguous
//   MFMA operand is produced by the transposing LDS read ds_read_b64_tr_b16,
//   with the 64-byte chunk index XOR-swizzled by k.  With trans_b the B tile
//   is [BN][BK] and is handled exactly like A.
//   The MFMA is issued with the operands swapped (B fragment as srcA, A
//   fragment as srcB) so each lane ends up with 4 consecutive n of one row m:
//   the epilogue then works on 4-wide pieces and stores 8 or 16 bytes.
//   Partial tiles: out-of-range 16-byte pieces are zero-filled in LDS (rows
//   beyond M, columns beyond N, k beyond K, convolution taps in the padding);
//   rows/columns beyond M/N are never stored.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
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

template <typename T> struct MfmaOp;
template <> struct MfmaOp<bf16_t> {
    static __device__ __forceinline__ f32x16 run(short8v a, short8v b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct MfmaOp<f16_t> {
    static __device__ __forceinline__ f32x16 run(short8v a, short8v b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
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

// 16-byte-chunk swizzle for a [rows][BK] 16-bit tile (row = BK*2 bytes).
template <int BK>
__device__ __forceinline__ int kmajor_offset(int row, int chunk) {
    constexpr int CPR = BK / 8;            // chunks per row
    constexpr int RP = 256 / (BK * 2);     // rows per 256 bytes (all 64 banks)
    int s = (row / RP) % CPR;
    return row * (BK * 2) + ((chunk ^ s) << 4);
}

// Byte offset inside a [BK][BN] 16-bit tile (row = BN*2 bytes) of byte `nbyte`
// of row k, 64-byte chunks XOR-swizzled by k.
template <int BN>
__device__ __forceinline__ int nmajor_offset(int k, int nbyte) {
    return k * (BN * 2) + ((((nbyte >> 6) ^ (k & 3)) << 6) | (nbyte & 63));
}

template <typename T, int BM, int BN, int BK, int WM, int WN, bool CONV, bool TRANS_B>
__global__ __launch_bounds__(WM * WN * 64) void gemm_mfma_kernel(Problem p, TileMap tmap) {
    constexpr int NT = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int FM = WTM / 32, FN = WTN / 32;
    constexpr int KSUB = BK / 16;
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int A_CHUNKS = BM * BK / 8, B_CHUNKS = BN * BK / 8;
    constexpr int CA = A_CHUNKS / NT, CB = B_CHUNKS / NT;
    static_assert(A_CHUNKS % NT == 0 && B_CHUNKS % NT == 0, "tile must split evenly over lanes");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32x32");
    static_assert(BK % 16 == 0 && (BK == 32 || BK == 64), "BK");
    static_assert(TRANS_B || BN == 128 || BN == 256, "n-major B tile needs BN of 128 or 256");

    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN;

    int b, tile_m, tile_n;
    map_tile(tmap, blockIdx.x, b, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const char* Abase = (const char*)p.A + (int64_t)b * p.stride_a * 2;
    const char* Bbase = (const char*)p.B + (int64_t)b * p.stride_b * 2;

    // ---- per-lane staging assignments (fixed for the whole K loop) ---------
    // A: chunk q -> (row, 16-byte chunk in the row)
    const char* a_ptr[CA];      // dense: address of the piece at k0 = 0
    bool a_row_ok[CA];
    int a_lds[CA], a_kofs[CA];
    int a_n[CA], a_ih0[CA], a_iw0[CA];   // conv: image index and top-left tap coordinate
    constexpr int A_CPR = BK / 8;
#pragma unroll
    for (int r = 0; r < CA; ++r) {
        int q = t + NT * r;
        int row = q / A_CPR, ch = q % A_CPR;
        a_lds[r] = kmajor_offset<BK>(row, ch);
        a_kofs[r] = ch * 8;
        int gm = m0 + row;
        a_row_ok[r] = gm < p.M;
        if (CONV) {
            int pix = p.conv.OH * p.conv.OW;
            int gmc = a_row_ok[r] ? gm : 0;
            int n = gmc / pix;
            int rem = gmc - n * pix;
            int oh = rem / p.conv.OW;
            int ow = rem - oh * p.conv.OW;
            a_n[r] = n;
            a_ih0[r] = oh * p.conv.stride_h - p.conv.pad_h;
            a_iw0[r] = ow * p.conv.stride_w - p.conv.pad_w;
            a_ptr[r] = Abase;
        } else {
            a_ptr[r] = Abase + ((int64_t)(a_row_ok[r] ? gm : 0) * p.lda + a_kofs[r]) * 2;
        }
    }
    // B
    const char* b_ptr[CB];
    bool b_ok[CB];
    int b_lds[CB], b_kofs[CB];
    constexpr int B_CPR = TRANS_B ? BK / 8 : BN / 8;
#pragma unroll
    for (int r = 0; r < CB; ++r) {
        int q = t + NT * r;
        int row = q / B_CPR, ch = q % B_CPR;
        if (TRANS_B) {          // tile [BN][BK]: row = n, chunk along k
            b_lds[r] = kmajor_offset<BK>(row, ch);
            b_kofs[r] = ch * 8;
            int gn = n0 + row;
            b_ok[r] = gn < p.N;
            b_ptr[r] = Bbase + ((int64_t)(b_ok[r] ? gn : 0) * p.ldb + b_kofs[r]) * 2;
        } else {                // tile [BK][BN]: row = k, chunk along n
            b_lds[r] = nmajor_offset<BN>(row, ch * 16);
            b_kofs[r] = row;
            int gn = n0 + ch * 8;
            b_ok[r] = gn < p.N;             // N % 8 == 0 on this path: whole chunk in or out
            b_ptr[r] = Bbase + ((int64_t)row * p.ldb + (b_ok[r] ? gn : 0)) * 2;
        }
    }

    int4v a_reg[CA], b_reg[CB];
    const int4v zero4 = {0, 0, 0, 0};

    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int r = 0; r < CA; ++r) {
            int k = k0 + a_kofs[r];
            bool ok = a_row_ok[r] && k < p.K;
            const char* src;
            if (CONV) {
                int tap = k / p.conv.Cin;
                int c = k - tap * p.conv.Cin;
                int kh = tap / p.conv.KW;
                int kw = tap - kh * p.conv.KW;
                int ih = a_ih0[r] + kh * p.conv.dil_h;
                int iw = a_iw0[r] + kw * p.conv.dil_w;
                ok = ok && ih >= 0 && ih < p.conv.H && iw >= 0 && iw < p.conv.W;
                src = Abase + ((((int64_t)a_n[r] * p.conv.H + ih) * p.conv.W + iw) * p.conv.Cin + c) * 2;
            } else {
                src = a_ptr[r] + (int64_t)k0 * 2;
            }
            a_reg[r] = ok ? *(const int4v*)src : zero4;
        }
#pragma unroll
        for (int r = 0; r < CB; ++r) {
            if (TRANS_B) {
                bool ok = b_ok[r] && (k0 + b_kofs[r]) < p.K;
                b_reg[r] = ok ? *(const int4v*)(b_ptr[r] + (int64_t)k0 * 2) : zero4;
            } else {
                bool ok = b_ok[r] && (k0 + b_kofs[r]) < p.K;
                b_reg[r] = ok ? *(const int4v*)(b_ptr[r] + (int64_t)k0 * p.ldb * 2) : zero4;
            }
        }
    };
    auto store_tiles = [&](int stage) {
        char* sa = lds + stage * STAGE;
        char* sb = sa + A_BYTES;
#pragma unroll
        for (int r = 0; r < CA; ++r) *(int4v*)(sa + a_lds[r]) = a_reg[r];
#pragma unroll
        for (int r = 0; r < CB; ++r) *(int4v*)(sb + b_lds[r]) = b_reg[r];
    };

    // ---- per-lane fragment read offsets -----------------------------------
    // A fragment (32 rows x 16 k): lane -> row lane%32, k-chunk lane/32 of the 2 in the k16 step
    const int frag_row = lane & 31, frag_kc = lane >> 5;
    // B via transposing read: 16-lane block -> 16 n; lane -> k row (lane%16)/4, n piece lane%4
    const int tr_k = ((lane & 15) >> 2) + ((lane >> 5) << 3);
    const int tr_nbyte = ((((lane >> 4) & 1) << 4) + ((lane & 3) << 2)) * 2;

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    auto compute = [&](int stage) {
        const char* sa = lds + stage * STAGE;
        const char* sb = sa + A_BYTES;
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) {
            short8v af[FM], bf[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                int row = wm * WTM + i * 32 + frag_row;
                af[i] = *(const short8v*)(sa + kmajor_offset<BK>(row, ks * 2 + frag_kc));
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                if (TRANS_B) {
                    int row = wn * WTN + j * 32 + frag_row;
                    bf[j] = *(const short8v*)(sb + kmajor_offset<BK>(row, ks * 2 + frag_kc));
                } else {
                    int nbyte = (wn * WTN + j * 32) * 2 + tr_nbyte;
                    int k = ks * 16 + tr_k;
                    short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        PBK_LDS_PTR(short4v, sb + nmajor_offset<BN>(k, nbyte)));
                    short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        PBK_LDS_PTR(short4v, sb + nmajor_offset<BN>(k + 4, nbyte)));
                    bf[j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
            }
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = MfmaOp<T>::run(bf[j], af[i], acc[i][j]);
        }
    };

    // ---- main loop: double-buffered LDS ------------------------------------
    const int KT = (p.K + BK - 1) / BK;
    if (KT > 0) {
        load_tiles(0);
        store_tiles(0);
    }
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const bool more = kt + 1 < KT;
        if (more) load_tiles((kt + 1) * BK);
        compute(kt & 1);
        if (more) store_tiles((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue in registers, then store ---------------------------------
    // lane holds, for block (i,j): row m = lane%32, columns 8*g + 4*(lane/32) + 0..3, g = 0..3
    const bool has_bias = epi_has_bias(p.epi);
    const int64_t c_batch = (int64_t)b * p.stride_c;
    const bool out_f32 = p.out_dtype == DT_F32;
    const int esz = out_f32 ? 4 : 2;
    const bool vec_ok = (p.ldc % 4 == 0) && (((uintptr_t)p.C + (uintptr_t)c_batch * esz) % 16 == 0) &&
                        (p.stride_c % 4 == 0);
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        int gm = m0 + wm * WTM + i * 32 + (lane & 31);
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                int gn = n0 + wn * WTN + j * 32 + g * 8 + ((lane >> 5) << 2);
                if (gm >= p.M || gn >= p.N) continue;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float bias = (has_bias && gn + e < p.N) ? p.bias[gn + e] : 0.0f;
                    v[e] = apply_epilogue(acc[i][j][g * 4 + e], p.alpha, bias, p.epi);
                }
                int64_t o = c_batch + (int64_t)gm * p.ldc + gn;
                if (vec_ok && gn + 3 < p.N) {
                    if (out_f32) {
                        f32x4 w = {v[0], v[1], v[2], v[3]};
                        *(f32x4*)((float*)p.C + o) = w;
                    } else {
                        int2v w;
                        w[0] = (int)to_bits16<T>(v[0]) | ((int)to_bits16<T>(v[1]) << 16);
                        w[1] = (int)to_bits16<T>(v[2]) | ((int)to_bits16<T>(v[3]) << 16);
                        *(int2v*)((uint16_t*)p.C + o) = w;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (gn + e >= p.N) break;
                        if (out_f32) ((float*)p.C)[o + e] = v[e];
                        else ((uint16_t*)p.C)[o + e] = to_bits16<T>(v[e]);
                    }
                }
            }
        }
    }
}

}  // namespace pbk
