// MFMA contraction kernel for gfx950: 16-bit inputs, fp32 accumulation.
//
// Structure (paper Sec. 4.3 multi-level tiling and fast buffers, Sec. 4.5
// on-the-fly packing, Sec. 4.6 mapping to matrix units, App. A.2 overlap of
// copy and compute), re-designed for CDNA4:
//   workgroup tile BM x BN x BK  ->  WM x WN waves, each a (BM/WM) x (BN/WN)
//   register tile of 32x32 MFMA blocks (v_mfma_f32_32x32x16), accumulators
//   live in registers for the whole K loop.
//   Global -> LDS staging without passing through registers: every wave issues
//   buffer_load_dwordx4 ... lds, each writing 64 x 16 bytes to 1 KiB of LDS.
//   Two LDS stages: the loads of k-tile t+1 are in flight while k-tile t is
//   multiplied; one barrier per k-tile.  Pieces that lie outside the matrix
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
//   the epilogue then works on 4-wide pieces and stores 8 or 16 bytes.
//   Rows/columns beyond M/N are never stored.
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

enum : int { MODE_DENSE = 0, MODE_TRANS_B = 1, MODE_CONV = 2 };

// buffer offsets at or above this are out of range for every descriptor we
// build (num_records = 2^31): the load returns zeros
constexpr unsigned kOob = 0x80000000u;

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
__device__ __forceinline__ int kmajor_swz(int row) {
    constexpr int CPR = BK / 8;            // chunks per row
    constexpr int RP = 256 / (BK * 2);     // rows per 256 bytes (all 64 banks)
    return (row / RP) % CPR;
}
template <int BK>
__device__ __forceinline__ int kmajor_offset(int row, int chunk) {
    return row * (BK * 2) + ((chunk ^ kmajor_swz<BK>(row)) << 4);
}

// Byte offset inside a [BK][BN] 16-bit tile (row = BN*2 bytes) of byte `nbyte`
// of row k, 64-byte chunks XOR-swizzled by k.
template <int BN>
__device__ __forceinline__ int nmajor_offset(int k, int nbyte) {
    return k * (BN * 2) + ((((nbyte >> 6) ^ (k & 3)) << 6) | (nbyte & 63));
}

// Raw buffer descriptor over [base, base + 2^31): stride 0, 32-bit data format.
__device__ __forceinline__ int4v make_rsrc(const void* base) {
    uint64_t a = (uint64_t)base;
    int4v r = {(int)(uint32_t)a, (int)(uint32_t)(a >> 32), (int)kOob, 0x00020000};
    return r;
}

// One wave-wide 1 KiB direct-to-LDS load: lane i -> LDS bytes [16 i, 16 i + 16)
// of the block at LDS byte address lds_addr (wave-uniform, carried in M0).
// Written as inline assembly so that the compiler does not serialise later LDS
// reads of the OTHER stage behind it; completion is awaited explicitly with
// s_waitcnt vmcnt(0) before the barrier that publishes the stage.  Nothing else
// in this kernel depends on M0.
__device__ __forceinline__ void dma16(int4v rsrc, unsigned lds_addr, unsigned voff) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_addr), "v"(voff), "s"(rsrc) : "memory");
}

__device__ __forceinline__ unsigned lds_addr_of(const char* p) {
    return (unsigned)(uintptr_t)PBK_LDS_PTR(const char, p);
}

template <typename T, int BM, int BN, int BK, int WM, int WN, int MODE>
__global__ __launch_bounds__(WM * WN * 64) void gemm_mfma_kernel(Problem p, TileMap tmap) {
    constexpr bool CONV = MODE == MODE_CONV;
    constexpr bool TRANS_B = MODE == MODE_TRANS_B;
    constexpr int NW = WM * WN;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int FM = WTM / 32, FN = WTN / 32;
    constexpr int KSUB = BK / 16;
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int A_BLKS = A_BYTES / 1024, B_BLKS = B_BYTES / 1024;     // 1 KiB per wave-load
    constexpr int CA = A_BLKS / NW, CB = B_BLKS / NW;
    static_assert(A_BLKS % NW == 0 && B_BLKS % NW == 0, "tile must split evenly over waves");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32x32");
    static_assert(BK == 32 || BK == 64, "BK");
    static_assert(TRANS_B || BN == 128 || BN == 256, "n-major B tile needs BN of 128 or 256");

    extern __shared__ __attribute__((aligned(1024))) char lds[];

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
    // n-major tile ([BK][BN]): 1 KiB block = NM_ROWS k-rows
    constexpr int NM_CPR = BN / 8;
    constexpr int NM_ROWS = 64 / NM_CPR;
    const int nm_row = lane / NM_CPR, nm_slot = lane % NM_CPR;

    const char* Abase = (const char*)p.A + (int64_t)b * p.stride_a * 2;
    const char* Bbase = (const char*)p.B + (int64_t)b * p.stride_b * 2;

    unsigned a_voff[CA];       // dense / trans: byte offset from the tile's row block at k0; conv: pixel base
    int a_kofs[CA];            // k offset (elements) of the piece inside the k-tile
    int a_ih0[CA], a_iw0[CA];  // conv: top-left tap coordinates
    bool a_ok[CA];
#pragma unroll
    for (int r = 0; r < CA; ++r) {
        int blk = wave * CA + r;
        int row = blk * KM_ROWS + km_row;
        int chunk = km_slot ^ kmajor_swz<BK>(row);
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
            a_ih0[r] = oh * p.conv.stride_h - p.conv.pad_h;
            a_iw0[r] = ow * p.conv.stride_w - p.conv.pad_w;
            // byte offset of pixel (n, ih0, iw0), channel 0; may be "negative" (wraps), fixed up per tap
            a_voff[r] = (unsigned)(((n * p.conv.H + a_ih0[r]) * p.conv.W + a_iw0[r]) * p.conv.Cin * 2);
        } else {
            a_voff[r] = a_ok[r] ? (unsigned)(row * (int)p.lda * 2 + chunk * 16) : kOob;
        }
    }
    unsigned b_voff[CB];
    int b_kofs[CB];
#pragma unroll
    for (int r = 0; r < CB; ++r) {
        int blk = wave * CB + r;
        if (TRANS_B) {
            int row = blk * KM_ROWS + km_row;
            int chunk = km_slot ^ kmajor_swz<BK>(row);
            b_kofs[r] = chunk * 8;
            b_voff[r] = (n0 + row < p.N) ? (unsigned)(row * (int)p.ldb * 2 + chunk * 16) : kOob;
        } else {
            int krow = blk * NM_ROWS + nm_row;
            int c64 = (nm_slot >> 2) ^ (krow & 3);
            int nbyte = (c64 << 6) | ((nm_slot & 3) << 4);
            b_kofs[r] = krow;
            b_voff[r] = (n0 + (nbyte >> 1) < p.N) ? (unsigned)(krow * (int)p.ldb * 2 + nbyte) : kOob;
        }
    }

    // Descriptor bases: A at (m0, 0), B at (0, n0) resp. (n0, 0); advanced by k0 per k-tile.
    const char* a_tile = CONV ? Abase : Abase + (int64_t)m0 * p.lda * 2;
    const char* b_tile = TRANS_B ? Bbase + (int64_t)n0 * p.ldb * 2 : Bbase + (int64_t)n0 * 2;

    const unsigned lds_base = (unsigned)__builtin_amdgcn_readfirstlane((int)lds_addr_of(lds));
    auto issue_loads = [&](int k0, int stage) {
        const unsigned sa = lds_base + stage * STAGE;
        const unsigned sb = sa + A_BYTES;
        const bool tail = k0 + BK > p.K;         // uniform: only the last k-tile can be partial
        if (CONV) {
            int4v ra = make_rsrc(a_tile);
            const bool one_tap = (p.conv.Cin % BK) == 0;   // whole k-tile inside one filter tap
            int tap_u = 0, c_u = 0, kh_u = 0, kw_u = 0;
            if (one_tap) {
                tap_u = k0 / p.conv.Cin; c_u = k0 - tap_u * p.conv.Cin;
                kh_u = tap_u / p.conv.KW; kw_u = tap_u - kh_u * p.conv.KW;
            }
#pragma unroll
            for (int r = 0; r < CA; ++r) {
                int k = k0 + a_kofs[r];
                int kh, kw, c;
                if (one_tap) { kh = kh_u; kw = kw_u; c = c_u + a_kofs[r]; }
                else {
                    int tap = k / p.conv.Cin;
                    c = k - tap * p.conv.Cin;
                    kh = tap / p.conv.KW;
                    kw = tap - kh * p.conv.KW;
                }
                int dh = kh * p.conv.dil_h, dw = kw * p.conv.dil_w;
                int ih = a_ih0[r] + dh, iw = a_iw0[r] + dw;
                bool ok = a_ok[r] && k < p.K && ih >= 0 && ih < p.conv.H && iw >= 0 && iw < p.conv.W;
                unsigned off = a_voff[r] + (unsigned)(((dh * p.conv.W + dw) * p.conv.Cin + c) * 2);
                dma16(ra, sa + (wave * CA + r) * 1024, ok ? off : kOob);
            }
        } else {
            int4v ra = make_rsrc(a_tile + (int64_t)k0 * 2);
#pragma unroll
            for (int r = 0; r < CA; ++r) {
                unsigned off = a_voff[r];
                if (tail && k0 + a_kofs[r] >= p.K) off = kOob;
                dma16(ra, sa + (wave * CA + r) * 1024, off);
            }
        }
        {
            int4v rb = make_rsrc(TRANS_B ? b_tile + (int64_t)k0 * 2
                                                          : b_tile + (int64_t)k0 * p.ldb * 2);
#pragma unroll
            for (int r = 0; r < CB; ++r) {
                unsigned off = b_voff[r];
                if (tail && k0 + b_kofs[r] >= p.K) off = kOob;
                dma16(rb, sb + (wave * CB + r) * 1024, off);
            }
        }
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

    auto read_a = [&](const char* sa, int ks, short8v (&af)[FM]) {
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            int row = wm * WTM + i * 32 + frag_row;
            af[i] = *(const short8v*)(sa + kmajor_offset<BK>(row, ks * 2 + frag_kc));
        }
    };
    auto read_b = [&](const char* sb, int ks, short8v (&bf)[FN]) {
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
    };

    auto compute = [&](int stage) {
        const char* sa = lds + stage * STAGE;
        const char* sb = sa + A_BYTES;
        short8v af[2][FM], bf[2][FN];
        read_a(sa, 0, af[0]);
        read_b(sb, 0, bf[0]);
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) {
            const int cur = ks & 1;
            if (ks + 1 < KSUB) {
                read_a(sa, ks + 1, af[cur ^ 1]);
                read_b(sb, ks + 1, bf[cur ^ 1]);
            }
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = MfmaOp<T>::run(bf[cur][j], af[cur][i], acc[i][j]);
        }
    };

    // ---- main loop: two LDS stages, loads of tile t+1 in flight during tile t
    const int KT = (p.K + BK - 1) / BK;
    if (KT > 0) issue_loads(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0f70);      // vmcnt(0): this wave's pieces have landed
    __syncthreads();
    for (int kt = 0; kt < KT - 1; ++kt) {
        issue_loads((kt + 1) * BK, (kt + 1) & 1);
        compute(kt & 1);
        __builtin_amdgcn_s_waitcnt(0x0f70);
        __syncthreads();
    }
    if (KT > 0) compute((KT - 1) & 1);

    // ---- epilogue in registers, then store ---------------------------------
    // lane holds, for block (i,j): row m = lane%32, columns 8*g + 4*(lane/32) + 0..3, g = 0..3
    const bool has_bias = epi_has_bias(p.epi);
    const int64_t c_batch = (int64_t)b * p.stride_c;
    const bool out_f32 = p.out_dtype == DT_F32;
    const int esz = out_f32 ? 4 : 2;
    const bool vec_ok = (p.ldc % 4 == 0) && (((uintptr_t)p.C + (uintptr_t)c_batch * esz) % 16 == 0);
    const int act = (p.epi == EPI_RELU || p.epi == EPI_BIAS_RELU) ? 1
                  : (p.epi == EPI_GELU_TANH || p.epi == EPI_BIAS_GELU_TANH) ? 2 : 0;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int gn = n0 + wn * WTN + j * 32 + g * 8 + ((lane >> 5) << 2);
            float bias[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (has_bias) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (gn + e < p.N) bias[e] = p.bias[gn + e];
            }
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                const int gm = m0 + wm * WTM + i * 32 + (lane & 31);
                if (gm >= p.M || gn >= p.N) continue;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float tt = fmaf(p.alpha, acc[i][j][g * 4 + e], bias[e]);
                    if (act == 1) tt = fmaxf(tt, 0.0f);
                    else if (act == 2) tt = gelu_tanh_f32(tt);
                    v[e] = tt;
                }
                const int64_t o = c_batch + (int64_t)gm * p.ldc + gn;
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
