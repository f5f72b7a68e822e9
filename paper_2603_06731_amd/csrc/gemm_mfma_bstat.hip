// Matrix-unit contraction for SHORT contractions with many output rows (K <= 256: the attention-score
// product Q K^T with the head dimension as K, 1x1 projections).  Such a problem is bound by the stores of
// its output, and a tile-per-workgroup kernel spends its time in a chain of latencies per tile (first
// loads, a few k-tiles, the stores) while every workgroup fetches (BM + BN) K operand values for BM BN
// outputs.
//
// Here the B operand of a workgroup's 256 columns is STATIONARY IN REGISTERS (paper Sec. 4.3: the operand
// that is reused across a loop is kept in the fastest buffer): each of the 4 waves keeps the MFMA
// fragments of its 64 columns over the whole contraction (K/2 registers per lane) and the workgroup walks
// down its share of the rows in steps of 64 (32 when K > 128).  Per step it fetches only the 64 x K piece of A
// (direct-to-LDS loads of whole 128-byte lines into a ring of three stages: the pieces of the next two steps
// are in flight), runs 16 (K/32) MFMAs per wave in two halves of 32 rows and stores 64 x 256 outputs: the
// pointwise tail is applied to the accumulators (Sec. 4.3 fusion), the rounded values pass once through the
// wave's own LDS slice to change lane ownership and leave as 16-byte stores along rows.  Operand traffic
// per output is a third of the 128x256 tile's, there is one barrier per step and no per-tile start-up.
// Nothing in the loop waits for a store: every step issues a FIXED number of loads and stores (buffer
// operations whose offset is out of range where nothing is to be moved), a wave's memory operations
// complete in issue order, and so "the piece of this step has landed" is an s_waitcnt on a constant count
// of younger operations.  Two workgroups share a compute unit (65 KiB of LDS, 170 registers; 253 at K = 256).
// A in LDS: per 64-deep piece [64 rows][64 k] with the main kernel's 16-byte-chunk swizzle; B passes once
// through LDS, 32 KiB at a time: k-major (trans_b) in the layout of A's pieces, row-major as [64 k][256 n]
// in the main kernel's n-major layout, read with the transposing LDS read.
#include "gemm_mfma_launch.h"

namespace pbk {
namespace {

constexpr int SBM = 64, SBN = 256;          // rows per step (32 when K > 128: the LDS ring holds three pieces of A), columns per workgroup
constexpr int SWAVES = 4;                   // waves, side by side along n
constexpr int SWTN = SBN / SWAVES;          // 64 columns per wave
constexpr int SFN = SWTN / 16;
constexpr int S_STAGES = 3;                 // LDS stages of A: the pieces of the next two steps are in flight
constexpr int S_SLICE = 4096;               // a wave's LDS slice for the epilogue's change of lane ownership

// How linear workgroup ids map to (batch entry, share of the rows, column tile): ids are regrouped so that
// an XCD owns a contiguous run (its L2 then sees each piece of A once for the column tiles that share it),
// column tile fastest.
struct StatMap {
    int tiles_n, msplit, chunk_rows, total, xcds;
};

template <typename T, bool TRANS_B, int KP>       // KP: 64-deep pieces of the contraction (K <= 64 KP)
__global__ __launch_bounds__(SWAVES * 64, 2) void gemm_mfma_bstat_kernel(Problem p, StatMap map) {
    constexpr int KS = 2 * KP;                    // MFMA k-steps
    constexpr int ROWS = KP <= 2 ? SBM : SBM / 2; // rows per step
    constexpr int S_PIECE = ROWS * 64 * 2;        // a 64-deep piece of a step's rows: 8 or 4 KiB
    constexpr int A_STAGE = KP * S_PIECE;
    constexpr int A_LOADS = KP * (ROWS / 8) / SWAVES;      // 1 KiB direct-to-LDS loads per wave and step
    extern __shared__ __attribute__((aligned(1024))) char lds[];     // S_STAGES A stages | 4 epilogue slices | bias

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);

    int id;
    {
        const int q = map.total / map.xcds, r = map.total % map.xcds;
        const int xcd = blockIdx.x % map.xcds, local = blockIdx.x / map.xcds;
        id = xcd * q + (xcd < r ? xcd : r) + local;
    }
    const int tn = id % map.tiles_n;
    const int rest = id / map.tiles_n;
    const int mc = rest % map.msplit, b = rest / map.msplit;
    const int n0 = tn * SBN;
    const int m_begin = mc * map.chunk_rows;
    const int m_end = min(p.M, m_begin + map.chunk_rows);
    if (m_begin >= m_end) return;

    const char* Abase = (const char*)p.A + (int64_t)b * p.stride_a * 2;
    const char* Bbase = (const char*)p.B + (int64_t)b * p.stride_b * 2;
    const unsigned lds_base = (unsigned)__builtin_amdgcn_readfirstlane((int)lds_addr_of(lds));

    // ---- the stationary operand: fragments of this wave's 64 columns over the whole contraction
    short8v bf[SFN][KS];
    const int f_row = lane & 15, f_kc = lane >> 4;
    if (TRANS_B) {
        // [256 n][64 k] at a time through LDS in the layout of A's pieces (whole 128-byte lines per row)
#pragma unroll
        for (int h = 0; h < KP; ++h) {
            const int4v rb = make_rsrc(Bbase + (int64_t)n0 * p.ldb * 2);
#pragma unroll
            for (int r = 0; r < 32 / SWAVES; ++r) {
                const int blk = wave * (32 / SWAVES) + r;
                const int row = blk * 8 + (lane >> 3), slot = lane & 7;
                const int k = h * 64 + (slot ^ kmajor_swz<64, true>(row)) * 8;
                const bool ok = n0 + row < p.N && k < p.K;
                dma16(rb, lds_base + blk * 1024, ok ? (unsigned)(row * (int)p.ldb * 2 + k * 2) : kOob);
            }
            wait_vmcnt<0>();
            __syncthreads();
#pragma unroll
            for (int ksl = 0; ksl < 2; ++ksl)
#pragma unroll
                for (int j = 0; j < SFN; ++j)
                    bf[j][2 * h + ksl] = *(const short8v*)(lds + kmajor_offset<64, true>(wave * SWTN + j * 16 + f_row, ksl * 4 + f_kc));
            __syncthreads();                      // the area is overwritten next (second half of B, or A)
        }
    } else {
        // [64 k][256 n] at a time through LDS (32 KiB from the start of the workgroup's LDS)
        const int t16_k = ((lane & 15) >> 2) + ((lane >> 4) << 3);
        const int t16_nbyte = (lane & 3) * 8;
#pragma unroll
        for (int h = 0; h < KP; ++h) {
            const int4v rb = make_rsrc(Bbase + ((int64_t)h * 64 * p.ldb + n0) * 2);
#pragma unroll
            for (int r = 0; r < 32 / SWAVES; ++r) {
                const int blk = wave * (32 / SWAVES) + r;
                const int krow = blk * 2 + (lane >> 5), slot = lane & 31;
                const int c64 = (slot >> 2) ^ (krow & 3);
                const int nbyte = (c64 << 6) | (((slot & 3) << 4) ^ nmajor_half(krow));
                const bool ok = n0 + (nbyte >> 1) < p.N && h * 64 + krow < p.K;
                dma16(rb, lds_base + blk * 1024, ok ? (unsigned)(krow * (int)p.ldb * 2 + nbyte) : kOob);
            }
            wait_vmcnt<0>();
            __syncthreads();
#pragma unroll
            for (int ksl = 0; ksl < 2; ++ksl)
#pragma unroll
                for (int j = 0; j < SFN; ++j) {
                    const char* r0 = lds + nmajor_offset<SBN>(ksl * 32 + t16_k, (wave * SWTN + j * 16) * 2 + t16_nbyte);
                    short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PBK_LDS_PTR(short4v, r0));
                    short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PBK_LDS_PTR(short4v, r0 + 4 * (SBN * 2)));
                    bf[j][2 * h + ksl] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
            __syncthreads();                      // the area is overwritten next (second half of B, or A)
        }
    }

    // ---- the streamed operand: a step's piece of A is KP x 8 blocks of 1 KiB (8 rows x 128 bytes)
    unsigned a_voff[A_LOADS];
    int a_row[A_LOADS];
#pragma unroll
    for (int r = 0; r < A_LOADS; ++r) {
        const int blk = wave * A_LOADS + r;
        const int piece = blk / (ROWS / 8);
        const int row = (blk % (ROWS / 8)) * 8 + (lane >> 3), slot = lane & 7;
        const int chunk = slot ^ kmajor_swz<64, true>(row);
        const int k = piece * 64 + chunk * 8;
        a_row[r] = row;
        a_voff[r] = k < p.K ? (unsigned)(row * (int)p.lda * 2 + k * 2) : kOob;
    }
    auto issue_a = [&](int m, int stage) {
        const int4v ra = make_rsrc(Abase + (int64_t)m * p.lda * 2);
#pragma unroll
        for (int r = 0; r < A_LOADS; ++r)
            dma16(ra, lds_base + stage * A_STAGE + (wave * A_LOADS + r) * 1024, m + a_row[r] < m_end ? a_voff[r] : kOob);      // (m may lie beyond m_end)
    };

    // ---- epilogue state: the bias of the wave's 64 columns waits in LDS (registers are what limits the number
    // of workgroups per compute unit); a lane reads the 4 values of each of its column groups per half step
    float* wbias = (float*)(lds + S_STAGES * A_STAGE + SWAVES * S_SLICE) + wave * SWTN;
    {
        const int col = n0 + wave * SWTN + lane;
        wbias[lane] = (epi_has_bias(p.epi) && col < p.N) ? p.bias[col] : 0.0f;
    }
    char* wlds = lds + S_STAGES * A_STAGE + wave * S_SLICE;
    auto walk = [&](auto act_tag, auto f32_tag) __attribute__((always_inline)) {
        constexpr int ACT = decltype(act_tag)::value;
        constexpr bool OUT_F32 = decltype(f32_tag)::value;
        constexpr int ESZ = OUT_F32 ? 4 : 2;
        constexpr int EPC = 16 / ESZ;                       // elements per 16-byte chunk
        constexpr int ROW_BYTES = SWTN * ESZ;               // a row of the wave tile
        constexpr int CPR = ROW_BYTES / 16;
        constexpr int RP = 256 / ROW_BYTES;                 // rows per 256 bytes
        constexpr int ROWS_PER_ST = 64 / CPR;               // rows one store instruction covers
        constexpr int HALF_ROWS = 32, HFM = 2, NHALF = ROWS / HALF_ROWS;   // a step is worked off in halves of 32 rows (one or two)
        constexpr int PASS_ROWS = S_SLICE / ROW_BYTES < HALF_ROWS ? S_SLICE / ROW_BYTES : HALF_ROWS;
        constexpr int PASSES = HALF_ROWS / PASS_ROWS;
        constexpr int ST_PER_PASS = PASS_ROWS / ROWS_PER_ST;
        constexpr int NS = NHALF * PASSES * ST_PER_PASS;        // store instructions per wave and step, issued unconditionally
        static_assert(NS <= 32, "vmcnt range");
        const int ld_row = lane / CPR, ld_chunk = lane % CPR;
        // (out of range for a lane whose columns lie beyond N: adding a row offset below 2^31 keeps it there)
        const unsigned c_voff = n0 + wave * SWTN + ld_chunk * EPC < p.N ? (unsigned)(ld_row * (int)p.ldc * ESZ + ld_chunk * 16) : kOob;
        const char* Cbase = (const char*)p.C + ((int64_t)b * p.stride_c + n0 + wave * SWTN) * ESZ;
        // The pieces of A of the next two steps are in flight.  A wave's memory operations complete in issue
        // order, and per step it issues A_LOADS loads (always: a piece beyond the end of the rows gets the
        // out-of-range offset and fills a stage nobody reads) followed, at the end of the step, by NS stores
        // (always: buffer stores with the out-of-range offset where nothing is to be written).  So "this
        // step's piece has landed" is a fixed count of younger operations that may still be under way: the
        // stores of the two previous steps and the loads of the next piece.  The piece requested at the top
        // of step s therefore waits behind the stores of step s - 1 in the memory queue but is not needed
        // before step s + 2, and the stores of a step have two steps' time to drain.
        int stage = 0, step = 0;
        issue_a(m_begin, 0);
        issue_a(m_begin + ROWS, 1);
        for (int m = m_begin; m < m_end; m += ROWS, ++step) {
            asm volatile("" ::: "memory");        // (the previous step's stores are issued: the counts below rely on it)
            if (step == 0) wait_vmcnt<A_LOADS>();
            else if (step == 1) wait_vmcnt<A_LOADS + NS>();
            else wait_vmcnt<A_LOADS + 2 * NS>();
            // every wave's part of the piece has landed; every wave has left the previous step, whose stage is
            // refilled next
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const int refill = stage == 0 ? S_STAGES - 1 : stage - 1;
            issue_a(m + 2 * ROWS, refill);
            const char* sa = lds + stage * A_STAGE;
            const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc(
                (void*)(Cbase + (int64_t)m * p.ldc * ESZ), 0, (int)kOob, 0x00020000);
            // the step in halves of 32 rows: 32 accumulators are live at a time
#pragma unroll
            for (int hf = 0; hf < NHALF; ++hf) {
                f32x4 acc[HFM][SFN];
#pragma unroll
                for (int i = 0; i < HFM; ++i)
#pragma unroll
                    for (int j = 0; j < SFN; ++j)
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.0f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    short8v af[HFM];
#pragma unroll
                    for (int i = 0; i < HFM; ++i)
                        af[i] = *(const short8v*)(sa + (ks >> 1) * S_PIECE +
                                                  kmajor_offset<64, true>((hf * HFM + i) * 16 + f_row, (ks & 1) * 4 + f_kc));
#pragma unroll
                    for (int i = 0; i < HFM; ++i)
#pragma unroll
                        for (int j = 0; j < SFN; ++j) acc[i][j] = MfmaOp16<T>::run(bf[j][ks], af[i], acc[i][j]);
                }
                // epilogue in registers, then once through the wave's LDS slice (16-byte chunks XOR-swizzled by
                // the row) so that a store instruction writes whole rows of the wave tile
#pragma unroll
                for (int ps = 0; ps < PASSES; ++ps) {
#pragma unroll
                    for (int ii = 0; ii < PASS_ROWS / 16; ++ii) {
                        const int i = ps * (PASS_ROWS / 16) + ii;
                        const int lrow = ii * 16 + f_row;
                        const int sw = (lrow / RP) % CPR;
#pragma unroll
                        for (int j = 0; j < SFN; ++j) {
                            float v[4];
                            const f32x4 bias4 = *(const f32x4*)(wbias + j * 16 + f_kc * 4);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                float x = fmaf(p.alpha, acc[i][j][e], bias4[e]);
                                if (ACT == 1) x = relu_keep_nan(x);
                                if (ACT == 2) x = gelu_tanh_f32(x);
                                v[e] = x;
                            }
                            const int cbyte = (j * 16 + f_kc * 4) * ESZ;
                            char* dst = wlds + lrow * ROW_BYTES + (((cbyte >> 4) ^ sw) << 4) + (cbyte & 15);
                            if (OUT_F32) {
                                *(f32x4*)dst = f32x4{v[0], v[1], v[2], v[3]};
                            } else {
                                *(int2v*)dst = int2v{(int)pack2<T>(v[0], v[1]), (int)pack2<T>(v[2], v[3])};
                            }
                        }
                    }
                    int4v w[ST_PER_PASS];
#pragma unroll
                    for (int q = 0; q < ST_PER_PASS; ++q) {
                        const int lrow = q * ROWS_PER_ST + ld_row;
                        const int sw = (lrow / RP) % CPR;
                        w[q] = *(const int4v*)(wlds + lrow * ROW_BYTES + ((ld_chunk ^ sw) << 4));
                    }
#pragma unroll
                    for (int q = 0; q < ST_PER_PASS; ++q) {
                        const int grow = hf * HALF_ROWS + ps * PASS_ROWS + q * ROWS_PER_ST;   // + ld_row: the lane's row in the step
                        const unsigned off = c_voff + (unsigned)(grow * (int)p.ldc * ESZ);
                        __builtin_amdgcn_raw_buffer_store_b128(w[q], rc, m + grow + ld_row < m_end ? off : kOob, 0, 0);
                    }
                }
            }
            stage = stage + 1 == S_STAGES ? 0 : stage + 1;
        }
        // the last two requests for A lie beyond the rows and only clear a stage: they have ended (all but the
        // last step's stores have) before the wave gives its LDS back
        wait_vmcnt<NS>();
    };
    const int act = (p.epi == EPI_RELU || p.epi == EPI_BIAS_RELU) ? 1
                  : (p.epi == EPI_GELU_TANH || p.epi == EPI_BIAS_GELU_TANH) ? 2 : 0;
    if (p.out_dtype == DT_F32) {
        if (act == 0) walk(IntTag<0>{}, BoolTag<true>{}); else if (act == 1) walk(IntTag<1>{}, BoolTag<true>{});
        else walk(IntTag<2>{}, BoolTag<true>{});
    } else {
        if (act == 0) walk(IntTag<0>{}, BoolTag<false>{}); else if (act == 1) walk(IntTag<1>{}, BoolTag<false>{});
        else walk(IntTag<2>{}, BoolTag<false>{});
    }
}

template <typename T, bool TRANS_B, int KP>
hipError_t launch_bstat_one(const Problem& p, hipStream_t stream) {
    auto kern = gemm_mfma_bstat_kernel<T, TRANS_B, KP>;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    DeviceShape ds;
    e = device_shape(dev, &ds);
    if (e != hipSuccess) return e;
    // the LDS a workgroup needs: two stages of A and the epilogue slices; B is staged 32 KiB at a time
    constexpr int ROWS = KP <= 2 ? SBM : SBM / 2;
    int lds_bytes = S_STAGES * KP * ROWS * 128 + SWAVES * S_SLICE + SBN * 4;
    if (lds_bytes < 32768) lds_bytes = 32768;
    static std::atomic<unsigned> attr_done{0};      // bit per device
    const unsigned bit = 1u << (dev & 31);
    if (!(attr_done.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_done.fetch_or(bit, std::memory_order_release);
    }
    StatMap map;
    map.tiles_n = (p.N + SBN - 1) / SBN;
    const int steps = (p.M + SBM - 1) / SBM;
    // rows per workgroup: as long a walk as still gives every slot of the chip (two workgroups per compute
    // unit) a workgroup, at least 4 steps (B is fetched once per workgroup)
    const long long cols = (long long)map.tiles_n * p.batch;
    const long long slots = (long long)ds.cus * 2;
    int split = (int)(slots / cols);
    if (split > steps / 4) split = steps / 4;
    if (split < 1) split = 1;
    int chunk_steps = (steps + split - 1) / split;
    map.chunk_rows = chunk_steps * SBM;
    map.msplit = (steps + chunk_steps - 1) / chunk_steps;
    const long long total = cols * map.msplit;
    if (total <= 0 || total > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    map.total = (int)total;
    map.xcds = ds.xcds;
    Problem pa = p;
    void* args[] = {&pa, &map};
    return hipLaunchKernel((const void*)kern, dim3((unsigned)total), dim3(SWAVES * 64), args, lds_bytes, stream);
}

template <typename T>
hipError_t launch_bstat_type(const Problem& p, hipStream_t stream) {
    if (p.K <= 64)
        return p.trans_b ? launch_bstat_one<T, true, 1>(p, stream) : launch_bstat_one<T, false, 1>(p, stream);
    if (p.K <= 128)
        return p.trans_b ? launch_bstat_one<T, true, 2>(p, stream) : launch_bstat_one<T, false, 2>(p, stream);
    if (p.K <= 192)
        return p.trans_b ? launch_bstat_one<T, true, 3>(p, stream) : launch_bstat_one<T, false, 3>(p, stream);
    return p.trans_b ? launch_bstat_one<T, true, 4>(p, stream) : launch_bstat_one<T, false, 4>(p, stream);
}

}  // namespace

// 16-bit plain matrices (no convolution) that meet the direct-to-LDS kernel's alignment rules, K <= 256
bool mfma_bstat_supported(const Problem& p) {
    if (p.in_dtype != DT_BF16 && p.in_dtype != DT_F16) return false;
    if (p.is_conv || p.K > 256 || p.R) return false;
    if (p.M > 0x7FFFFFFF - 4 * SBM) return false;       // (the walk requests pieces up to two steps beyond its last row)
    // whole aligned 16-byte chunks of C (the stores are 16 bytes per lane, per-lane offsets 32-bit)
    const int esz = p.out_dtype == DT_F32 ? 4 : 2, epc = 16 / esz;
    if (p.N % epc || p.ldc % epc || p.stride_c % epc || (reinterpret_cast<uintptr_t>(p.C) & 15)) return false;
    if ((int64_t)SBM * p.ldc * esz + 4096 >= ((int64_t)1 << 31)) return false;
    return mfma_supported(p);
}

// Where it is ahead of the tile-per-workgroup configurations: store-bound problems with enough rows for a
// workgroup to walk and enough columns for its 256-wide strip
bool mfma_bstat_preferred(const Problem& p) {
    if (p.M < 512 || p.N < 256) return false;
    const long long steps = (long long)((p.M + SBM - 1) / SBM) * ((p.N + SBN - 1) / SBN) * p.batch;
    return steps >= 1536;
}

hipError_t launch_mfma_bstat(const Problem& p, hipStream_t stream, const char** name) {
    *name = p.K <= 64 ? "mfma16_bstat_64x256_k64_w1x4_occ2" : p.K <= 128 ? "mfma16_bstat_64x256_k128_w1x4_occ2"
          : p.K <= 192 ? "mfma16_bstat_32x256_k192_w1x4_occ2" : "mfma16_bstat_32x256_k256_w1x4_occ2";
    return p.in_dtype == DT_BF16 ? launch_bstat_type<bf16_t>(p, stream) : launch_bstat_type<f16_t>(p, stream);
}

}  // namespace pbk
