// Fused attention kernel for gfx950: O = softmax(alpha Q K^T + bias) V with the
// scores, the softmax and the weights living only in registers.
//
// This is the hand-written counterpart of what the paper reaches with its
// reduce-reduce fusion (the softmax reductions and the second matmul fused
// into the key loop of the first, with a correction applied to the running
// output whenever the running row maximum moves) and its matrix-unit fusion
// (nothing between the two matmuls goes back to on-chip memory), Sec. 4.4.
//
// Work split: a workgroup of 4 waves owns 128 query rows of one batch entry,
// each wave 32 of them, and walks the keys in tiles of 64, two blocks of 32
// each.  K and V tiles are shared by the 4 waves: they are fetched straight
// into LDS (buffer_load ... lds, double buffered, one barrier per tile), rows
// beyond Nk arrive as zeros.  The scores of block j+1 are computed while block
// j's exponentials run, so the K tiles are shifted by half a tile against the V
// tiles; the weights of block j multiply V while block j+1's row maximum is
// found.  Two workgroups share a CU, so that one wave's softmax arithmetic
// also overlaps the other's MFMAs on every SIMD.  The tiles that lie entirely
// inside the key range (and below the causal diagonal) run in an instance of
// the loop body without any range test: a body with branches is split into
// basic blocks, and the compiler then sinks the softmax arithmetic out of the
// MFMA slots it was written into.
//
// Register layouts (v_mfma_f32_32x32x16, D[i][j] += sum_k A[i][k] B[k][j]; a lane
// supplies row i = lane%32 of A and column j = lane%32 of B, 8 consecutive k
// starting at 8*(lane/32), and receives column j = lane%32, rows
// 8g + 4*(lane/32) + t of D in register 4g + t):
//   S^T = K Q^T:  A = K rows from LDS (k-major, ds_read_b128), B = Q (registers,
//                 loaded once).  A lane then holds 16 scores of ONE query per
//                 32-key block: the row maximum and sum need one exchange with
//                 lane^32 only, and the correction factor is a per-lane scalar.
//   O^T = V^T P^T: B = the lane's own weights, rounded to 16 bits, taken in
//                 the key order the lane already holds them (contraction order
//                 is free as long as both operands agree); A = V^T produced by
//                 the transposing LDS read from the d-contiguous V tile with the
//                 matching key order.  No weight ever changes lane or touches LDS.
#include "gemm_mfma_launch.h"
#include <type_traits>

namespace pbk {
namespace {

constexpr int ATT_BQ = 128;     // query rows per workgroup
constexpr int ATT_BKV = 64;     // keys per tile
constexpr int ATT_NW = 4;
constexpr float ATT_SLACK = 8.0f; // log2 of how far a block's scores may exceed the softmax reference point

// 64-byte-chunk swizzle of the d-contiguous V tile [keys][D]: rows that share
// LDS banks (256-byte period) get different chunk positions.
template <int D> __device__ __forceinline__ int v_swz(int key) {
    constexpr int RPB = 256 / (D * 2) > 0 ? 256 / (D * 2) : 1;   // rows per bank period
    constexpr int C64 = (D * 2) / 64;                            // 64-byte chunks per row
    return (key / RPB) % C64;
}
template <int D> __device__ __forceinline__ int v_offset(int key, int dbyte) {
    return key * (D * 2) + ((((dbyte >> 6) ^ v_swz<D>(key)) << 6) | (dbyte & 63));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// dma16 for operands that are already scalar: the descriptor comes from make_rsrc (its
// address words went through readfirstlane) and the LDS address from a scalar base plus a
// constant, so nothing has to be made uniform again for every load.
__device__ __forceinline__ void dma16_s(int4v rsrc, unsigned lds_addr, unsigned voff) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_addr), "v"(voff), "s"(rsrc) : "memory", "m0");
}

// HAS_BIAS: an additive bias is read.  PRE: scores are multiplied by alpha*log2(e) (and the
// bias added) before the row maximum is taken; without it (no bias, alpha > 0) the maximum is
// taken on the raw scores and the scaling rides in the multiply-add in front of the exponential.
// CAUSAL: query q attends to keys <= q + (Nk - Nq).  The key tiles beyond the workgroup's last visible key
// are not visited at all; in the blocks that the diagonal crosses the hidden scores are set to -inf like
// the keys beyond Nk.
template <typename T, int D, bool HAS_BIAS, bool PRE, bool CAUSAL>
__global__ __launch_bounds__(ATT_NW * 64, 2) void attention_mfma_kernel(AttnProblem p, int q_tiles, int total, int xcds) {
    constexpr int KS = D / 16;                    // k16 steps of Q K^T
    constexpr int JD = D / 32;                    // 32-wide blocks of the head dimension
    constexpr int NPV = 2 * JD;                   // MFMAs of O^T += V^T P^T per 32-key block
    constexpr int TILE = ATT_BKV * D * 2;         // bytes of one K or V tile
    constexpr int BLKS = TILE / 1024;             // 1 KiB wave-loads per tile
    constexpr int CPW = BLKS / ATT_NW;            // per wave
    static_assert(BLKS % ATT_NW == 0 && CPW >= 1, "tile must split evenly over the waves");
    constexpr int CPR = D / 8;                    // 16-byte slots per row
    constexpr int ROWS = 64 / CPR;                // rows per wave-load
    constexpr float LOG2E = 1.4426950408889634f;

    // K slot 0 | K slot 1 | V slot 0 | V slot 1
    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = lane >> 5, col = lane & 31;

    // workgroups are dealt round-robin to the 8 XCDs: regroup so that one XCD (one L2)
    // owns a contiguous run of (batch, query tile) pairs and re-uses that batch's K and V
    const int xq = total / xcds, xr = total % xcds;
    const int xcd = blockIdx.x % xcds, local = blockIdx.x / xcds;
    const int id = xcd * xq + (xcd < xr ? xcd : xr) + local;
    const int b = id / q_tiles;
    // (causal: the last query tiles have the most keys to visit and are started first)
    const int q_tile = CAUSAL ? q_tiles - 1 - (id - b * q_tiles) : id - b * q_tiles;
    const int q0 = q_tile * ATT_BQ + wave * 32;
    const int c_off = p.Nk - p.Nq;                 // causal: key visible iff key <= query + c_off

    const char* Kb = (const char*)p.K + (int64_t)b * p.stride_k * 2;
    const char* Vb = (const char*)p.V + (int64_t)b * p.stride_v * 2;

    // ---- per-lane source offsets of the direct-to-LDS loads (lane i lands at byte 16 i)
    unsigned k_voff[CPW], v_voff[CPW];
    int ld_row[CPW];
#pragma unroll
    for (int r = 0; r < CPW; ++r) {
        const int row = (wave * CPW + r) * ROWS + lane / CPR;
        const int slot = lane % CPR;
        ld_row[r] = row;
        k_voff[r] = (unsigned)(row * (int)p.ldk * 2 + ((slot ^ kmajor_swz<D>(row)) << 4));
        const int c64 = (slot >> 2) ^ v_swz<D>(row);
        v_voff[r] = (unsigned)(row * (int)p.ldv * 2 + ((c64 << 6) | ((slot & 3) << 4)));
    }
    const unsigned lds_base = (unsigned)__builtin_amdgcn_readfirstlane((int)lds_addr_of(lds));
    // V tile t: keys [64 t, 64 t + 64).
    auto issue_v = [&](int t) {
        const int key0 = t * ATT_BKV;
        const int4v rv = make_rsrc(Vb + (int64_t)key0 * p.ldv * 2);
        const unsigned sv = lds_base + (2 + (t & 1)) * TILE;
        if (key0 + ATT_BKV <= p.Nk) {             // whole tile inside: no per-lane test (wave-uniform)
#pragma unroll
            for (int r = 0; r < CPW; ++r) dma16_s(rv, sv + (wave * CPW + r) * 1024, v_voff[r]);
        } else {
#pragma unroll
            for (int r = 0; r < CPW; ++r)
                dma16_s(rv, sv + (wave * CPW + r) * 1024, key0 + ld_row[r] < p.Nk ? v_voff[r] : kOob);
        }
    };
    // K tile t is shifted by half a tile: keys [64 t + 32, 64 t + 96), because the scores of
    // a 32-key block are computed one block ahead of its softmax.  t = -1 holds keys [0, 32)
    // in its upper half.
    auto issue_k = [&](int t) {
        const int key0 = t * ATT_BKV + 32;
        const unsigned sk = lds_base + (t & 1) * TILE;
        if (t < 0) {
            const int4v rk = make_rsrc(Kb);
#pragma unroll
            for (int r = 0; r < CPW; ++r) {
                const bool ok = ld_row[r] >= 32 && ld_row[r] - 32 < p.Nk;
                dma16_s(rk, sk + (wave * CPW + r) * 1024, ok ? k_voff[r] - (unsigned)(32 * (int)p.ldk * 2) : kOob);
            }
        } else {
            const int4v rk = make_rsrc(Kb + (int64_t)key0 * p.ldk * 2);
            if (key0 + ATT_BKV <= p.Nk) {
#pragma unroll
                for (int r = 0; r < CPW; ++r) dma16_s(rk, sk + (wave * CPW + r) * 1024, k_voff[r]);
            } else {
#pragma unroll
                for (int r = 0; r < CPW; ++r)
                    dma16_s(rk, sk + (wave * CPW + r) * 1024, key0 + ld_row[r] < p.Nk ? k_voff[r] : kOob);
            }
        }
    };

    int NT = (p.Nk + ATT_BKV - 1) / ATT_BKV;
    if (CAUSAL) {
        // the workgroup's last visible key (at least one tile is walked, so that every wave meets the barriers)
        const long long last = (long long)q_tile * ATT_BQ + ATT_BQ - 1 + c_off;
        const int nt_vis = last < 0 ? 1 : (int)(last / ATT_BKV) + 1;
        NT = nt_vis < NT ? nt_vis : NT;
    }
    issue_k(-1);
    issue_v(0);
    issue_k(0);

    // ---- Q fragments: column q = lane%32, d = 16 ks + 8 h .. +8, straight from global
    Frag<1> qf[KS];
    {
        const int q = q0 + col;
        const char* qp = (const char*)p.Q + ((int64_t)b * p.stride_q + (int64_t)q * p.ldq) * 2;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            short8v v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (q < p.Nq) v = *(const short8v*)(qp + (ks * 16 + h * 8) * 2);
            qf[ks].c[0] = v;
        }
    }

    f32x16 o_acc[JD];
#pragma unroll
    for (int j = 0; j < JD; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) o_acc[j][e] = 0.0f;
    float m_run = -INFINITY;      // softmax reference point of the row (log2 domain), same in lane and lane^32
    float l_run = 0.0f;           // this lane's share of the running row sum
    float neg_m = 0.0f;           // minus the reference point (0 while it is still -inf)
    float thr = -INFINITY;        // a score above this (before scaling unless PRE) moves the reference point

    const float c1 = p.alpha * LOG2E;
    const bool bias_vec = HAS_BIAS && (((uintptr_t)p.bias & 15) == 0) && (p.ld_bias % 4 == 0) && (p.stride_bias % 4 == 0);
    const float* bias_row = HAS_BIAS ? p.bias + (int64_t)b * p.stride_bias + (int64_t)(q0 + col) * p.ld_bias : nullptr;
    const bool q_ok = q0 + col < p.Nq;

    // transposing-read lane constants: key (lane%16)/4 + 4h within a 16-key step, d = 4*(lane%4) of a 16-wide block
    const int tr_key = ((lane & 15) >> 2) + (h << 2);
    const int tr_dbyte = ((((lane >> 4) & 1) << 4) + ((lane & 3) << 2)) * 2;

    // Per-lane LDS offsets of the fragment reads; slot, block and step only add constants
    // (both swizzles are periodic in 8 rows), which go into the instructions' offset fields.
    int koff[KS], voff[JD];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) koff[ks] = kmajor_offset<D>(col, ks * 2 + h);
#pragma unroll
    for (int j = 0; j < JD; ++j) voff[j] = v_offset<D>(tr_key, j * 64 + tr_dbyte);

    // K fragments of one 32-key block are read KPF k16 steps ahead of the MFMA that uses them
    constexpr int KPF = KS < 3 ? KS : 3;
    Frag<1> kfr[4];
    auto read_k = [&](int cbyte, int ks) {        // cbyte: slot and block offset, compile-time at every call
        kfr[ks & 3].c[0] = *(const short8v*)(lds + koff[ks] + cbyte);
    };
    // V^T fragments of one 32-key block: 2 steps of 16 keys x JD blocks of 32 d, read one per score MFMA
    Frag<1> vfr[2][JD];
    auto read_v1 = [&](int cbyte, int f) {       // fragment f = st * JD + j, in the order the P V MFMAs use them
        const int st = f / JD, j = f % JD;
        short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PBK_LDS_PTR(short4v, lds + voff[j] + cbyte + (st * 16) * (D * 2)));
        short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PBK_LDS_PTR(short4v, lds + voff[j] + cbyte + (st * 16 + 8) * (D * 2)));
        vfr[st][j].c[0] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    // Scores of a block, in place.  Register 4g + t is key kbase + 8 g + 4 h + t.  Elements [e0, e1).
    // PRE: to the log2 domain (times alpha*log2 e), plus bias.  Keys beyond Nk are removed
    // (RAGGED blocks only).
    auto scale_scores = [&](f32x16& sv, int kbase, const float (&bias)[16], auto ragged_tag, int e0, int e1) {
        constexpr bool RAGGED = decltype(ragged_tag)::value;
        if (!PRE && !RAGGED) return;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            if (e < e0 || e >= e1) continue;
            float v = sv[e];
            if (PRE) v *= c1;
            if (HAS_BIAS) v = fmaf(bias[e], LOG2E, v);
            if (RAGGED) {
                const int key = kbase + (e >> 2) * 8 + h * 4 + (e & 3);
                if (key >= p.Nk || (CAUSAL && key > q0 + col + c_off)) v = -INFINITY;
            }
            sv[e] = v;
        }
    };
    auto load_bias = [&](int kbase, float (&bias)[16]) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int key = kbase + g * 8 + h * 4;
            float bv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (q_ok) {
                if (bias_vec && key + 3 < p.Nk) {
                    f32x4 v4 = *(const f32x4*)(bias_row + key);
                    bv[0] = v4[0]; bv[1] = v4[1]; bv[2] = v4[2]; bv[3] = v4[3];
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        if (key + t < p.Nk) bv[t] = bias_row[key + t];
                }
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) bias[g * 4 + t] = bv[t];
        }
    };
    auto block_max = [&](const f32x16& sv) {
        float m = -INFINITY;
#pragma unroll
        for (int e = 0; e < 16; ++e) m = fmaxf(m, sv[e]);
        return PRE ? m : m * c1;          // c1 > 0 without PRE: the maximum commutes with the scaling
    };
    auto exchange_max = [&](float v) {                       // maximum with lane ^ 32, no LDS round trip
        const unsigned u = __builtin_bit_cast(unsigned, v);
        auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        return fmaxf(__builtin_bit_cast(float, (unsigned)r[0]), __builtin_bit_cast(float, (unsigned)r[1]));
    };
    // The reference point m_run only has to stay within 2^ATT_SLACK of the true running
    // maximum for nothing to overflow: it is moved (and the accumulated sum and output
    // corrected) only when a block exceeds it by more than that.  Weights and sum use the
    // same reference, so the quotient is unchanged.  bmax: block maximum of the row (both halves).
    auto move_reference = [&](float bmax) {
        const bool move = bmax > m_run + ATT_SLACK;                 // same in lane and lane^32
        const float m_new = move ? bmax : m_run;
        const float m_sub = m_new == -INFINITY ? 0.0f : m_new;   // every key so far removed by a -inf bias
        const float corr = fast_exp2(m_run - m_sub);             // 1 where the lane does not move
        m_run = m_new;
        neg_m = -m_sub;
        thr = PRE ? m_new + ATT_SLACK : (m_new + ATT_SLACK) / c1;
        l_run *= corr;
#pragma unroll
        for (int j = 0; j < JD; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) o_acc[j][e] *= corr;
    };
    // The test that runs for every block is a per-lane one on the lane's own half of the row, against the
    // threshold kept in the units of the scores; only when some lane of the wave exceeds it are the halves
    // exchanged and the reference points moved.
    auto check_reference = [&](float half_max) {
        if (__builtin_amdgcn_ballot_w64(half_max > thr) != 0)
            move_reference(exchange_max(PRE ? half_max : half_max * c1));
    };

    // ---- prologue: scores of block 0 (keys 0..31, upper half of K slot 1), its reference point
    f32x16 s_blk[2];              // scores / weights of the block being consumed and of the next one
    wait_vmcnt<0>();
    __syncthreads();
    {
#pragma unroll
        for (int e = 0; e < 16; ++e) s_blk[0][e] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            read_k(TILE + 32 * D * 2, ks);
            s_blk[0] = MfmaOp<T>::run(kfr[ks & 3], qf[ks], s_blk[0]);
        }
        float bias0[16];
        if (HAS_BIAS) load_bias(0, bias0);
        if (32 > p.Nk || (CAUSAL && 31 > q0 + c_off)) scale_scores(s_blk[0], 0, bias0, TailYes{}, 0, 16);
        else scale_scores(s_blk[0], 0, bias0, TailNo{}, 0, 16);
        float bmax = block_max(s_blk[0]);
        bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
        move_reference(bmax);
    }

    // ---- main loop over 64-key tiles, two 32-key blocks each.  A block j (scores already in
    // registers) takes 2 KS' MFMAs: the KS of the NEXT block's scores, then the NPV of its own
    // weights times V; the softmax arithmetic is dealt over the slots behind these MFMAs so that
    // every MFMA has about the same number of vector instructions behind it:
    //   behind score MFMA ks:        exponentials of weight pairs [ks NP1/KS, (ks+1) NP1/KS)
    //   behind P V MFMA (st 0, j):   the remaining pairs (they feed st 1), scaling / masking of the next scores
    //   behind P V MFMA (st 1, j):   row sum of the rounded weights, the lane's maximum of the next scores
    // PAR: parity of the tile = LDS slot, compile-time so that every LDS address is a per-lane
    // register plus an immediate.  CLEAN: the tile, the two score blocks computed in it and the
    // next tile's loads are all inside the key range (and below the diagonal): no test, no branch
    // other than the rare move of the reference point, so the body is one basic block and the
    // order written here is the order that runs.
    constexpr int NP1 = 5;                                    // weight pairs finished under the score MFMAs (st 0 needs 4)
    auto pair_sum = [&](int w, float acc) {                  // acc + both 16-bit weights of w
        if constexpr (sizeof(T) == 2 && std::is_same<T, bf16_t>::value) {
            typedef __attribute__((ext_vector_type(2))) __bf16 b2;
            const b2 one = {(__bf16)1.0f, (__bf16)1.0f};
            return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(b2, w), one, acc, false);
        } else {
            typedef __attribute__((ext_vector_type(2))) _Float16 h2;
            const h2 one = {(_Float16)1.0f, (_Float16)1.0f};
            return __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, w), one, acc, false);
        }
    };
    auto issue_in = [&](int t) {                              // tile t's V and K, every row inside the key range
        const int4v rv = make_rsrc(Vb + (int64_t)t * ATT_BKV * p.ldv * 2);
        const unsigned sv = lds_base + (2 + (t & 1)) * TILE;
#pragma unroll
        for (int r = 0; r < CPW; ++r) dma16_s(rv, sv + (wave * CPW + r) * 1024, v_voff[r]);
        const int4v rk = make_rsrc(Kb + (int64_t)(t * ATT_BKV + 32) * p.ldk * 2);
        const unsigned sk = lds_base + (t & 1) * TILE;
#pragma unroll
        for (int r = 0; r < CPW; ++r) dma16_s(rk, sk + (wave * CPW + r) * 1024, k_voff[r]);
    };
    auto tile = [&](int t, auto par_tag, auto clean_tag) {
        constexpr int PAR = decltype(par_tag)::value;
        constexpr bool CLEAN = decltype(clean_tag)::value;
        wait_vmcnt<0>();              // this wave's pieces of V(t), K(t) have landed
        __syncthreads();              // everyone's have; everyone is done with V(t-1), K(t-1)
        // the first fragment reads of the tile go out before the (scalar-heavy) issue of the
        // next tile's loads, which hides their LDS latency
#pragma unroll
        for (int ks = 0; ks < KPF; ++ks) read_k(PAR * TILE, ks);
        __builtin_amdgcn_sched_barrier(0);
        // Without a bias the next tile's loads go out right away.  With one, the bias is read
        // with ordinary loads whose completion (vmcnt counts every vector memory operation, in
        // order) would also wait for direct-to-LDS loads issued before them: the first block's
        // bias is therefore requested now, while nothing else is in flight, and the tile loads
        // are issued after it has been consumed.
        float bias_first[16];
        if (HAS_BIAS) load_bias(t * ATT_BKV + 32, bias_first);
        else if (CLEAN) issue_in(t + 1);
        else if (t + 1 < NT) { issue_v(t + 1); issue_k(t + 1); }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
            f32x16& s_cur = s_blk[hb];
            f32x16& s_nxt = s_blk[hb ^ 1];
            const int kcb = PAR * TILE + 32 * hb * (D * 2);           // K rows of the next block
            const int vcb = (2 + PAR) * TILE + 32 * hb * (D * 2);     // V rows of this block
            const int knext = t * ATT_BKV + 32 * hb + 32;             // first key of the next block
            int pw[8];                 // the block's 16 weights, rounded and packed in pairs
            auto weights = [&](int i) {
                const float p0 = fast_exp2(PRE ? s_cur[2 * i] + neg_m : fmaf(s_cur[2 * i], c1, neg_m));
                const float p1 = fast_exp2(PRE ? s_cur[2 * i + 1] + neg_m : fmaf(s_cur[2 * i + 1], c1, neg_m));
                pw[i] = (int)pack2<T>(p0, p1);
            };

            // ---- scores of the next block, weights of this one
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks + KPF < KS) read_k(kcb, ks + KPF);
                // one V fragment of this block per score MFMA (there are KS = 2 JD of each), in the order of
                // their use: no burst of LDS reads stands between the blocks
                read_v1(vcb, ks);
                __builtin_amdgcn_sched_barrier(0);
                if (ks == 0) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) s_nxt[e] = 0.0f;
                }
                s_nxt = MfmaOp<T>::run(kfr[ks & 3], qf[ks], s_nxt);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (i >= ks * NP1 / KS && i < (ks + 1) * NP1 / KS) weights(i);
                __builtin_amdgcn_sched_barrier(0);
            }

            // ---- weights times V
            float biasn[16];
            if (HAS_BIAS) {
                if (hb == 0) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) biasn[e] = bias_first[e];
                } else {
                    load_bias(knext, biasn);
                }
            }
            // wave-uniform: the block reaches beyond Nk, or beyond what the wave's first query sees
            const bool ragged = !CLEAN && (knext + 32 > p.Nk || (CAUSAL && knext + 31 > q0 + c_off));
            float bmax = -INFINITY;
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                Frag<1> pf;
                int4v pv = {pw[4 * st], pw[4 * st + 1], pw[4 * st + 2], pw[4 * st + 3]};
                pf.c[0] = __builtin_bit_cast(short8v, pv);
#pragma unroll
                for (int j = 0; j < JD; ++j) {
                    o_acc[j] = MfmaOp<T>::run(vfr[st][j], pf, o_acc[j]);
                    __builtin_amdgcn_sched_barrier(0);
                    if (hb == 0 && st == 1 && j == 0) {
                        // the score MFMAs are done with the K fragment registers: the first fragments of the
                        // tile's second block are fetched now (same K slot, rows 32..63)
#pragma unroll
                        for (int ks = 0; ks < KPF; ++ks) read_k(PAR * TILE + 32 * (D * 2), ks);
                    }
                    if (st == 0) {
#pragma unroll
                        for (int i = NP1; i < 8; ++i)
                            if (i - NP1 >= j * (8 - NP1) / JD && i - NP1 < (j + 1) * (8 - NP1) / JD) weights(i);
                        if (CLEAN) scale_scores(s_nxt, knext, biasn, TailNo{}, j * 16 / JD, (j + 1) * 16 / JD);
                        else if (ragged) scale_scores(s_nxt, knext, biasn, TailYes{}, j * 16 / JD, (j + 1) * 16 / JD);
                        else scale_scores(s_nxt, knext, biasn, TailNo{}, j * 16 / JD, (j + 1) * 16 / JD);
                    } else {
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            if (i >= j * 8 / JD && i < (j + 1) * 8 / JD) l_run = pair_sum(pw[i], l_run);
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            if (e >= j * 16 / JD && e < (j + 1) * 16 / JD) bmax = fmaxf(bmax, s_nxt[e]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            check_reference(bmax);
            if (HAS_BIAS && hb == 0 && t + 1 < NT) { issue_v(t + 1); issue_k(t + 1); }
        }
    };
    // leading tiles that need no test: both score blocks computed in tile t end at key 64 t + 95, the loads
    // issued in it (tile t + 1) end at key 64 t + 159
    int n_clean = 0;
    if (!HAS_BIAS) {
        long long lim = ((long long)p.Nk - 160) / ATT_BKV + 1;
        if (p.Nk < 160) lim = 0;
        if (lim > NT - 1) lim = NT - 1;
        if (CAUSAL) {
            const long long vis = (long long)q0 + c_off - 95;          // 64 t <= vis
            const long long l3 = vis < 0 ? 0 : vis / ATT_BKV + 1;
            if (lim > l3) lim = l3;
        }
        n_clean = lim < 0 ? 0 : (int)(lim & ~1LL);
    }
    int t = 0;
    for (; t < n_clean; t += 2) {
        tile(t, IntTag<0>{}, TailYes{});
        tile(t + 1, IntTag<1>{}, TailYes{});
    }
    for (; t + 1 < NT; t += 2) {
        tile(t, IntTag<0>{}, TailNo{});
        tile(t + 1, IntTag<1>{}, TailNo{});
    }
    if (t < NT) tile(t, IntTag<0>{}, TailNo{});

    // ---- normalise and store: the lane holds, for query q0 + lane%32, d = 32 j + 8 g + 4 h + 0..3
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = 1.0f / l_tot;
    if (q_ok) {
        char* op = (char*)p.O + ((int64_t)b * p.stride_o + (int64_t)(q0 + col) * p.ldo) * 2;
#pragma unroll
        for (int j = 0; j < JD; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                int2v w;
                w[0] = (int)pack2<T>(o_acc[j][g * 4 + 0] * inv, o_acc[j][g * 4 + 1] * inv);
                w[1] = (int)pack2<T>(o_acc[j][g * 4 + 2] * inv, o_acc[j][g * 4 + 3] * inv);
                *(int2v*)(op + (j * 32 + g * 8 + h * 4) * 2) = w;
            }
    }
}

template <typename T, int D>
hipError_t launch_d(const AttnProblem& p, hipStream_t stream) {
    constexpr int LDS_BYTES = 2 * 2 * ATT_BKV * D * 2;
    const void* kern = p.causal ? (const void*)attention_mfma_kernel<T, D, false, false, true>
                       : p.bias ? (const void*)attention_mfma_kernel<T, D, true, true, false>
                       : p.alpha > 0.0f ? (const void*)attention_mfma_kernel<T, D, false, false, false>
                                        : (const void*)attention_mfma_kernel<T, D, false, true, false>;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    DeviceShape ds;
    e = device_shape(dev, &ds);
    if (e != hipSuccess) return e;
    int xcds = ds.xcds;
    int q_tiles = (p.Nq + ATT_BQ - 1) / ATT_BQ;
    long long total = (long long)q_tiles * p.batch;
    if (total <= 0 || total > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    int tot = (int)total;
    AttnProblem pa = p;
    void* args[] = {&pa, &q_tiles, &tot, &xcds};
    return hipLaunchKernel(kern, dim3((unsigned)total), dim3(ATT_NW * 64), args, LDS_BYTES, stream);
}

template <typename T>
hipError_t launch_t(const AttnProblem& p, hipStream_t stream, const char** name) {
    switch (p.D) {
    case 32: *name = p.causal ? "attn_mfma_q128_kv64_d32_causal" : "attn_mfma_q128_kv64_d32"; return launch_d<T, 32>(p, stream);
    case 64: *name = p.causal ? "attn_mfma_q128_kv64_d64_causal" : "attn_mfma_q128_kv64_d64"; return launch_d<T, 64>(p, stream);
    case 128: *name = p.causal ? "attn_mfma_q128_kv64_d128_causal" : "attn_mfma_q128_kv64_d128"; return launch_d<T, 128>(p, stream);
    default: return hipErrorInvalidValue;
    }
}

bool al(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace

// The fused kernel moves K and V in whole aligned 16-byte pieces and Q in
// 16-byte, O in 8-byte pieces.
bool attention_mfma_supported(const AttnProblem& p) {
    if (p.dtype != DT_BF16 && p.dtype != DT_F16) return false;
    if (p.D != 32 && p.D != 64 && p.D != 128) return false;
    if (p.causal && (p.bias || !(p.alpha > 0.0f))) return false;      // the causal form is built for the plain variant
    if (!al(p.Q, 16) || !al(p.K, 16) || !al(p.V, 16) || !al(p.O, 8)) return false;
    if (p.ldq % 8 || p.ldk % 8 || p.ldv % 8 || p.ldo % 4) return false;
    if (p.stride_q % 8 || p.stride_k % 8 || p.stride_v % 8 || p.stride_o % 4) return false;
    // per-lane buffer offsets are 32-bit and must stay below 2^31
    const int64_t lim = (int64_t)1 << 31;
    if (ATT_BKV * p.ldk * 2 + 256 >= lim || ATT_BKV * p.ldv * 2 + 256 >= lim) return false;
    return true;
}

hipError_t launch_attention_mfma(const AttnProblem& p, hipStream_t stream, const char** name) {
    return p.dtype == DT_BF16 ? launch_t<bf16_t>(p, stream, name) : launch_t<f16_t>(p, stream, name);
}

}  // namespace pbk
