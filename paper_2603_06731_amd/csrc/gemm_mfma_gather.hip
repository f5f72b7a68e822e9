// Matrix-unit contraction for 16-bit operands that the direct-to-LDS kernel cannot take: K, leading
// dimensions, N (row-major B) or the channel count of a convolution that are not multiples of 8,
// or bases that are not 16-byte aligned.  The paper's own worked example is of this kind (127 input
// channels, K = 1143: Sec. 4.5, partial tiles padded with zeros on the fly).
//
// Same tiling idea as the main kernel (Sec. 4.3 / 4.5 / 4.6), with the staging done through
// registers.  A piece is eight elements that are neighbours in memory (eight k of a row of a k-major
// operand, eight n of a k-row of a row-major B); every piece is ONE 16-byte load from an address that is
// only 2-byte aligned, issued unconditionally (so that the loads of three k-tiles can be in flight at
// any time: the compiler counts them).  What a piece must not contain is removed afterwards, in
// registers, when it is moved to LDS: elements beyond the end of K or of a filter tap are cleared,
// pieces that lie in the padding, beyond K or beyond M / N are cleared entirely; a piece whose 16 bytes
// would run over the end of the operand is read from 16 bytes before that end and shifted down.
// A convolution runs over a K axis in which every filter tap is rounded up to a multiple of eight
// channels (k' = tap * ceil8(Cin) + c), so that a piece never spans two taps; the weight rows of the
// padding channels are cleared like the image's.
// Pieces go to LDS in the main kernel's layouts: k-major [rows][32 k] with the 16-byte chunk index
// XOR-swizzled by the row (A, the image, a k-major B), n-major [32 k][128 n] read with the transposing
// LDS read (row-major B, weights).
// 128 x 128 x 32 tile, 2 x 2 waves, v_mfma_f32_16x16x32, LDS double-buffered: while k-tile t is
// multiplied, the pieces of k-tiles t+1 .. t+3 are in flight to registers; one barrier per k-tile.
// The epilogue is the main kernel's (registers, then the LDS shuffle or direct stores).
#include "gemm_mfma_launch.h"

namespace pbk {
namespace {

constexpr int GBM = 128, GBN = 128, GBK = 32;
constexpr int GWM = 2, GWN = 2;
constexpr int G_TILE_BYTES = GBM * GBK * 2;          // 8 KiB, the same for A and B
constexpr int G_STAGE = 2 * G_TILE_BYTES;

// 16 bytes from an address that is only known to be 2-byte aligned (one global_load_dwordx4)
// (the pointer is stated to be a global-memory one: a generic load would also count as an LDS operation)
__device__ __forceinline__ int4v ld_vec16(const char* ptr) {
    typedef const __attribute__((address_space(1))) char* global_ptr;
    int4v w;
    __builtin_memcpy(&w, (global_ptr)ptr, 16);
    return w;
}

// sixteen zero bytes in device memory: what a piece in the padding of an image, or a weight row of a padding
// channel, is read from (the load stays unconditional and the piece needs no clearing afterwards)
__device__ const int4v kZeroPiece = {0, 0, 0, 0};

// Where a piece is read from and what is kept of it: `meta` = number of leading elements to keep (0 .. 8)
// + 16 * number of elements to drop at the front first (the piece was read from that many elements
// before its place because 16 bytes from its place would have run over the end of the operand).
// kPlain = keep everything.
constexpr int kPlain = 8;
constexpr int kAllPlain = kPlain * 0x01010101;       // four pieces, one byte each
struct PieceSrc { const char* ptr; int meta; };

// want: address of the piece's first element (anything at or above the operand's base when !ok);
// last16: the last address of the operand from which 16 bytes can be read
__device__ __forceinline__ PieceSrc piece_src(const char* want, const char* last16, bool ok, int cnt) {
    PieceSrc s;
    s.ptr = want <= last16 ? want : last16;
    const int shift = (int)((want - s.ptr) >> 1);
    // a piece with at least one element inside the operand starts at most 14 bytes after last16
    s.meta = (ok && cnt > 0 && shift < 8) ? (cnt | (shift << 4)) : 0;
    return s;
}

__device__ __forceinline__ int4v piece_fix(int4v v, int meta) {
    const int cnt = meta & 15, shift = meta >> 4;
    unsigned w0 = (unsigned)v[0], w1 = (unsigned)v[1], w2 = (unsigned)v[2], w3 = (unsigned)v[3];
    if (shift) {
        if (shift & 4) { w0 = w2; w1 = w3; w2 = 0; w3 = 0; }
        if (shift & 2) { w0 = w1; w1 = w2; w2 = w3; w3 = 0; }
        if (shift & 1) {
            w0 = (w0 >> 16) | (w1 << 16); w1 = (w1 >> 16) | (w2 << 16);
            w2 = (w2 >> 16) | (w3 << 16); w3 >>= 16;
        }
    }
    auto keep = [&](unsigned w, int q) -> int {
        return (int)(cnt >= 2 * q + 2 ? w : cnt == 2 * q + 1 ? (w & 0xFFFFu) : 0u);
    };
    return int4v{keep(w0, 0), keep(w1, 1), keep(w2, 2), keep(w3, 3)};
}

template <typename T, int MODE>
__global__ __launch_bounds__(GWM * GWN * 64, 2) void gemm_mfma_gather_kernel(Problem p, TileMap tmap) {
    constexpr bool CONV = MODE == MODE_CONV;
    constexpr bool TRANS_B = MODE == MODE_TRANS_B;
    constexpr int NT = GWM * GWN * 64;
    constexpr int WTM = GBM / GWM, WTN = GBN / GWN;
    constexpr int FM = WTM / 16, FN = WTN / 16;
    constexpr int PIECES = GBM * (GBK / 8) / NT;     // 16-byte pieces of a tile per thread (2)
    static_assert(GBM == GBN && PIECES * NT == GBM * (GBK / 8), "tile geometry");

    extern __shared__ __attribute__((aligned(1024))) char lds[];        // 2 x (A tile | B tile)
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / GWN, wn = wave % GWN;

    int b, tile_m, tile_n;
    map_tile(tmap, blockIdx.x, b, tile_m, tile_n);
    const int m0 = tile_m * GBM, n0 = tile_n * GBN;
    const char* Abase = (const char*)p.A + (int64_t)b * p.stride_a * 2;
    const char* Bbase = (const char*)p.B + (int64_t)b * p.stride_b * 2;
    // the K axis the loop runs over: a convolution's taps rounded up to whole pieces
    const int Cp = CONV ? (p.conv.Cin + 7) & ~7 : 0;
    const int taps = CONV ? p.conv.KH * p.conv.KW : 0;
    const int Kloop = CONV ? taps * Cp : p.K;
    // the last addresses from which 16 bytes can be read (each operand holds at least 8 elements)
    const int64_t a_elems = CONV ? (int64_t)(p.M / (p.conv.OH * p.conv.OW)) * p.conv.H * p.conv.W * p.conv.Cin
                                 : (int64_t)(p.M - 1) * p.lda + p.K;
    const int64_t b_elems = TRANS_B ? (int64_t)(p.N - 1) * p.ldb + p.K : (int64_t)(p.K - 1) * p.ldb + p.N;
    const char* a_last16 = Abase + a_elems * 2 - 16;
    const char* b_last16 = Bbase + b_elems * 2 - 16;

    // ---- A (k-major source): piece = (row, chunk of 8 k); four neighbouring threads cover a row of the k-tile.
    // The thread's two pieces differ in the row only (+64).
    const int a_chunk = t & 3;
    int a_row[PIECES];
    bool a_ok[PIECES];
    const char* a_cur[PIECES];       // dense: address of the piece in the next k-tile to fetch; conv: the pixel's image
    int a_ih0[PIECES], a_iw0[PIECES];
    // conv: (channel, tap) of the thread's pieces in the next k-tile to fetch
    int a_c = 0, a_tap = 0;
    if (CONV) {
        const int k = a_chunk * 8;                    // the pieces' place on the padded K axis in k-tile 0
        a_tap = k / Cp;
        a_c = k - a_tap * Cp;
    }
    // one k-tile further on the padded K axis: adv_tap taps and adv_c channels, with at most one carry
    const int adv_tap = CONV ? GBK / Cp : 0, adv_c = CONV ? GBK - adv_tap * Cp : 0;
    // tap / KW by multiplication (exact for tap < 2^20 / KW)
    const unsigned kw_magic = CONV ? (1u << 20) / (unsigned)p.conv.KW + 1u : 0u;
    const char* zero_piece = (const char*)&kZeroPiece;
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
        a_row[i] = (t >> 2) + (NT / 4) * i;
        const int gm = m0 + a_row[i];
        a_ok[i] = gm < p.M;
        const int gmc = a_ok[i] ? gm : p.M - 1;       // rows beyond M read a row that exists
        if (CONV) {
            const int pix = p.conv.OH * p.conv.OW;
            const int n = gmc / pix, rem = gmc - n * pix;
            const int oh = rem / p.conv.OW, ow = rem - oh * p.conv.OW;
            a_ih0[i] = oh * p.conv.stride_h - p.conv.pad_h;
            a_iw0[i] = ow * p.conv.stride_w - p.conv.pad_w;
            a_cur[i] = Abase + (int64_t)n * p.conv.H * p.conv.W * p.conv.Cin * 2;
        } else {
            a_cur[i] = Abase + ((int64_t)gmc * p.lda + a_chunk * 8) * 2;
        }
    }
    // ---- B: k-major source (trans_b): pieces like A's.  n-major source (row-major B, the weights of a
    // convolution): a piece is eight neighbouring n of one k-row: b_row = k-row in the tile, b_chunk = which
    // eight n; the thread's two pieces differ in the k-row only (+16).
    const int b_chunk = TRANS_B ? (t & 3) : (t & 15);
    int b_row[PIECES];
    bool b_ok[PIECES];
    const char* b_cur[PIECES];       // address of the piece in the next k-tile to fetch (conv: of its first n in row 0)
    int b_c[PIECES], b_tap[PIECES];  // conv: (channel, tap) of the piece's k-row in the next k-tile to fetch
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
        if (TRANS_B) {
            b_row[i] = (t >> 2) + (NT / 4) * i;
            b_ok[i] = n0 + b_row[i] < p.N;
            b_cur[i] = Bbase + ((int64_t)(b_ok[i] ? n0 + b_row[i] : p.N - 1) * p.ldb + b_chunk * 8) * 2;
        } else {
            b_row[i] = (t >> 4) + (NT / 16) * i;
            b_ok[i] = n0 + b_chunk * 8 < p.N;
            // (a piece beyond N reads column N - 1 onwards: it stays inside B wherever the careful path is not taken)
            b_cur[i] = Bbase + (int64_t)(b_ok[i] ? n0 + b_chunk * 8 : p.N - 1) * 2;
            if (CONV) { b_tap[i] = b_row[i] / Cp; b_c[i] = b_row[i] - b_tap[i] * Cp; }
            else b_cur[i] += (int64_t)b_row[i] * p.ldb * 2;
        }
    }
    const int64_t b_step = TRANS_B ? GBK * 2 : (int64_t)GBK * p.ldb * 2;     // dense: B's advance per k-tile

    const int KT = (Kloop + GBK - 1) / GBK;
    // k-tiles from kt_careful on are fetched by the careful path (it keeps every load inside its operand and
    // works out what to keep of each piece); before it no piece can run over the end of an operand:
    //  - dense: every piece of a k-tile before the last lies inside its row (k-major) or in a k-row that has
    //    a successor (n-major; the over-read of a piece that straddles N needs ldb >= 8 to stay in it);
    //  - conv: the same for the weights; the piece at the end of a tap of an image whose channel count is not a
    //    multiple of 8 is read as the tap's LAST eight channels and shifted down afterwards, so it never
    //    leaves its pixel (needs Cin >= 8).
    int kt_careful = KT - 1;
    if (!TRANS_B && p.ldb < 8) kt_careful = 0;
    if (CONV && p.conv.Cin < 8) kt_careful = 0;

    // the pieces of NPF k-tiles are in flight to registers at any time: a workgroup is often alone on its
    // compute unit (these are the odd, small problems), so the memory latency is covered by depth
    constexpr int NPF = 3;
    int4v avs[NPF][PIECES], bvs[NPF][PIECES];
    int metas[NPF];                  // one byte per piece: A's, then B's

    // fetch the pieces of k-tile kt into register set S (loads are issued here and waited for at the first
    // use); called for kt = 0, 1, 2, ... in order, also for up to NPF k-tiles beyond the last (those pieces
    // are cleared).  No load sits under a branch.
    auto gather = [&](int kt, auto set_tag, auto careful_tag) __attribute__((always_inline)) {
        constexpr int S = decltype(set_tag)::value;
        constexpr bool CAREFUL = decltype(careful_tag)::value != 0;
        const int k0 = kt * GBK;
        int meta = 0;
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const char* want;
            bool ok = true;
            int cnt = 8;
            if (CONV) {
                const int kh = (int)(((unsigned)a_tap * kw_magic) >> 20), kw = a_tap - kh * p.conv.KW;
                const int ih = a_ih0[i] + kh * p.conv.dil_h, iw = a_iw0[i] + kw * p.conv.dil_w;
                ok = a_ok[i] && a_tap < taps && (unsigned)ih < (unsigned)p.conv.H && (unsigned)iw < (unsigned)p.conv.W;
                want = a_cur[i] + (unsigned)(((ih * p.conv.W + iw) * p.conv.Cin + a_c) * 2);
                cnt = min(8, p.conv.Cin - a_c);
                if (!CAREFUL) {
                    // a piece in the padding is read from the zero piece and kept whole; a piece at the end of a
                    // tap is read Cp - Cin channels earlier and marked to be shifted down by as many
                    const int back = cnt < 8 ? Cp - p.conv.Cin : 0;
                    want = ok ? want - 2 * back : zero_piece;
                    cnt = ok ? (8 | (back << 4)) : 8;
                    ok = true;
                } else if (!ok) {
                    want = a_cur[i];
                }
            } else {
                want = a_cur[i];
                a_cur[i] += GBK * 2;
                if (CAREFUL) { ok = a_ok[i]; cnt = min(max(p.K - (k0 + a_chunk * 8), 0), 8); }
            }
            PieceSrc s;
            if (CAREFUL) s = piece_src(want, a_last16, ok, cnt);
            else { s.ptr = want; s.meta = ok ? cnt : 0; }
            avs[S][i] = ld_vec16(s.ptr);
            meta |= s.meta << (8 * i);
        }
        if (CONV) {                                   // advance the pieces' place by one k-tile
            a_c += adv_c; a_tap += adv_tap;
            if (a_c >= Cp) { a_c -= Cp; ++a_tap; }
        }
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const char* want;
            bool ok = true;
            int cnt = 8;
            if (CONV) {
                ok = b_tap[i] < taps && b_c[i] < p.conv.Cin;      // a weight row that exists
                const int row = ok ? b_tap[i] * p.conv.Cin + b_c[i] : 0;
                want = b_cur[i] + (int64_t)row * p.ldb * 2;
                if (!CAREFUL) { want = ok ? want : zero_piece; ok = true; }
                else ok = ok && b_ok[i];
                int c = b_c[i] + adv_c, tap = b_tap[i] + adv_tap;
                if (c >= Cp) { c -= Cp; ++tap; }
                b_c[i] = c; b_tap[i] = tap;
            } else {
                want = b_cur[i];
                b_cur[i] += b_step;
                if (CAREFUL) {
                    ok = b_ok[i];
                    if (TRANS_B) cnt = min(max(p.K - (k0 + b_chunk * 8), 0), 8);
                    else ok = ok && k0 + b_row[i] < p.K;
                }
            }
            PieceSrc s;
            if (CAREFUL) s = piece_src(want, b_last16, ok, cnt);
            else { s.ptr = want; s.meta = ok ? cnt : 0; }
            bvs[S][i] = ld_vec16(s.ptr);
            meta |= s.meta << (8 * (PIECES + i));
        }
        metas[S] = meta;
    };
    auto stash = [&](int stage, auto set_tag) __attribute__((always_inline)) {
        constexpr int S = decltype(set_tag)::value;
        char* sa = lds + stage * G_STAGE;
        char* sb = sa + G_TILE_BYTES;
        int4v va[PIECES], vb[PIECES];
#pragma unroll
        for (int i = 0; i < PIECES; ++i) { va[i] = avs[S][i]; vb[i] = bvs[S][i]; }
        if (metas[S] != kAllPlain) {                  // rare: one branch for the thread's four pieces
#pragma unroll
            for (int i = 0; i < PIECES; ++i) {
                va[i] = piece_fix(va[i], (metas[S] >> (8 * i)) & 255);
                vb[i] = piece_fix(vb[i], (metas[S] >> (8 * (PIECES + i))) & 255);
            }
        }
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            *(int4v*)(sa + kmajor_offset<GBK, true>(a_row[i], a_chunk)) = va[i];
            if (TRANS_B) *(int4v*)(sb + kmajor_offset<GBK, true>(b_row[i], b_chunk)) = vb[i];
            else *(int4v*)(sb + nmajor_offset<GBN>(b_row[i], b_chunk * 16)) = vb[i];
        }
    };

    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.0f;

    const int f_row = lane & 15, f_kc = lane >> 4;
    // transposing read of the n-major B tile: 16-lane block q covers k rows 8q .. 8q+3 (second read: +4);
    // lane -> row (lane % 16) / 4, n piece lane % 4
    const int t16_k = ((lane & 15) >> 2) + ((lane >> 4) << 3);
    const int t16_nbyte = (lane & 3) * 8;
    // k-tile kt (its pieces were gathered into set S): multiply it from LDS stage kt % 2, move k-tile kt+1
    // (set S+1) into the other stage, which was last read before the previous barrier, and start fetching
    // k-tile kt+3 into set S, which has just been emptied
    auto step = [&](int kt, auto set_tag, auto careful_tag) __attribute__((always_inline)) {
        constexpr int S = decltype(set_tag)::value;
        const char* sa = lds + (kt & 1) * G_STAGE;
        const char* sb = sa + G_TILE_BYTES;
        short8v af[FM], bf[FN];
#pragma unroll
        for (int i = 0; i < FM; ++i)
            af[i] = *(const short8v*)(sa + kmajor_offset<GBK, true>(wm * WTM + i * 16 + f_row, f_kc));
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            if (TRANS_B) {
                bf[j] = *(const short8v*)(sb + kmajor_offset<GBK, true>(wn * WTN + j * 16 + f_row, f_kc));
            } else {
                const char* r0 = sb + nmajor_offset<GBN>(t16_k, (wn * WTN + j * 16) * 2 + t16_nbyte);
                short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PBK_LDS_PTR(short4v, r0));
                short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PBK_LDS_PTR(short4v, r0 + 4 * (GBN * 2)));
                bf[j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        }
        gather(kt + NPF, set_tag, careful_tag);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) acc[i][j] = MfmaOp16<T>::run(bf[j], af[i], acc[i][j]);
        stash((kt + 1) & 1, IntTag<(S + 1) % NPF>{});
        __syncthreads();
    };
    int kt = 0;
    if (kt_careful >= NPF) {
        gather(0, IntTag<0>{}, IntTag<0>{});
        gather(1, IntTag<1>{}, IntTag<0>{});
        gather(2, IntTag<2>{}, IntTag<0>{});
    } else {
        gather(0, IntTag<0>{}, IntTag<1>{});
        gather(1, IntTag<1>{}, IntTag<1>{});
        gather(2, IntTag<2>{}, IntTag<1>{});
        kt_careful = 0;
    }
    stash(0, IntTag<0>{});
    __syncthreads();
    // steps whose fetches (k-tiles kt + 3 .. kt + 5) all come before the careful ones
    for (; kt + 2 * NPF - 1 < kt_careful; kt += NPF) {
        step(kt, IntTag<0>{}, IntTag<0>{});
        step(kt + 1, IntTag<1>{}, IntTag<0>{});
        step(kt + 2, IntTag<2>{}, IntTag<0>{});
    }
    for (; kt < KT; kt += NPF) {
        step(kt, IntTag<0>{}, IntTag<1>{});
        if (kt + 1 >= KT) break;
        step(kt + 1, IntTag<1>{}, IntTag<1>{});
        if (kt + 2 >= KT) break;
        step(kt + 2, IntTag<2>{}, IntTag<1>{});
    }

    const int act = (p.epi == EPI_RELU || p.epi == EPI_BIAS_RELU) ? 1
                  : (p.epi == EPI_GELU_TANH || p.epi == EPI_BIAS_GELU_TANH) ? 2 : 0;
    char* wlds = lds + wave * ((2 * G_STAGE) / (GWM * GWN));
    EpiCtx<T, f32x4, FM, FN, WTM, WTN, (2 * G_STAGE) / (GWM * GWN)> ctx{p, acc, wlds, m0 + wm * WTM, n0 + wn * WTN, lane,
                                                                      (int64_t)b * p.stride_c};
    if (p.out_dtype == DT_F32) {
        if (act == 0) ctx.template run<0, true>(); else if (act == 1) ctx.template run<1, true>();
        else ctx.template run<2, true>();
    } else {
        if (act == 0) ctx.template run<0, false>(); else if (act == 1) ctx.template run<1, false>();
        else ctx.template run<2, false>();
    }
}

template <typename T, int MODE>
hipError_t launch_gather_mode(const Problem& p, hipStream_t stream) {
    auto kern = gemm_mfma_gather_kernel<T, MODE>;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    DeviceShape ds;
    e = device_shape(dev, &ds);
    if (e != hipSuccess) return e;
    TileMap tm;
    tm.tiles_m = (p.M + GBM - 1) / GBM;
    tm.tiles_n = (p.N + GBN - 1) / GBN;
    tm.tiles_per_batch = tm.tiles_m * tm.tiles_n;
    const long long total = (long long)tm.tiles_per_batch * p.batch;
    if (total <= 0 || total > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    tm.total = (int)total;
    tm.group_m = 8;
    tm.xcds = ds.xcds;
    Problem pa = p;
    void* args[] = {&pa, &tm};
    return hipLaunchKernel((const void*)kern, dim3((unsigned)total), dim3(GWM * GWN * 64), args, 2 * G_STAGE, stream);
}

template <typename T>
hipError_t launch_gather_type(const Problem& p, hipStream_t stream) {
    if (p.is_conv) return launch_gather_mode<T, MODE_CONV>(p, stream);
    if (p.trans_b) return launch_gather_mode<T, MODE_TRANS_B>(p, stream);
    return launch_gather_mode<T, MODE_DENSE>(p, stream);
}

}  // namespace

// 16-bit operands of any alignment and any K, N, leading dimensions and channel count; convolutions that
// are not transposed.  Each operand must hold the 16 bytes of one piece, and one image must stay below
// 2 GiB (32-bit offsets inside an image).
bool mfma_gather_supported(const Problem& p) {
    if (p.in_dtype != DT_BF16 && p.in_dtype != DT_F16) return false;
    if (p.K < 1 || p.M < 1 || p.N < 1) return false;
    int64_t a_elems, b_elems;
    if (p.is_conv) {
        if (p.conv.transposed) return false;
        // tap -> (kh, kw) by multiplication is exact below 2^20 / KW taps
        if ((int64_t)p.conv.KH * p.conv.KW + 16 >= ((int64_t)1 << 20) / p.conv.KW) return false;
        const int64_t img = (int64_t)p.conv.H * p.conv.W * p.conv.Cin;
        if (img * 2 + 64 >= ((int64_t)1 << 31)) return false;
        a_elems = (int64_t)(p.M / (p.conv.OH * p.conv.OW)) * img;
        // the loop runs over taps * ceil8(Cin)
        if ((int64_t)p.conv.KH * p.conv.KW * ((p.conv.Cin + 7) & ~7) + 4 * GBK >= ((int64_t)1 << 31)) return false;
    } else {
        a_elems = (int64_t)(p.M - 1) * p.lda + p.K;
    }
    b_elems = p.trans_b ? (int64_t)(p.N - 1) * p.ldb + p.K : (int64_t)(p.K - 1) * p.ldb + p.N;
    if ((int64_t)p.K + 4 * GBK >= ((int64_t)1 << 30)) return false;
    return a_elems >= 8 && b_elems >= 8;
}

hipError_t launch_mfma_gather(const Problem& p, hipStream_t stream, const char** name) {
    *name = "mfma16_gather_128x128x32_w2x2";
    return p.in_dtype == DT_BF16 ? launch_gather_type<bf16_t>(p, stream) : launch_gather_type<f16_t>(p, stream);
}

}  // namespace pbk
