// C ABI of libpbk: argument validation and dispatch.  No allocation, no
// synchronisation; every call enqueues at most one kernel on the caller's stream.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <climits>
#include "../../include/pbk.h"
#include "pbk_problem.h"

namespace {

thread_local const char* g_last_kernel = "";
// residual operand of the call being assembled on this thread (set by the *_residual entry points)
thread_local const void* g_residual = nullptr;
thread_local int64_t g_ldr = 0;
thread_local float g_beta = 0.0f;

int64_t elem_size(int dt) {
    return dt == pbk::DT_F32 ? 4 : (dt == pbk::DT_BF16 || dt == pbk::DT_F16) ? 2 : 1;   // FP8 and int8: 1
}

bool is_fp8(int dt) { return dt == PBK_FP8_E4M3 || dt == PBK_FP8_E5M2; }
bool valid_in_dtype(int dt) { return dt >= PBK_F32 && dt <= PBK_FP8_E5M2; }   // int8 has its own entry points
bool valid_out_dtype(int dt) { return dt == PBK_F32 || dt == PBK_BF16 || dt == PBK_F16; }

bool aligned(const void* p, int64_t a) { return (reinterpret_cast<uintptr_t>(p) % (uintptr_t)a) == 0; }

// Kernel choice overrides (benchmarking and test aid).  A choice is "generic" (the fallback
// kernel), "mfma" (the matrix-unit path, automatic tile configuration), "mfma:<id>" (one tile
// configuration) or "gather" (the matrix-unit kernel that stages through registers).  The environment variables PBK_FORCE_KERNEL and PBK_GROUP_M are read ONCE,
// at the first call of the process; pbk_force_kernel() overrides the former per thread.
// force: 0 automatic, 1 generic, 2 mfma, 3 the gathering mfma kernel, 4 the small fp32 kernel, 5 "bstat" (the
// B-stationary kernel for short contractions); cfg: -1 or id
struct Choice { int force; int cfg; };

bool parse_choice(const char* e, Choice* c) {
    c->force = 0; c->cfg = -1;
    if (!e || !*e) return true;
    if (!std::strcmp(e, "generic")) { c->force = 1; return true; }
    if (!std::strcmp(e, "mfma")) { c->force = 2; return true; }
    if (!std::strcmp(e, "gather")) { c->force = 3; return true; }
    if (!std::strcmp(e, "small")) { c->force = 4; return true; }
    if (!std::strcmp(e, "bstat")) { c->force = 5; return true; }
    if (!std::strncmp(e, "mfma:", 5) && e[5] >= '0' && e[5] <= '9') { c->force = 2; c->cfg = std::atoi(e + 5); return true; }
    return false;
}

struct EnvOverrides { Choice choice; int group_m; };
const EnvOverrides& env_overrides() {
    static const EnvOverrides o = [] {
        EnvOverrides r{};
        if (!parse_choice(std::getenv("PBK_FORCE_KERNEL"), &r.choice)) r.choice = Choice{0, -1};
        r.group_m = 0;
        if (const char* e = std::getenv("PBK_GROUP_M")) { int g = std::atoi(e); if (g > 0) r.group_m = g; }
        return r;
    }();
    return o;
}

thread_local bool g_choice_set = false;      // pbk_force_kernel() was called on this thread
thread_local Choice g_choice = {0, -1};

int forced_choice(int* cfg) {
    const Choice& c = g_choice_set ? g_choice : env_overrides().choice;
    *cfg = c.cfg;
    return c.force;
}

pbk_status check_common(int in_dtype, int out_dtype, int epi, const float* bias) {
    if (!valid_in_dtype(in_dtype) || !valid_out_dtype(out_dtype)) return PBK_ERR_DTYPE;
    if (out_dtype != PBK_F32 && out_dtype != in_dtype && !is_fp8(in_dtype)) return PBK_ERR_DTYPE;
    if (epi < PBK_EPI_NONE || epi > PBK_EPI_GELU_TANH) return PBK_ERR_EPILOGUE;
    if (pbk::epi_has_bias(epi) && !bias) return PBK_ERR_EPILOGUE;
    if (bias && !aligned(bias, 4)) return PBK_ERR_ALIGN;
    return PBK_OK;
}

pbk_status dispatch(const pbk::Problem& p_in, hipStream_t stream) {
    pbk::Problem p = p_in;
    if (g_residual) { p.R = g_residual; p.ldr = g_ldr; p.beta = g_beta; }
    int cfg = -1;
    int force = forced_choice(&cfg);
    const char* name = "";
    hipError_t e;
    const bool can_mfma = pbk::mfma_supported(p);
    // operands the direct-to-LDS kernel cannot take (ragged K, N, leading dimensions, channel counts,
    // unaligned bases) still run on the matrix units, staged through registers, when there is enough work
    const bool can_gather = pbk::mfma_gather_supported(p);
    const bool want_gather = !can_mfma && can_gather && (long long)p.M * p.N >= 4096 && p.K >= 16;
    // fp32 problems of a few hundred 16 x 16 tiles: one wave per tile
    const bool can_small = pbk::small_f32_supported(p);
    // short contractions over many rows: the B-stationary kernel
    const bool can_bstat = pbk::mfma_bstat_supported(p);
    if ((force == 2 && !can_mfma && !can_gather) || (force == 3 && !can_gather) || (force == 4 && !can_small) ||
        (force == 5 && !can_bstat))
        return PBK_ERR_UNSUPPORTED;
    if (force == 5 || (force == 0 && can_bstat && pbk::mfma_bstat_preferred(p)))
        e = pbk::launch_mfma_bstat(p, stream, &name);
    else if (force == 4 || (force == 0 && can_small && pbk::small_f32_preferred(p) && !(can_mfma && pbk::mfma_preferred(p))))
        e = pbk::launch_small_f32(p, stream, &name);
    else if (can_mfma && force != 1 && force != 3 && (force == 2 || pbk::mfma_preferred(p)))
        e = pbk::launch_mfma(p, stream, cfg, &name);
    else if (force == 3 || (force == 2 && !can_mfma) || (force == 0 && want_gather))
        e = pbk::launch_mfma_gather(p, stream, &name);
    else
        e = pbk::launch_generic(p, stream, &name);
    if (e != hipSuccess) {
        std::fprintf(stderr, "libpbk: launch of %s failed: %s\n", name, hipGetErrorString(e));
        return PBK_ERR_HIP;
    }
    g_last_kernel = name;
    return PBK_OK;
}

// Quantised epilogue parameters of the int8 entry points.
pbk_status check_quant(const float* scale, const float* bias, float mid_scale, const float* mul,
                       const float* add, float out_scale, int out_dtype) {
    if (out_dtype != PBK_INT8 && out_dtype != PBK_F32) return PBK_ERR_DTYPE;
    if (!scale) return PBK_ERR_EPILOGUE;
    if (!(mid_scale >= 0.0f) || (out_dtype == PBK_INT8 && !(out_scale > 0.0f))) return PBK_ERR_EPILOGUE;
    if (!aligned(scale, 4) || (bias && !aligned(bias, 4)) || (mul && !aligned(mul, 4)) || (add && !aligned(add, 4)))
        return PBK_ERR_ALIGN;
    return PBK_OK;
}

// Unfolded batch norm of the call being assembled on this thread (set by the *_int8_bn entry points)
thread_local const float* g_bn_mean = nullptr;
thread_local const float* g_bn_var = nullptr;
thread_local float g_bn_eps = 0.0f;

void set_quant(pbk::Problem& p, const float* scale, const float* bias, float mid_scale, const float* mul,
               const float* add, int relu, float out_scale) {
    p.q_mean = g_bn_mean; p.q_var = g_bn_var; p.q_eps = g_bn_eps;
    p.in_dtype = pbk::DT_INT8;
    p.bias = bias;
    p.q_scale = scale; p.q_mul = mul; p.q_add = add;
    p.q_mid = mid_scale; p.q_out = out_scale; p.q_relu = relu ? 1 : 0;
    p.epi = pbk::EPI_NONE; p.alpha = 1.0f;
}

// Shared tail of the convolution entry points.  pad_h / pad_w are the near-side (top, left)
// paddings; OH / OW the output size the caller derived (negative = empty or invalid).
pbk_status conv_common(const void* x, const void* w, void* y, const float* bias,
                       int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                       int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                       int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                       int64_t OH, int64_t OW, int transposed,
                       int in_dtype, int out_dtype, float alpha, int epi, hipStream_t stream,
                       const float* q_scale = nullptr, const float* q_mul = nullptr, const float* q_add = nullptr,
                       float q_mid = 0.0f, float q_out = 0.0f, int q_relu = 0, bool quant = false) {
    // quant: the call comes from the int8 entry point, which has validated its own parameters;
    // from every other entry point PBK_INT8 is not an input type (check_common rejects it)
    if (!quant) {
        pbk_status s = check_common(in_dtype, out_dtype, epi, bias);
        if (s != PBK_OK) return s;
    } else if (in_dtype != PBK_INT8 || !q_scale) {
        return PBK_ERR_DTYPE;
    }
    if (N < 0 || H < 1 || W < 1 || Cin < 1 || Cout < 1 || KH < 1 || KW < 1) return PBK_ERR_SHAPE;
    if (stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0 || dil_h < 1 || dil_w < 1)
        return PBK_ERR_SHAPE;
    const int64_t lim = 1 << 24;   // keeps every 32-bit index computation in range
    if (H > lim || W > lim || Cin > lim || Cout > lim || KH > 4096 || KW > 4096 ||
        stride_h > 4096 || stride_w > 4096 || pad_h > lim || pad_w > lim || dil_h > 4096 || dil_w > 4096)
        return PBK_ERR_SHAPE;
    if (OH < 1 || OW < 1 || OH > (lim << 4) || OW > (lim << 4)) return PBK_ERR_SHAPE;
    if (N == 0) return PBK_OK;
    if (!x || !w || !y) return PBK_ERR_NULL;
    int64_t gm = N * OH * OW, gk = KH * KW * Cin;
    if (gm > INT_MAX || gk > INT_MAX || N * H * W > INT_MAX) return PBK_ERR_SHAPE;
    if (!aligned(x, elem_size(in_dtype)) || !aligned(w, elem_size(in_dtype)) ||
        !aligned(y, elem_size(out_dtype)))
        return PBK_ERR_ALIGN;

    pbk::Problem p{};
    p.A = x; p.B = w; p.C = y; p.bias = bias;
    p.M = (int)gm; p.N = (int)Cout; p.K = (int)gk; p.batch = 1;
    p.lda = gk;            // of the virtual im2col matrix; never dereferenced as such
    p.ldb = Cout; p.ldc = Cout;
    p.in_dtype = in_dtype; p.out_dtype = out_dtype;
    p.trans_b = 0;
    p.is_conv = 1;
    p.epi = epi; p.alpha = alpha;
    p.conv.H = (int)H; p.conv.W = (int)W; p.conv.Cin = (int)Cin;
    p.conv.OH = (int)OH; p.conv.OW = (int)OW;
    p.conv.KH = (int)KH; p.conv.KW = (int)KW;
    p.conv.stride_h = (int)stride_h; p.conv.stride_w = (int)stride_w;
    p.conv.pad_h = (int)pad_h; p.conv.pad_w = (int)pad_w;
    p.conv.dil_h = (int)dil_h; p.conv.dil_w = (int)dil_w;
    p.conv.transposed = transposed;
    // A 1x1 filter at stride 1 without padding IS the matmul [N H W][Cin] x [Cin][Cout] (Sec. 4.5: the virtual
    // matmul's rows are then the pixels themselves): it takes the plain-matrix kernels, which carry no tap
    // arithmetic, and with few input channels the store-bound B-stationary one.
    if (KH == 1 && KW == 1 && stride_h == 1 && stride_w == 1 && pad_h == 0 && pad_w == 0 && !transposed &&
        OH == H && OW == W) {
        p.is_conv = 0;
        p.lda = Cin;
    }
    if (quant) set_quant(p, q_scale, bias, q_mid, q_mul, q_add, q_relu, q_out);
    return dispatch(p, stream);
}

}  // namespace

namespace pbk {
int group_m_override() { return env_overrides().group_m; }
}

extern "C" {

pbk_status pbk_batched_matmul(const void* A, const void* B, void* C, const float* bias,
                              int64_t batch, int64_t M, int64_t N, int64_t K,
                              int64_t lda, int64_t ldb, int64_t ldc,
                              int64_t stride_a, int64_t stride_b, int64_t stride_c,
                              pbk_dtype in_dtype, pbk_dtype out_dtype, int trans_b,
                              float alpha, pbk_epilogue epi, hipStream_t stream) {
    pbk_status s = check_common(in_dtype, out_dtype, epi, bias);
    if (s != PBK_OK) return s;
    if (batch < 0 || M < 0 || N < 0 || K < 0) return PBK_ERR_SHAPE;
    if (M > INT_MAX || N > INT_MAX || K > INT_MAX || batch > INT_MAX) return PBK_ERR_SHAPE;
    if (batch == 0 || M == 0 || N == 0) return PBK_OK;
    if (!C || (K > 0 && (!A || !B))) return PBK_ERR_NULL;
    if (lda < K || ldc < N || ldb < (trans_b ? K : N)) return PBK_ERR_STRIDE;
    if (stride_a < 0 || stride_b < 0 || stride_c < 0) return PBK_ERR_STRIDE;
    if (batch > 1 && stride_c < (M - 1) * ldc + N) return PBK_ERR_STRIDE;
    if (!aligned(A, elem_size(in_dtype)) || !aligned(B, elem_size(in_dtype)) ||
        !aligned(C, elem_size(out_dtype)))
        return PBK_ERR_ALIGN;

    pbk::Problem p{};
    p.A = A; p.B = B; p.C = C; p.bias = bias;
    p.M = (int)M; p.N = (int)N; p.K = (int)K; p.batch = (int)batch;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.stride_a = stride_a; p.stride_b = stride_b; p.stride_c = stride_c;
    p.in_dtype = in_dtype; p.out_dtype = out_dtype;
    p.trans_b = trans_b ? 1 : 0;
    p.is_conv = 0;
    p.epi = epi; p.alpha = alpha;
    return dispatch(p, stream);
}

pbk_status pbk_matmul_residual(const void* A, const void* B, void* C, const float* bias, const void* R,
                               int64_t M, int64_t N, int64_t K,
                               int64_t lda, int64_t ldb, int64_t ldc, int64_t ldr,
                               pbk_dtype in_dtype, pbk_dtype out_dtype, int trans_b,
                               float alpha, float beta, pbk_epilogue epi, hipStream_t stream) {
    if (!R && M > 0 && N > 0) return PBK_ERR_NULL;
    if (ldr < N) return PBK_ERR_STRIDE;
    if (valid_out_dtype(out_dtype) && !aligned(R, elem_size(out_dtype))) return PBK_ERR_ALIGN;
    g_residual = R; g_ldr = ldr; g_beta = beta;
    pbk_status s = pbk_batched_matmul(A, B, C, bias, 1, M, N, K, lda, ldb, ldc, 0, 0, 0,
                                      in_dtype, out_dtype, trans_b, alpha, epi, stream);
    g_residual = nullptr;
    return s;
}

pbk_status pbk_matmul(const void* A, const void* B, void* C, const float* bias,
                      int64_t M, int64_t N, int64_t K,
                      int64_t lda, int64_t ldb, int64_t ldc,
                      pbk_dtype in_dtype, pbk_dtype out_dtype, int trans_b,
                      float alpha, pbk_epilogue epi, hipStream_t stream) {
    return pbk_batched_matmul(A, B, C, bias, 1, M, N, K, lda, ldb, ldc, 0, 0, 0,
                              in_dtype, out_dtype, trans_b, alpha, epi, stream);
}

pbk_status pbk_conv2d_nhwc_pad4(const void* x, const void* w, void* y, const float* bias,
                                int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                int64_t pad_top, int64_t pad_bottom, int64_t pad_left, int64_t pad_right,
                                int64_t dil_h, int64_t dil_w,
                                pbk_dtype in_dtype, pbk_dtype out_dtype,
                                float alpha, pbk_epilogue epi, hipStream_t stream) {
    int64_t OH = -1, OW = -1;
    const int64_t lim = 1 << 24;
    const bool sane = pad_top >= 0 && pad_bottom >= 0 && pad_left >= 0 && pad_right >= 0 &&
                      pad_top <= lim && pad_bottom <= lim && pad_left <= lim && pad_right <= lim &&
                      H >= 1 && W >= 1 && H <= lim && W <= lim && KH >= 1 && KW >= 1 && KH <= 4096 && KW <= 4096 &&
                      stride_h >= 1 && stride_w >= 1 && dil_h >= 1 && dil_w >= 1 && dil_h <= 4096 && dil_w <= 4096;
    if (sane) {
        const int64_t span_h = H + pad_top + pad_bottom - dil_h * (KH - 1) - 1;
        const int64_t span_w = W + pad_left + pad_right - dil_w * (KW - 1) - 1;
        if (span_h >= 0 && span_w >= 0) { OH = span_h / stride_h + 1; OW = span_w / stride_w + 1; }
    }
    return conv_common(x, w, y, bias, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, sane ? pad_top : -1,
                       sane ? pad_left : -1, dil_h, dil_w, OH, OW, 0, in_dtype, out_dtype, alpha, epi, stream);
}

pbk_status pbk_conv2d_nhwc(const void* x, const void* w, void* y, const float* bias,
                           int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                           int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                           int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                           pbk_dtype in_dtype, pbk_dtype out_dtype,
                           float alpha, pbk_epilogue epi, hipStream_t stream) {
    return pbk_conv2d_nhwc_pad4(x, w, y, bias, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w,
                                pad_h, pad_h, pad_w, pad_w, dil_h, dil_w, in_dtype, out_dtype, alpha, epi, stream);
}

pbk_status pbk_conv2d_nhwc_residual(const void* x, const void* w, void* y, const float* bias, const void* r,
                                    int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                    int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                    int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                                    pbk_dtype in_dtype, pbk_dtype out_dtype,
                                    float alpha, float beta, pbk_epilogue epi, hipStream_t stream) {
    if (!r && N > 0) return PBK_ERR_NULL;
    if (valid_out_dtype(out_dtype) && !aligned(r, elem_size(out_dtype))) return PBK_ERR_ALIGN;
    g_residual = r; g_ldr = Cout; g_beta = beta;
    pbk_status s = pbk_conv2d_nhwc(x, w, y, bias, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w,
                                   dil_h, dil_w, in_dtype, out_dtype, alpha, epi, stream);
    g_residual = nullptr;
    return s;
}

pbk_status pbk_conv2d_transpose_nhwc(const void* x, const void* w, void* y, const float* bias,
                                     int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                     int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                     int64_t pad_h, int64_t pad_w, int64_t out_pad_h, int64_t out_pad_w,
                                     int64_t dil_h, int64_t dil_w,
                                     pbk_dtype in_dtype, pbk_dtype out_dtype,
                                     float alpha, pbk_epilogue epi, hipStream_t stream) {
    int64_t OH = -1, OW = -1;
    const int64_t lim = 1 << 24;
    const bool sane = H >= 1 && W >= 1 && H <= lim && W <= lim && KH >= 1 && KW >= 1 && KH <= 4096 && KW <= 4096 &&
                      stride_h >= 1 && stride_w >= 1 && stride_h <= 4096 && stride_w <= 4096 &&
                      dil_h >= 1 && dil_w >= 1 && dil_h <= 4096 && dil_w <= 4096 &&
                      pad_h >= 0 && pad_w >= 0 && pad_h <= lim && pad_w <= lim && out_pad_h >= 0 && out_pad_w >= 0 &&
                      (out_pad_h < stride_h || out_pad_h < dil_h) && (out_pad_w < stride_w || out_pad_w < dil_w);
    if (sane) {
        OH = (H - 1) * stride_h - 2 * pad_h + dil_h * (KH - 1) + out_pad_h + 1;
        OW = (W - 1) * stride_w - 2 * pad_w + dil_w * (KW - 1) + out_pad_w + 1;
        if (OH < 1 || OW < 1) OH = OW = -1;
    }
    return conv_common(x, w, y, bias, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w,
                       dil_h, dil_w, OH, OW, 1, in_dtype, out_dtype, alpha, epi, stream);
}

pbk_status pbk_matmul_int8(const int8_t* A, const int8_t* B, void* C,
                           int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb, int64_t ldc, int trans_b,
                           const float* scale, const float* bias, float mid_scale,
                           const float* mul, const float* add, int relu, float out_scale,
                           pbk_dtype out_dtype, hipStream_t stream) {
    pbk_status s = check_quant(scale, bias, mid_scale, mul, add, out_scale, out_dtype);
    if (s != PBK_OK) return s;
    if (M < 0 || N < 0 || K < 0 || M > INT_MAX || N > INT_MAX) return PBK_ERR_SHAPE;
    if (K > 131071) return PBK_ERR_UNSUPPORTED;       // the sum of K products must fit 32 bits
    if (M == 0 || N == 0) return PBK_OK;
    if (!C || (K > 0 && (!A || !B))) return PBK_ERR_NULL;
    if (lda < K || ldc < N || ldb < (trans_b ? K : N)) return PBK_ERR_STRIDE;
    if (!aligned(C, elem_size(out_dtype))) return PBK_ERR_ALIGN;
    pbk::Problem p{};
    p.A = A; p.B = B; p.C = C;
    p.M = (int)M; p.N = (int)N; p.K = (int)K; p.batch = 1;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.out_dtype = out_dtype;
    p.trans_b = trans_b ? 1 : 0;
    set_quant(p, scale, bias, mid_scale, mul, add, relu, out_scale);
    return dispatch(p, stream);
}

pbk_status pbk_conv2d_nhwc_int8(const int8_t* x, const int8_t* w, void* y,
                                int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                                const float* scale, const float* bias, float mid_scale,
                                const float* mul, const float* add, int relu, float out_scale,
                                pbk_dtype out_dtype, hipStream_t stream) {
    pbk_status s = check_quant(scale, bias, mid_scale, mul, add, out_scale, out_dtype);
    if (s != PBK_OK) return s;
    if (KH >= 1 && KW >= 1 && Cin >= 1 && KH <= 4096 && KW <= 4096 && Cin <= (1 << 24) && KH * KW * Cin > 131071)
        return PBK_ERR_UNSUPPORTED;
    int64_t OH = -1, OW = -1;
    if (H >= 1 && W >= 1 && KH >= 1 && KW >= 1 && stride_h >= 1 && stride_w >= 1 && pad_h >= 0 && pad_w >= 0 &&
        dil_h >= 1 && dil_w >= 1 && H <= (1 << 24) && W <= (1 << 24) && pad_h <= (1 << 24) && pad_w <= (1 << 24) &&
        KH <= 4096 && KW <= 4096 && dil_h <= 4096 && dil_w <= 4096) {
        const int64_t span_h = H + 2 * pad_h - dil_h * (KH - 1) - 1, span_w = W + 2 * pad_w - dil_w * (KW - 1) - 1;
        if (span_h >= 0 && span_w >= 0) { OH = span_h / stride_h + 1; OW = span_w / stride_w + 1; }
    }
    return conv_common(x, w, y, bias, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w,
                       OH, OW, 0, PBK_INT8, out_dtype, 1.0f, PBK_EPI_NONE, stream, scale, mul, add, mid_scale,
                       out_scale, relu, true);
}

pbk_status pbk_matmul_int8_bn(const int8_t* A, const int8_t* B, void* C,
                              int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb, int64_t ldc, int trans_b,
                              const float* scale, const float* bias, float mid_scale,
                              const float* mean, const float* var, float eps, const float* gamma, const float* beta,
                              int relu, float out_scale, pbk_dtype out_dtype, hipStream_t stream) {
    if (!mean || !var || !gamma || !beta) return PBK_ERR_EPILOGUE;
    if (!aligned(mean, 4) || !aligned(var, 4)) return PBK_ERR_ALIGN;
    g_bn_mean = mean; g_bn_var = var; g_bn_eps = eps;
    pbk_status s = pbk_matmul_int8(A, B, C, M, N, K, lda, ldb, ldc, trans_b, scale, bias, mid_scale, gamma, beta, relu,
                                   out_scale, out_dtype, stream);
    g_bn_mean = nullptr; g_bn_var = nullptr;
    return s;
}

pbk_status pbk_conv2d_nhwc_int8_bn(const int8_t* x, const int8_t* w, void* y,
                                   int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                   int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                   int64_t pad_h, int64_t pad_w, int64_t dil_h, int64_t dil_w,
                                   const float* scale, const float* bias, float mid_scale,
                                   const float* mean, const float* var, float eps, const float* gamma, const float* beta,
                                   int relu, float out_scale, pbk_dtype out_dtype, hipStream_t stream) {
    if (!mean || !var || !gamma || !beta) return PBK_ERR_EPILOGUE;
    if (!aligned(mean, 4) || !aligned(var, 4)) return PBK_ERR_ALIGN;
    g_bn_mean = mean; g_bn_var = var; g_bn_eps = eps;
    pbk_status s = pbk_conv2d_nhwc_int8(x, w, y, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w,
                                        scale, bias, mid_scale, gamma, beta, relu, out_scale, out_dtype, stream);
    g_bn_mean = nullptr; g_bn_var = nullptr;
    return s;
}

static pbk_status attention_common(const void* Q, const void* K, const void* V, const float* bias, void* O,
                                   int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                                   int64_t ldq, int64_t ldk, int64_t ldv, int64_t ldo,
                                   int64_t stride_q, int64_t stride_k, int64_t stride_v, int64_t stride_o,
                                   int64_t ld_bias, int64_t stride_bias,
                                   pbk_dtype dtype, float alpha, int causal, hipStream_t stream) {
    if (dtype != PBK_F32 && dtype != PBK_BF16 && dtype != PBK_F16) return PBK_ERR_DTYPE;
    if (batch < 0 || Nq < 0 || Nk < 0 || D < 1) return PBK_ERR_SHAPE;
    if (batch > INT_MAX || Nq > INT_MAX || Nk > INT_MAX || D > INT_MAX) return PBK_ERR_SHAPE;
    if (batch == 0 || Nq == 0) return PBK_OK;
    if (Nk == 0) return PBK_ERR_SHAPE;                 // a softmax over no keys
    if (batch * Nq > INT_MAX) return PBK_ERR_SHAPE;
    if (!Q || !K || !V || !O) return PBK_ERR_NULL;
    if (ldq < D || ldk < D || ldv < D || ldo < D) return PBK_ERR_STRIDE;
    if (stride_q < 0 || stride_k < 0 || stride_v < 0 || stride_o < 0) return PBK_ERR_STRIDE;
    if (batch > 1 && stride_o < (Nq - 1) * ldo + D) return PBK_ERR_STRIDE;
    if (bias && (ld_bias < Nk || stride_bias < 0)) return PBK_ERR_STRIDE;
    const int64_t esz = elem_size(dtype);
    if (!aligned(Q, esz) || !aligned(K, esz) || !aligned(V, esz) || !aligned(O, esz)) return PBK_ERR_ALIGN;
    if (bias && !aligned(bias, 4)) return PBK_ERR_ALIGN;

    pbk::AttnProblem p{};
    p.Q = Q; p.K = K; p.V = V; p.bias = bias; p.O = O;
    p.batch = (int)batch; p.Nq = (int)Nq; p.Nk = (int)Nk; p.D = (int)D;
    p.ldq = ldq; p.ldk = ldk; p.ldv = ldv; p.ldo = ldo;
    p.stride_q = stride_q; p.stride_k = stride_k; p.stride_v = stride_v; p.stride_o = stride_o;
    p.ld_bias = bias ? ld_bias : 0; p.stride_bias = bias ? stride_bias : 0;
    p.dtype = dtype; p.alpha = alpha; p.causal = causal;

    int cfg = -1;
    const int force = forced_choice(&cfg);
    const bool can_mfma = pbk::attention_mfma_supported(p);
    if (force == 2 && !can_mfma) return PBK_ERR_UNSUPPORTED;
    const bool use_mfma = can_mfma && force != 1;
    if (!use_mfma && D > 512) return PBK_ERR_UNSUPPORTED;
    const char* name = "";
    hipError_t e = use_mfma ? pbk::launch_attention_mfma(p, stream, &name)
                            : pbk::launch_attention_generic(p, stream, &name);
    if (e != hipSuccess) {
        std::fprintf(stderr, "libpbk: launch of %s failed: %s\n", name, hipGetErrorString(e));
        return PBK_ERR_HIP;
    }
    g_last_kernel = name;
    return PBK_OK;
}

pbk_status pbk_attention(const void* Q, const void* K, const void* V, const float* bias, void* O,
                         int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                         int64_t ldq, int64_t ldk, int64_t ldv, int64_t ldo,
                         int64_t stride_q, int64_t stride_k, int64_t stride_v, int64_t stride_o,
                         int64_t ld_bias, int64_t stride_bias,
                         pbk_dtype dtype, float alpha, hipStream_t stream) {
    return attention_common(Q, K, V, bias, O, batch, Nq, Nk, D, ldq, ldk, ldv, ldo, stride_q, stride_k, stride_v, stride_o,
                            ld_bias, stride_bias, dtype, alpha, 0, stream);
}

pbk_status pbk_attention_causal(const void* Q, const void* K, const void* V, void* O,
                                int64_t batch, int64_t Nq, int64_t Nk, int64_t D,
                                int64_t ldq, int64_t ldk, int64_t ldv, int64_t ldo,
                                int64_t stride_q, int64_t stride_k, int64_t stride_v, int64_t stride_o,
                                pbk_dtype dtype, float alpha, hipStream_t stream) {
    return attention_common(Q, K, V, nullptr, O, batch, Nq, Nk, D, ldq, ldk, ldv, ldo, stride_q, stride_k, stride_v, stride_o,
                            0, 0, dtype, alpha, 1, stream);
}

const char* pbk_status_string(pbk_status s) {
    switch (s) {
    case PBK_OK: return "ok";
    case PBK_ERR_NULL: return "required pointer is NULL";
    case PBK_ERR_SHAPE: return "invalid shape";
    case PBK_ERR_STRIDE: return "leading dimension or batch stride too small";
    case PBK_ERR_ALIGN: return "pointer not aligned to its element size";
    case PBK_ERR_DTYPE: return "unsupported dtype combination";
    case PBK_ERR_EPILOGUE: return "unknown epilogue or missing bias";
    case PBK_ERR_UNSUPPORTED: return "request not supported by this build";
    case PBK_ERR_HIP: return "HIP runtime error at launch";
    default: return "unknown status";
    }
}

int pbk_version(void) { return 100; }

const char* pbk_last_kernel(void) { return g_last_kernel; }

pbk_status pbk_force_kernel(const char* choice) {
    Choice c;
    if (!parse_choice(choice, &c)) return PBK_ERR_UNSUPPORTED;
    g_choice_set = choice != nullptr && *choice != 0;
    g_choice = c;
    return PBK_OK;
}

}  // extern "C"
