"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects invalid arguments before any
launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pbk():
    import paper_2603_06731_amd as m
    if not os.path.exists(m.lib_path()):
        from paper_2603_06731_amd import build
        build.build()
    return m


def declared_symbols():
    src = open(os.path.join(ROOT, "include", "pbk.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(pbk_[a-z0-9_]+)\s*\(", src)))


def test_header_symbols_are_exported(pbk):
    names = declared_symbols()
    assert set(names) == set(pbk.EXPORTED_SYMBOLS)
    L = ctypes.CDLL(pbk.lib_path())
    for n in names:
        assert hasattr(L, n), n


def test_version_and_status_strings(pbk):
    assert pbk.pbk_version() >= 100
    seen = {pbk.pbk_status_string(s) for s in range(9)}
    assert len(seen) == 9 and pbk.pbk_status_string(0) == "ok"
    assert pbk.pbk_status_string(99) == "unknown status"


def test_matmul_argument_errors(pbk):
    F32, BF16, F16 = 0, 1, 2
    P = 0x1000           # fake, aligned, never dereferenced: every call below fails validation
    mm = pbk.pbk_matmul
    assert mm(P, P, P, None, -1, 2, 2, 2, 2, 2, F32, F32, 0, 1.0, 0) == 2          # shape
    assert mm(P, P, P, None, 2, 2, 2, 1, 2, 2, F32, F32, 0, 1.0, 0) == 3           # lda < K
    assert mm(P, P, P, None, 2, 4, 2, 2, 2, 4, F32, F32, 0, 1.0, 0) == 3           # ldb < N
    assert mm(P, P, P, None, 2, 4, 3, 3, 2, 4, F32, F32, 1, 1.0, 0) == 3           # ldb < K (trans)
    assert mm(P, P, P, None, 2, 4, 2, 2, 4, 3, F32, F32, 0, 1.0, 0) == 3           # ldc < N
    assert mm(None, P, P, None, 2, 2, 2, 2, 2, 2, F32, F32, 0, 1.0, 0) == 1        # null A
    assert mm(P, P, None, None, 2, 2, 2, 2, 2, 2, F32, F32, 0, 1.0, 0) == 1        # null C
    assert mm(P, P, P, None, 2, 2, 2, 2, 2, 2, 7, F32, 0, 1.0, 0) == 5             # dtype
    assert mm(P, P, P, None, 2, 2, 2, 2, 2, 2, BF16, F16, 0, 1.0, 0) == 5          # in/out pair
    assert mm(P, P, P, None, 2, 2, 2, 2, 2, 2, F32, BF16, 0, 1.0, 0) == 5
    assert mm(P, P, P, None, 2, 2, 2, 2, 2, 2, F32, 3, 0, 1.0, 0) == 5             # FP8 is never an output type
    assert mm(P, P, P, None, 2, 2, 2, 2, 2, 2, 3, 4, 0, 1.0, 0) == 5
    assert mm(P, P, P, None, 2, 2, 2, 2, 2, 2, 5, F32, 0, 1.0, 0) == 5             # unknown input type
    assert mm(P, P, P, None, 0, 2, 2, 2, 2, 2, 3, BF16, 0, 1.0, 0) == 0            # FP8 in, bf16 out: valid pair
    assert mm(P, P, P, None, 2, 2, 2, 2, 2, 2, F32, F32, 0, 1.0, 9) == 6           # epilogue
    assert mm(P, P, P, None, 2, 2, 2, 2, 2, 2, F32, F32, 0, 1.0, 3) == 6           # bias missing
    assert mm(P + 2, P, P, None, 2, 2, 2, 2, 2, 2, F32, F32, 0, 1.0, 0) == 4       # alignment
    assert mm(P, P, P + 1, None, 2, 2, 2, 2, 2, 2, BF16, BF16, 0, 1.0, 0) == 4
    assert mm(P, P, P, None, 0, 2, 2, 2, 2, 2, F32, F32, 0, 1.0, 0) == 0           # empty: ok, no launch


def test_batched_argument_errors(pbk):
    P = 0x1000
    bm = pbk.pbk_batched_matmul
    assert bm(P, P, P, None, 2, 4, 4, 4, 4, 4, 4, 16, 16, 15, 1, 1, 0, 1.0, 0) == 3   # stride_c overlaps
    assert bm(P, P, P, None, 2, 4, 4, 4, 4, 4, 4, -1, 16, 16, 1, 1, 0, 1.0, 0) == 3
    assert bm(P, P, P, None, -2, 4, 4, 4, 4, 4, 4, 16, 16, 16, 1, 1, 0, 1.0, 0) == 2
    assert bm(P, P, P, None, 0, 4, 4, 4, 4, 4, 4, 16, 16, 16, 1, 1, 0, 1.0, 0) == 0


def test_conv_argument_errors(pbk):
    P = 0x1000
    cv = pbk.pbk_conv2d_nhwc
    ok_tail = (1, 1, 1.0, 0)
    assert cv(P, P, P, None, 1, 2, 2, 8, 8, 3, 3, 1, 1, 0, 0, 1, 1, *ok_tail) == 2    # empty output
    assert cv(P, P, P, None, 1, 8, 8, 8, 8, 3, 3, 0, 1, 0, 0, 1, 1, *ok_tail) == 2    # stride 0
    assert cv(P, P, P, None, 1, 8, 8, 8, 8, 3, 3, 1, 1, -1, 0, 1, 1, *ok_tail) == 2   # negative pad
    assert cv(P, P, P, None, 1, 8, 8, 0, 8, 3, 3, 1, 1, 0, 0, 1, 1, *ok_tail) == 2    # Cin 0
    assert cv(None, P, P, None, 1, 8, 8, 8, 8, 3, 3, 1, 1, 0, 0, 1, 1, *ok_tail) == 1
    assert cv(P, P, P, None, 1, 8, 8, 8, 8, 3, 3, 1, 1, 0, 0, 1, 1, 1, 1, 1.0, 1) == 6  # bias missing
    assert cv(P, P, P, None, 0, 8, 8, 8, 8, 3, 3, 1, 1, 0, 0, 1, 1, *ok_tail) == 0    # no images


def test_attention_argument_errors(pbk):
    F32, BF16 = 0, 1
    P = 0x1000           # fake, aligned, never dereferenced: every call below fails validation
    att = pbk.pbk_attention

    def call(Q=P, K=P, V=P, bias=None, O=P, batch=2, Nq=8, Nk=8, D=16, ldq=16, ldk=16, ldv=16, ldo=16,
             sq=128, sk=128, sv=128, so=128, ldb=0, sb=0, dtype=BF16):
        return att(Q, K, V, bias, O, batch, Nq, Nk, D, ldq, ldk, ldv, ldo, sq, sk, sv, so, ldb, sb, dtype, 1.0)
    assert call(dtype=3) == 5 and call(dtype=9) == 5          # FP8 / unknown element type
    assert call(Nq=-1) == 2 and call(D=0) == 2 and call(batch=-3) == 2
    assert call(Nk=0) == 2                                    # softmax over no keys
    assert call(batch=0) == 0 and call(Nq=0) == 0             # nothing to do
    assert call(Nq=0, Nk=0) == 0
    assert call(Q=None) == 1 and call(K=None) == 1 and call(V=None) == 1 and call(O=None) == 1
    assert call(ldq=15) == 3 and call(ldk=8) == 3 and call(ldv=15) == 3 and call(ldo=1) == 3
    assert call(sq=-1) == 3 and call(so=100) == 3             # output entries would overlap
    assert call(bias=P, ldb=7) == 3 and call(bias=P, ldb=8, sb=-1) == 3
    assert call(Q=P + 1) == 4 and call(O=P + 1) == 4 and call(bias=P + 2, ldb=8) == 4
    assert call(Q=P + 2, dtype=F32) == 4
    assert call(D=600, ldq=600, ldk=600, ldv=600, ldo=600, sq=4800, sk=4800, sv=4800, so=4800, dtype=F32) == 7


def test_causal_attention_argument_errors(pbk):
    BF16 = 1
    P = 0x1000
    att = pbk.pbk_attention_causal

    def call(Q=P, K=P, V=P, O=P, batch=2, Nq=8, Nk=8, D=16, ldq=16, ldk=16, ldv=16, ldo=16,
             sq=128, sk=128, sv=128, so=128, dtype=BF16):
        return att(Q, K, V, O, batch, Nq, Nk, D, ldq, ldk, ldv, ldo, sq, sk, sv, so, dtype, 1.0)
    assert call(dtype=5) == 5 and call(Nk=0) == 2 and call(batch=0) == 0
    assert call(V=None) == 1 and call(ldk=8) == 3 and call(so=100) == 3 and call(Q=P + 1) == 4


def test_conv_variant_argument_errors(pbk):
    F32 = 0
    P = 0x1000
    pad4 = pbk.pbk_conv2d_nhwc_pad4
    tr = pbk.pbk_conv2d_transpose_nhwc

    def p4(N=1, H=8, W=8, Cin=4, Cout=4, KH=3, KW=3, sh=1, sw=1, pt=0, pb=0, pl=0, pr=0, dh=1, dw=1, x=P):
        return pad4(x, P, P, None, N, H, W, Cin, Cout, KH, KW, sh, sw, pt, pb, pl, pr, dh, dw, F32, F32, 1.0, 0)
    assert p4(pt=-1) == 2 and p4(pr=-2) == 2 and p4(sh=0) == 2 and p4(dw=0) == 2
    assert p4(H=2, pt=0, pb=0) == 2                 # empty output
    assert p4(N=0) == 0
    assert p4(x=None) == 1

    def t(N=1, H=4, W=4, Cin=4, Cout=4, KH=3, KW=3, sh=2, sw=2, ph=0, pw=0, oh=0, ow=0, dh=1, dw=1, x=P):
        return tr(x, P, P, None, N, H, W, Cin, Cout, KH, KW, sh, sw, ph, pw, oh, ow, dh, dw, F32, F32, 1.0, 0)
    assert t(oh=2) == 2                             # out_pad must stay below stride or dilation
    assert t(oh=-1) == 2 and t(ph=-1) == 2 and t(sh=0) == 2
    assert t(H=1, W=1, KH=1, KW=1, sh=1, sw=1, ph=1, pw=1) == 2      # empty output
    assert t(N=0) == 0 and t(x=None) == 1


def test_int8_argument_errors(pbk):
    P = 0x1000
    mm = pbk.pbk_matmul_int8

    def call(A=P, B=P, C=P, M=4, N=4, K=16, lda=16, ldb=16, ldc=4, tb=1, scale=P, bias=None, mid=0.0, mul=None,
             add=None, relu=0, out_scale=1.0, out=5):
        return mm(A, B, C, M, N, K, lda, ldb, ldc, tb, scale, bias, mid, mul, add, relu, out_scale, out)
    assert call(out=1) == 5 and call(out=2) == 5              # outputs are int8 or fp32
    assert call(scale=None) == 6 and call(out_scale=0.0) == 6 and call(mid=-1.0) == 6
    assert call(M=-1) == 2 and call(K=131072, lda=131072, ldb=131072) == 7
    assert call(A=None) == 1 and call(C=None) == 1
    assert call(lda=8) == 3 and call(ldc=3) == 3 and call(tb=0, ldb=3) == 3
    assert call(scale=P + 2) == 4 and call(out=0, C=P + 2) == 4
    assert call(M=0) == 0


def test_residual_argument_errors(pbk):
    F32 = 0
    P = 0x1000
    mr = pbk.pbk_matmul_residual
    assert mr(P, P, P, None, None, 2, 2, 2, 2, 2, 2, 2, F32, F32, 0, 1.0, 1.0, 0) == 1       # R missing
    assert mr(P, P, P, None, P, 2, 2, 2, 2, 2, 2, 1, F32, F32, 0, 1.0, 1.0, 0) == 3          # ldr < N
    assert mr(P, P, P, None, P + 2, 2, 2, 2, 2, 2, 2, 2, F32, F32, 0, 1.0, 1.0, 0) == 4      # R misaligned
    assert mr(P, P, P, None, P, 2, 2, 2, 1, 2, 2, 2, F32, F32, 0, 1.0, 1.0, 0) == 3          # lda < K (plain checks still run)
    assert mr(P, P, P, None, P, 0, 2, 2, 2, 2, 2, 2, F32, F32, 0, 1.0, 1.0, 0) == 0
    cr = pbk.pbk_conv2d_nhwc_residual
    assert cr(P, P, P, None, None, 1, 4, 4, 2, 2, 3, 3, 1, 1, 1, 1, 1, 1, F32, F32, 1.0, 1.0, 0) == 1
    assert cr(P, P, P, None, P, 1, 4, 4, 2, 2, 3, 3, 0, 1, 1, 1, 1, 1, F32, F32, 1.0, 1.0, 0) == 2


def test_int8_is_not_an_input_type_of_the_plain_convolution_calls(pbk):
    """PBK_INT8 (5) reaches the quantised epilogue only through pbk_conv2d_nhwc_int8, which checks
    its own parameters; every other convolution entry point must refuse it before any launch."""
    P = 0x1000
    INT8, F32 = 5, 0
    geom = (1, 8, 8, 16, 16, 3, 3, 1, 1)                     # N H W Cin Cout KH KW stride
    for out in (F32, INT8):
        assert pbk.pbk_conv2d_nhwc(P, P, P, None, *geom, 1, 1, 1, 1, INT8, out, 1.0, 0) == 5
        assert pbk.pbk_conv2d_nhwc_pad4(P, P, P, None, *geom, 1, 1, 1, 1, 1, 1, INT8, out, 1.0, 0) == 5
        assert pbk.pbk_conv2d_transpose_nhwc(P, P, P, None, *geom, 1, 1, 0, 0, 1, 1, INT8, out, 1.0, 0) == 5
        assert pbk.pbk_conv2d_nhwc_residual(P, P, P, None, P, *geom, 1, 1, 1, 1, INT8, out, 1.0, 1.0, 0) == 5
    assert pbk.pbk_matmul_residual(P, P, P, None, P, 2, 2, 2, 2, 2, 2, 2, INT8, F32, 0, 1.0, 1.0, 0) == 5
    # the int8 entry point itself still validates: missing scale, bad output type
    cq = pbk.pbk_conv2d_nhwc_int8
    assert cq(P, P, P, *geom, 1, 1, 1, 1, None, None, 0.0, None, None, 0, 1.0, INT8) == 6
    assert cq(P, P, P, *geom, 1, 1, 1, 1, P, None, 0.0, None, None, 0, 1.0, 1) == 5
    assert cq(P, P, P, 0, *geom[1:], 1, 1, 1, 1, P, None, 0.0, None, None, 0, 1.0, INT8) == 0     # no images


def test_force_kernel_choices(pbk):
    assert pbk.pbk_force_kernel("generic") == 0
    assert pbk.pbk_force_kernel("mfma") == 0 and pbk.pbk_force_kernel("mfma:7") == 0
    assert pbk.pbk_force_kernel("gather") == 0 and pbk.pbk_force_kernel("small") == 0
    assert pbk.pbk_force_kernel("mfma:") == 7 and pbk.pbk_force_kernel("fastest") == 7
    assert pbk.pbk_force_kernel("") == 0 and pbk.pbk_force_kernel(None) == 0


def test_int8_unfolded_batch_norm_argument_errors(pbk):
    P = 0x1000
    mm = pbk.pbk_matmul_int8_bn

    def call(mean=P, var=P, gamma=P, beta=P, scale=P, out=5, M=4):
        return mm(P, P, P, M, 4, 16, 16, 16, 4, 1, scale, None, 0.0, mean, var, 1e-5, gamma, beta, 1, 1.0, out)
    assert call(mean=None) == 6 and call(var=None) == 6 and call(gamma=None) == 6 and call(beta=None) == 6
    assert call(mean=P + 2) == 4 and call(scale=None) == 6 and call(out=1) == 5
    assert call(M=0) == 0
    cv = pbk.pbk_conv2d_nhwc_int8_bn
    geom = (1, 8, 8, 16, 16, 3, 3, 1, 1, 1, 1, 1, 1)
    assert cv(P, P, P, *geom, P, None, 0.0, None, P, 1e-5, P, P, 0, 1.0, 5) == 6
    assert cv(P, P, P, 0, *geom[1:], P, None, 0.0, P, P, 1e-5, P, P, 0, 1.0, 5) == 0
