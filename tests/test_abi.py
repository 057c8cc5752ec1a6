"""Host-only checks of the C ABI: the library loads, exports everything the
header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2104_08378_amd import sp24

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sp24.h")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sp24_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert {"sp24_prune", "sp24_compress", "sp24_decompress", "sp24_spmm", "sp24_gemm_dense"} <= set(names)
    L = sp24.lib()
    for n in names:
        assert hasattr(L, n), n


def test_size_functions_follow_the_storage_closed_forms():
    # Sec. 3.1: K/2 values and 2 bits per kept value -> K/8 bytes per row
    for dt, es in ((sp24.torch.float16, 2), (sp24.torch.bfloat16, 2), (sp24.torch.int8, 1)):
        M, K = 96, 256
        v, m = sp24.sp24_values_bytes(M, K, dt), sp24.sp24_meta_bytes(M, K, dt)
        assert v == M * K // 2 * es and m == M * K // 8
        assert v + m == M * K * (es / 2 + 1 / 8)
        assert sp24.sp24_meta_bytes(M, K, dt, "tiled") == m
    assert sp24.sp24_values_bytes(8, 24, sp24.torch.float16) == 0      # K % 16
    assert sp24.sp24_values_bytes(8, 48, sp24.torch.int8) == 0         # K % 32
    assert sp24.sp24_meta_bytes(48, 64, sp24.torch.int8, "tiled") == 0  # M % 32
    assert sp24.sp24_meta_bytes(64, 96, sp24.torch.int8, "tiled") == 0  # K % 64


def test_status_strings():
    assert sp24.status_string(0) == "ok"
    for s in range(1, 8):
        assert sp24.status_string(s) not in ("ok", "unknown status")


OK, NULL, SHAPE, ALIGN, DTYPE, LAYOUT = 0, 1, 2, 3, 4, 5
P = 0x10000  # a fake, aligned, never dereferenced device address


@pytest.mark.parametrize("args,want", [
    ((0, P, 32, 64, 64, 64, sp24.F16, None), NULL),
    ((P, P + 0x100000, 32, 24, 64, 64, sp24.F16, None), SHAPE),      # K % 16
    ((P, P + 0x100000, 32, 48, 64, 64, sp24.I8, None), SHAPE),       # K % 32
    ((P, P + 0x100000, 32, 64, 32, 64, sp24.F16, None), SHAPE),      # lda < K
    ((P + 2, P + 0x100000, 32, 64, 64, 64, sp24.F16, None), ALIGN),
    ((P, P + 0x100000, 32, 64, 68, 64, sp24.F16, None), ALIGN),      # row pitch not 16 B
    ((P, P + 0x100000, 32, 64, 64, 64, 7, None), DTYPE),
    ((P, P + 0x100000, 32, 64, 64, 64, sp24.F32, None), DTYPE),
    ((P, P + 64, 32, 64, 64, 64, sp24.F16, None), SHAPE),            # partial overlap
    ((P, P, 32, 64, 64, 128, sp24.F16, None), SHAPE),                # in place needs equal pitch
    ((P, P + 0x100000, -1, 64, 64, 64, sp24.F16, None), SHAPE),
    ((0, 0, 0, 64, 64, 64, sp24.F16, None), OK),                     # empty: nothing to do
])
def test_prune_rejects_bad_arguments_on_the_host(args, want):
    assert sp24.lib().sp24_prune(*args) == want


def test_compress_and_decompress_validation():
    L = sp24.lib()
    big = P + 0x1000000
    assert L.sp24_compress(P, big, big * 2, 48, 64, 64, sp24.F16, sp24.TILED, None) == LAYOUT
    assert L.sp24_compress(P, big, big * 2, 64, 96, 96, sp24.I8, sp24.TILED, None) == LAYOUT
    assert L.sp24_compress(P, big, big * 2, 64, 64, 64, sp24.F16, 9, None) == LAYOUT
    assert L.sp24_compress(P, 0, big, 64, 64, 64, sp24.F16, sp24.CANONICAL, None) == NULL
    assert L.sp24_compress(P, P + 16, big, 64, 64, 64, sp24.F16, sp24.CANONICAL, None) == SHAPE   # V inside A
    assert L.sp24_compress(P, big + 8, big * 2, 64, 64, 64, sp24.F16, sp24.CANONICAL, None) == ALIGN
    assert L.sp24_decompress(big, big * 2, P, 64, 40, 64, sp24.F16, sp24.CANONICAL, None) == SHAPE
    assert L.sp24_decompress(big, 0, P, 64, 64, 64, sp24.F16, sp24.CANONICAL, None) == NULL
    assert L.sp24_decompress(0, 0, 0, 0, 64, 64, sp24.I8, sp24.CANONICAL, None) == OK


def test_matmul_validation():
    L = sp24.lib()
    V, Mt, B, D = P, P + 0x1000000, P + 0x2000000, P + 0x3000000

    def spmm(M=64, N=64, K=64, ldb=64, ldd=64, i=sp24.F16, o=sp24.F32, bo=0, lay=0, V=V, Mt=Mt, B=B, D=D):
        return L.sp24_spmm(V, Mt, B, D, M, N, K, ldb, ldd, i, o, bo, lay, None)

    assert spmm(o=sp24.I32) == DTYPE and spmm(i=sp24.I8, o=sp24.F32) == DTYPE and spmm(i=sp24.F32) == DTYPE
    assert spmm(K=72) == SHAPE and spmm(ldb=32) == SHAPE and spmm(ldd=32) == SHAPE and spmm(N=-2) == SHAPE
    assert spmm(bo=2) == LAYOUT and spmm(lay=3) == LAYOUT and spmm(M=48, lay=sp24.TILED) == LAYOUT
    assert spmm(B=0) == NULL and spmm(Mt=0) == NULL and spmm(D=0) == NULL
    assert spmm(D=D + 2) == ALIGN and spmm(B=B + 1) == ALIGN and spmm(V=V + 8) == ALIGN
    assert spmm(D=B) == SHAPE                                         # output aliases an input
    assert spmm(M=0) == OK and spmm(N=0) == OK
    assert L.sp24_gemm_dense(V, B, D, 64, 64, 64, 32, 64, 64, sp24.F16, sp24.F32, 0, None) == SHAPE
    assert L.sp24_gemm_dense(0, B, D, 64, 64, 64, 64, 64, 64, sp24.F16, sp24.F32, 0, None) == NULL
    assert L.sp24_gemm_dense(V, B, D, 64, 64, 64, 64, 64, 64, sp24.I8, sp24.F16, 0, None) == DTYPE


def test_convolution_validation():
    L = sp24.lib()
    V, Mt, X, D = P, P + 0x1000000, P + 0x2000000, P + 0x3000000

    def conv(M=64, n=2, H=8, W=8, C=16, R=3, S=3, ph=1, pw=1, sh=1, sw=1, ldd=128, i=sp24.F16, o=sp24.F32, lay=0, V=V, Mt=Mt, X=X, D=D):
        return L.sp24_spmm_conv2d(V, Mt, X, D, M, n, H, W, C, R, S, ph, pw, sh, sw, ldd, i, o, lay, None)

    assert conv(o=sp24.I32) == DTYPE and conv(i=sp24.I8, o=sp24.F16) == DTYPE
    assert conv(C=12) == SHAPE                       # 24 bytes per pixel: a 16-byte run would straddle taps
    assert conv(C=8, R=1, S=1, ph=0, pw=0) == SHAPE  # K = 8 is not a legal inner dimension for 16-bit types
    assert conv(i=sp24.I8, o=sp24.I32, C=16, R=1, S=1, ph=0, pw=0) == SHAPE   # K = 16 for int8
    assert conv(R=11, ph=1) == SHAPE and conv(sh=0) == SHAPE and conv(ph=-1) == SHAPE and conv(H=0) == SHAPE
    assert conv(ldd=100) == SHAPE                    # N = 2*8*8 = 128 columns
    assert conv(X=0) == NULL and conv(D=0) == NULL and conv(Mt=0) == NULL
    assert conv(X=X + 1) == ALIGN and conv(D=D + 2) == ALIGN and conv(V=V + 8) == ALIGN
    assert conv(D=X) == SHAPE                        # output aliases the input
    assert conv(M=48, lay=sp24.TILED) == LAYOUT
    assert conv(M=0) == OK and conv(n=0) == OK
    dense = L.sp24_conv2d_dense
    assert dense(V, X, D, 64, 2, 8, 8, 16, 3, 3, 1, 1, 1, 1, 100, 128, sp24.F16, sp24.F32, None) == SHAPE   # lda < K = 144
    assert dense(0, X, D, 64, 2, 8, 8, 16, 3, 3, 1, 1, 1, 1, 144, 128, sp24.F16, sp24.F32, None) == NULL
    assert dense(V, X, D, 0, 2, 8, 8, 16, 3, 3, 1, 1, 1, 1, 144, 128, sp24.F16, sp24.F32, None) == OK


def test_scaled_product_validation():
    L = sp24.lib()
    V, Mt, B, D, W, Bi = P, P + 0x1000000, P + 0x2000000, P + 0x3000000, P + 0x4000000, P + 0x5000000
    f = ctypes.c_float

    def scaled(o=sp24.I8, W=W, Bi=Bi, D=D, M=64):
        return L.sp24_spmm_i8_scaled(V, Mt, B, D, M, 64, 64, 64, 64, W, f(1.0), Bi, 0, f(1.0), o, 0, 0, None)

    assert scaled(o=sp24.I32) == DTYPE
    assert scaled(W=0) == NULL and scaled(W=W + 2) == ALIGN and scaled(Bi=Bi + 1) == ALIGN
    assert scaled(D=W) == SHAPE              # output aliases the scales
    assert scaled(M=0) == OK
    assert L.sp24_gemm_dense_i8_scaled(V, B, D, 64, 64, 64, 64, 64, 64, 0, f(1.0), 0, 0, f(1.0), sp24.F16, 0, None) == NULL
    assert L.sp24_gemm_dense_i8_scaled(V, B, D, 64, 64, 64, 64, 64, 64, W, f(1.0), 0, 0, f(1.0), sp24.I32, 0, None) == DTYPE


def test_fixed_mask_validation():
    L = sp24.lib()
    W, Mt, Pp, V = P, P + 0x1000000, P + 0x2000000, P + 0x3000000

    def apply(M=64, K=64, ldw=64, ldp=64, t=sp24.F16, lay=0, W=W, Mt=Mt, Pp=Pp):
        return L.sp24_mask_apply(W, Mt, Pp, M, K, ldw, ldp, t, lay, None)

    assert apply(t=sp24.F32) == DTYPE and apply(lay=2) == LAYOUT and apply(K=24) == SHAPE and apply(ldp=32) == SHAPE
    assert apply(M=48, lay=sp24.TILED) == LAYOUT
    assert apply(Mt=0) == NULL and apply(W=0) == NULL and apply(Mt=Mt + 4) == ALIGN and apply(Pp=Pp + 2) == ALIGN
    assert apply(Pp=W, ldp=128) == SHAPE and apply(Pp=Mt) == SHAPE and apply(M=0) == OK
    comp = L.sp24_compress_masked
    assert comp(W, Mt, 0, 64, 64, 64, sp24.I8, 0, None) == NULL and comp(W, 0, V, 64, 64, 64, sp24.I8, 0, None) == NULL
    assert comp(W, Mt, W, 64, 64, 64, sp24.I8, 0, None) == SHAPE and comp(W, Mt, V, 64, 48, 64, sp24.I8, 0, None) == SHAPE
    assert comp(W, Mt, V, 0, 64, 64, sp24.I8, 0, None) == OK


def test_transposable_pruning_validation():
    L = sp24.lib()
    A, Pp = P, P + 0x1000000
    f = L.sp24_prune_transposable
    assert f(A, Pp, 64, 64, 64, 64, sp24.F32, None) == DTYPE
    assert f(A, Pp, 62, 64, 64, 64, sp24.F16, None) == SHAPE          # M % 4
    assert f(A, Pp, 64, 24, 64, 64, sp24.F16, None) == SHAPE          # K % 16
    assert f(A, Pp, 64, 64, 32, 64, sp24.F16, None) == SHAPE
    assert f(0, Pp, 64, 64, 64, 64, sp24.F16, None) == NULL and f(A, Pp + 4, 64, 64, 64, 64, sp24.F16, None) == ALIGN
    assert f(A, A + 64, 64, 64, 64, 64, sp24.I8, None) == SHAPE       # partial overlap
    assert f(A, Pp, 0, 64, 64, 64, sp24.F16, None) == OK


def test_channel_permutation_validation():
    L = sp24.lib()
    A, Pp, perm, tot = P, P + 0x1000000, P + 0x2000000, P + 0x3000000
    f = L.sp24_permute_columns
    assert f(A, perm, Pp, 64, 64, 64, 64, sp24.F32, None) == DTYPE
    assert f(A, perm, Pp, 64, 24, 64, 64, sp24.F16, None) == SHAPE       # K % 16
    assert f(A, perm, Pp, 64, 64, 32, 64, sp24.F16, None) == SHAPE       # lda < K
    assert f(A, perm, Pp, 64, 1 << 31, 1 << 31, 1 << 31, sp24.I8, None) == SHAPE   # K must fit the int32 entries
    assert f(0, perm, Pp, 64, 64, 64, 64, sp24.F16, None) == NULL and f(A, 0, Pp, 64, 64, 64, 64, sp24.F16, None) == NULL
    assert f(A, perm + 2, Pp, 64, 64, 64, 64, sp24.F16, None) == ALIGN and f(A, perm, Pp + 4, 64, 64, 64, 64, sp24.F16, None) == ALIGN
    assert f(A, perm, A, 64, 64, 64, 64, sp24.I8, None) == SHAPE         # in place is not possible for a gather
    assert f(A, Pp + 64, Pp, 64, 64, 64, 64, sp24.I8, None) == SHAPE     # the order must not lie in the output
    assert f(A, perm, Pp, 0, 64, 64, 64, sp24.F16, None) == OK
    g = L.sp24_retained_magnitude
    assert g(A, perm, tot, 64, 64, 64, sp24.I32, None) == DTYPE
    assert g(A, perm, tot, 64, 48, 64, sp24.I8, None) == SHAPE           # K % 32
    assert g(0, perm, tot, 64, 64, 64, sp24.F16, None) == NULL and g(A, perm, 0, 64, 64, 64, sp24.F16, None) == NULL
    assert g(A, perm, tot + 4, 64, 64, 64, sp24.F16, None) == ALIGN and g(A, perm + 1, tot, 64, 64, 64, sp24.F16, None) == ALIGN
    assert g(A, perm, A + 64, 64, 64, 64, sp24.F16, None) == SHAPE       # the total must not lie in the matrix
    h = L.sp24_permute_rows
    assert h(A, perm, Pp, 64, 64, 64, 64, sp24.I32, None) == DTYPE
    assert h(A, perm, Pp, 1 << 31, 64, 64, 64, sp24.I8, None) == SHAPE  # M must fit the int32 entries
    assert h(A, 0, Pp, 64, 64, 64, 64, sp24.F16, None) == NULL and h(A, perm + 2, Pp, 64, 64, 64, 64, sp24.F16, None) == ALIGN
    assert h(A, perm, A + 128, 64, 64, 64, 64, sp24.F16, None) == SHAPE   # overlapping source and destination
    assert h(A, perm, Pp, 0, 64, 64, 64, sp24.F16, None) == OK


def test_split_product_validation_and_workspace_size():
    """Only paths that launch nothing: failing checks, and M = 0."""
    L = sp24.lib()
    w = L.sp24_splitk_workspace_bytes
    # slices x M x (N rounded up to 4) x 4 bytes; slices: at most 8, workgroups up to one per compute unit, chosen by
    # the documented estimate (5 us + 400 ns per step; a split costs 6 us + the images at 4 TB/s, twice)
    assert w(8192, 64, 8192, sp24.BF16) == 4 * 8192 * 64 * 4             # 64 tiles of 128x128, 128 steps
    assert w(256, 65, 4096, sp24.F16) == 8 * 256 * 68 * 4
    assert w(512, 512, 8192, sp24.I8) == 8 * 512 * 512 * 4               # 64 steps: eight slices of 8
    assert w(1024, 1024, 1024, sp24.I8) == 0                             # 8 steps: not worth a second kernel
    assert w(2048, 256, 4096, sp24.I8) == 0                              # the images would cost more than the steps saved
    assert w(8192, 128, 8192, sp24.I8) == 4 * 8192 * 128 * 4
    assert w(4096, 4096, 1024, sp24.BF16) == 0                           # fills the chip: not split
    assert w(32, 256, 8192, sp24.I8) == 8 * 32 * 256 * 4                 # few rows: two 128x128 tiles, 64 steps
    assert w(8, 256, 8192, sp24.F16) == 8 * 8 * 256 * 4 and w(8, 32, 8192, sp24.F16) == 0   # N <= 32, M < 32: the general kernel
    # N <= 32 (one workgroup per 32 rows): slices of whole 64-column tiles, 130 / 80 ns per tile, a split costs 8 us
    assert w(8192, 16, 8192, sp24.BF16) == 0                             # 256 row blocks fill the chip
    assert w(4096, 16, 16384, sp24.BF16) == 2 * 4096 * 16 * 4
    assert w(512, 32, 16384, sp24.I8) == 8 * 512 * 32 * 4
    assert w(96, 7, 8192, sp24.F16) == 4 * 96 * 8 * 4                    # at least 32 tiles per slice; rows padded to 8 values
    assert w(4096, 16, 4096, sp24.BF16) == 0 and w(16, 16, 16384, sp24.I8) == 0
    assert w(256, 256, 24, sp24.F16) == 0 and w(256, 256, 4096, sp24.F32) == 0 and w(-1, 256, 4096, sp24.I8) == 0
    V, meta, B, D, ws = P, P + 0x1000000, P + 0x2000000, P + 0x3000000, P + 0x4000000
    f = L.sp24_spmm_splitk
    need = w(256, 64, 4096, sp24.BF16)
    assert need > 0
    base = (256, 64, 4096, 4096, 64, sp24.BF16, sp24.BF16, 0, sp24.CANONICAL)
    assert f(V, meta, B, D, 256, 64, 4096, 4096, 64, sp24.BF16, sp24.I32, 0, sp24.CANONICAL, ws, need, None) == DTYPE
    assert f(V, meta, B, D, 256, 64, 4104, 4104, 64, sp24.BF16, sp24.BF16, 0, sp24.CANONICAL, ws, need, None) == SHAPE
    assert f(V, meta, B, D, *base, 0, need, None) == NULL
    assert f(V, meta, B, D, *base, ws + 8, need, None) == ALIGN
    assert f(V, meta, B, D, *base, ws, need - 1, None) == SHAPE
    assert f(V, meta, B, D, *base, D + 64, need, None) == SHAPE           # workspace over the output
    assert f(V, meta, B, D, *base, V, need, None) == SHAPE and f(V, meta, B, D, *base, B, need, None) == SHAPE
    assert f(V, meta, B, D, 0, 64, 4096, 4096, 64, sp24.BF16, sp24.BF16, 0, sp24.CANONICAL, 0, 0, None) == OK
    g = L.sp24_gemm_dense_splitk
    A = V
    dbase = (256, 64, 8192, 8192, 8192, 64, sp24.I8, sp24.I32, 0)
    need8 = w(256, 64, 8192, sp24.I8)
    assert need8 > 0
    assert g(A, B, D, 256, 64, 8192, 8192, 8192, 64, sp24.I8, sp24.F32, 0, ws, need8, None) == DTYPE
    assert g(A, B, D, 256, 64, 8192, 4096, 8192, 64, sp24.I8, sp24.I32, 0, ws, need8, None) == SHAPE   # lda < K
    assert g(A, B, D, *dbase, 0, need8, None) == NULL and g(A, B, D, *dbase, ws + 4, need8, None) == ALIGN
    assert g(A, B, D, *dbase, ws, need8 // 2, None) == SHAPE and g(A, B, D, *dbase, A + 4096, need8, None) == SHAPE
    assert g(A, B, D, 256, 0, 8192, 8192, 8192, 64, sp24.I8, sp24.I32, 0, 0, 0, None) == OK


def test_split_workspace_is_a_whole_number_of_images():
    """Over random legal shapes: 0, or between 2 and 8 images of M x (N rounded up to 4) accumulator values."""
    import random
    L = sp24.lib()
    rnd = random.Random(5)
    seen = set()
    for _ in range(4000):
        t = rnd.choice([sp24.F16, sp24.BF16, sp24.I8])
        unit = 32 if t == sp24.I8 else 16
        M = rnd.choice([1, 31, 32, 63, 64, 100, 256, 1000, 4096, 8192, 20000])
        N = rnd.choice([1, 7, 16, 32, 33, 64, 100, 128, 256, 1000, 4096])
        K = unit * rnd.randint(1, 2048)
        b = L.sp24_splitk_workspace_bytes(M, N, K, t)
        image = M * ((N + 3) // 4 * 4) * 4
        assert b % image == 0
        assert b == 0 or 2 <= b // image <= 8, (M, N, K, t, b)
        seen.add(b // image)
    assert {0, 2, 4, 8} <= seen


def test_static_scratch_variant_checks_on_the_host():
    # sp24_spmm_splitk_static validates like sp24_spmm_splitk and refuses, before any device call, a shape whose
    # split needs more than the static array holds
    L = sp24.lib()
    f = L.sp24_spmm_splitk_static
    V, META, B, D = P, P + 0x4000000, P + 0x8000000, P + 0x10000000
    M, N, K = 8192, 128, 8192
    assert L.sp24_splitk_workspace_bytes(M, N, K, sp24.BF16) > sp24.STATIC_SCRATCH_BYTES
    assert f(V, META, B, D, M, N, K, K, N, sp24.BF16, sp24.BF16, sp24.B_KMAJOR, sp24.TILED, None) == 7
    assert f(0, META, B, D, M, N, K, K, N, sp24.BF16, sp24.BF16, sp24.B_KMAJOR, sp24.TILED, None) == NULL
    assert f(V, META, B, D, M, N, K + 8, K + 8, N, sp24.BF16, sp24.BF16, sp24.B_KMAJOR, sp24.TILED, None) == SHAPE
    assert f(V, META, B, D, M, N, K, K, N, sp24.BF16, sp24.I32, sp24.B_KMAJOR, sp24.TILED, None) == DTYPE
    assert f(V, META, B, D, 0, N, K, K, N, sp24.BF16, sp24.BF16, sp24.B_KMAJOR, sp24.TILED, None) == OK     # empty
    header = open(HEADER).read()
    assert "#define SP24_STATIC_SCRATCH_BYTES (8u << 20)" in header and sp24.STATIC_SCRATCH_BYTES == 8 << 20


def test_permute_search_validation():
    f = sp24.lib().sp24_permute_search
    A, PERM = P, P + 0x4000000
    assert f(0, PERM, 64, 64, 64, sp24.F16, 1, None) == NULL
    assert f(A, 0, 64, 64, 64, sp24.F16, 1, None) == NULL
    assert f(A, PERM + 2, 64, 64, 64, sp24.F16, 1, None) == ALIGN
    assert f(A, PERM, 64, 40, 64, sp24.F16, 1, None) == SHAPE           # K % 16
    assert f(A, PERM, 64, 48, 64, sp24.I8, 1, None) == SHAPE            # K % 32
    assert f(A, PERM, 64, 64, 32, sp24.F16, 1, None) == SHAPE           # lda < K
    assert f(A, PERM, 64, 64, 64, sp24.F16, -1, None) == SHAPE
    assert f(A, PERM, 64, 64, 64, sp24.F16, 65, None) == SHAPE
    assert f(A, A + 64, 64, 64, 64, sp24.F16, 1, None) == SHAPE         # perm inside A
    assert f(A, PERM, 64, 64, 64, sp24.F32, 1, None) == DTYPE
    assert f(A, PERM, 0, 64, 64, sp24.F16, 3, None) == OK               # empty: nothing to do
    assert f(A, PERM, 64, 64, 64, sp24.F16, 0, None) == OK              # no sweeps: nothing launched
