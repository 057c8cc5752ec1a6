"""GPU parity: the HIP library, called through its C ABI, against the CPU
oracle on the same seeded inputs.  Bit-exact for prune / compress / metadata /
decompress and for the int8 product; floating products within max relative
error 1e-2 of the fp64 oracle (the denominator floored at 1e-3 of the result's
RMS so that cancelled-out entries do not blow the ratio up)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2104_08378_amd import sp24, synth
from util import OUT_DT, out_to_f64, tiled_from_canonical, to_bits, to_gpu

pytestmark = pytest.mark.gpu

NAME_OF = {"f16": "tiny_f16", "bf16": "ffn_bf16", "i8": "square_i8"}
REL_TOL = 1e-2


def rel_err(got, ref):
    floor = 1e-3 * np.sqrt(np.mean(ref * ref)) + 1e-300
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor)))


def adversarial(dtype, M, K, seed):
    """Ties, zeros, signed zeros, NaN/inf, -128: every corner of the selection rule."""
    rng = np.random.default_rng(seed)
    if dtype == "i8":
        pool = np.array([-128, -127, -2, -1, 0, 0, 1, 2, 127], dtype=np.int8)
        return rng.choice(pool, size=(M, K))
    if dtype == "f16":
        pool = np.array([0x0000, 0x8000, 0x3C00, 0xBC00, 0x3C01, 0x0001, 0x8001, 0x7C00, 0xFC00, 0x7E00, 0xFE01, 0x7BFF], dtype=np.uint16)
    else:
        pool = np.array([0x0000, 0x8000, 0x3F80, 0xBF80, 0x3F81, 0x0001, 0x8001, 0x7F80, 0xFF80, 0x7FC0, 0xFF81, 0x7F7F], dtype=np.uint16)
    return rng.choice(pool, size=(M, K))


SHAPES = [(1, 16), (5, 48), (33, 80), (64, 64), (96, 192), (257, 1040)]


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
@pytest.mark.parametrize("kind", ["workload", "adversarial"])
def test_prune_compress_decompress_canonical_bit_exact(dtype, kind):
    for i, (M, K) in enumerate(SHAPES):
        if dtype == "i8":
            K = (K + 31) // 32 * 32
        if kind == "workload":
            A, _ = synth.make(NAME_OF[dtype], M=M, N=16, K=K, seed=i)
        else:
            A = adversarial(dtype, M, K, i)
        Ad = to_gpu(A, dtype)
        P = sp24.sp24_prune(Ad)
        V, meta = sp24.sp24_compress(Ad)
        P2 = sp24.sp24_decompress(V, meta)
        torch.cuda.synchronize()
        oP = oracle.prune(A, dtype)
        oV, ometa = oracle.compress(A, dtype)
        assert np.array_equal(to_bits(P), oP), (dtype, kind, M, K)
        assert np.array_equal(to_bits(V), oV), (dtype, kind, M, K)
        assert np.array_equal(to_bits(meta), ometa), (dtype, kind, M, K)
        assert np.array_equal(to_bits(P2), oP), (dtype, kind, M, K)
        # in place
        Q = Ad.clone()
        sp24.sp24_prune(Q, out=Q)
        assert np.array_equal(to_bits(Q), oP)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_strided_rows(dtype):
    M, K, ld = 37, 96, 160
    A, _ = synth.make(NAME_OF[dtype], M=M, N=16, K=ld, seed=3)
    Ad = to_gpu(A, dtype)[:, :K]
    Pbuf = torch.zeros((M, ld), dtype=Ad.dtype, device="cuda")
    sp24.sp24_prune(Ad, out=Pbuf[:, :K])
    V, meta = sp24.sp24_compress(Ad)
    oP = oracle.prune(np.ascontiguousarray(A[:, :K]), dtype)
    oV, ometa = oracle.compress(np.ascontiguousarray(A[:, :K]), dtype)
    assert np.array_equal(to_bits(Pbuf)[:, :K], oP)
    assert (to_bits(Pbuf)[:, K:] == 0).all()
    assert np.array_equal(to_bits(V), oV) and np.array_equal(to_bits(meta), ometa)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_tiled_layout_is_the_documented_permutation(dtype):
    for i, (M, K) in enumerate([(32, 64), (64, 192), (160, 320)]):
        A = adversarial(dtype, M, K, 10 + i) if i == 1 else synth.make(NAME_OF[dtype], M=M, N=16, K=K, seed=i)[0]
        Ad = to_gpu(A, dtype)
        V, meta = sp24.sp24_compress(Ad, layout="tiled")
        P = sp24.sp24_decompress(V, meta, layout="tiled")
        oV, ometa = oracle.compress(A, dtype)
        wantV, wantmeta = tiled_from_canonical(oV, ometa, dtype)
        assert np.array_equal(to_bits(V), wantV), (dtype, M, K)
        assert np.array_equal(to_bits(meta), wantmeta), (dtype, M, K)
        assert np.array_equal(to_bits(P), oracle.prune(A, dtype))


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
@pytest.mark.parametrize("layout", ["canonical", "tiled"])
def test_fixed_mask_operations_bit_exact(dtype, layout):
    """Sec. 4.1 Step 3: the pattern of one matrix applied to another, and its compressed values."""
    for i, (M, K) in enumerate([(32, 64), (96, 192), (160, 1088)] if layout == "tiled" else [(1, 32), (37, 96), (96, 192), (257, 1056)]):
        A, _ = synth.make(NAME_OF[dtype], M=M, N=16, K=K, seed=i)
        W = adversarial(dtype, M, K, 40 + i) if i == 1 else synth.make(NAME_OF[dtype], M=M, N=16, K=K, seed=20 + i)[0]
        _, ometa = oracle.compress(A, dtype)
        Ad, Wd = to_gpu(A, dtype), to_gpu(W, dtype)
        V0, meta = sp24.sp24_compress(Ad, layout=layout)
        P = sp24.sp24_mask_apply(Wd, meta, layout=layout)
        V = sp24.sp24_compress_masked(Wd, meta, layout=layout)
        P2 = sp24.sp24_decompress(V, meta, layout=layout)
        Q = Wd.clone()
        sp24.sp24_mask_apply(Q, meta, layout=layout, out=Q)                    # in place
        torch.cuda.synchronize()
        want = oracle.mask_apply(W, ometa, dtype)
        assert np.array_equal(to_bits(P), want), (dtype, layout, M, K)
        assert np.array_equal(to_bits(Q), want)
        assert np.array_equal(to_bits(P2), want)
        wantV = oracle.compress_masked(W, ometa, dtype)
        if layout == "tiled":
            wantV, _ = tiled_from_canonical(wantV, ometa, dtype)
        assert np.array_equal(to_bits(V), wantV), (dtype, layout, M, K)
        # on the matrix the pattern came from, both reproduce prune / compress
        assert np.array_equal(to_bits(sp24.sp24_mask_apply(Ad, meta, layout=layout)), oracle.prune(A, dtype))
        assert torch.equal(sp24.sp24_compress_masked(Ad, meta, layout=layout).view(torch.uint8), V0.view(torch.uint8))


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_transposable_pruning_bit_exact(dtype):
    """Sec. 6: the exhaustive 4x4-block search; the result and its transpose both compress without loss."""
    for i, (M, K) in enumerate([(4, 32), (36, 96), (128, 256), (260, 1056)]):
        A = adversarial(dtype, M, K, 50 + i) if i == 1 else synth.make(NAME_OF[dtype], M=M, N=16, K=K, seed=30 + i)[0]
        Ad = to_gpu(A, dtype)
        P = sp24.sp24_prune_transposable(Ad)
        Q = Ad.clone()
        sp24.sp24_prune_transposable(Q, out=Q)
        torch.cuda.synchronize()
        want = oracle.prune_transposable(A, dtype)
        assert np.array_equal(to_bits(P), want), (dtype, M, K)
        assert np.array_equal(to_bits(Q), want)
    # the pruned matrix and its transpose are both fixed points of one-directional pruning (both are 2:4)
    M = K = 128
    A = synth.make(NAME_OF[dtype], M=M, N=16, K=K, seed=77)[0]
    P = sp24.sp24_prune_transposable(to_gpu(A, dtype))
    Pt = P.t().contiguous()
    assert torch.equal(sp24.sp24_prune(P).view(torch.uint8), P.view(torch.uint8))
    assert torch.equal(sp24.sp24_prune(Pt).view(torch.uint8), Pt.view(torch.uint8))


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_transposable_pruning_breaks_ties_as_the_search_order_says(dtype):
    """Blocks made of very few distinct magnitudes: most of the 90 patterns tie, and the first one visited must win."""
    rng = np.random.default_rng(91)
    M, K = 64, 256
    if dtype == "i8":
        A = rng.choice(np.array([-1, 0, 1, 1, -128], dtype=np.int8), size=(M, K))
    else:
        one = 0x3C00 if dtype == "f16" else 0x3F80
        A = rng.choice(np.array([0x0000, one, one | 0x8000, 0x8000], dtype=np.uint16), size=(M, K))
    P = sp24.sp24_prune_transposable(to_gpu(A, dtype))
    assert np.array_equal(to_bits(P), oracle.prune_transposable(A, dtype))


MM_CASES = [
    # dtype, out, M, N, K
    ("f16", "f32", 32, 32, 64),
    ("f16", "f16", 96, 80, 208),      # ragged N, K % 64 != 0
    ("bf16", "bf16", 64, 200, 128),
    ("bf16", "f32", 50, 33, 48),      # ragged M and N
    ("i8", "i32", 64, 96, 128),
    ("i8", "i32", 45, 70, 96),
]


def unaligned_rows(B):
    """The same matrix as a view whose rows start K + 4 elements apart: no 16-byte alignment, so the products run
    the general kernel."""
    wide = torch.zeros((B.shape[0], B.shape[1] + 4), dtype=B.dtype, device=B.device)
    wide[:, :B.shape[1]] = B
    return wide[:, :B.shape[1]]


def run_mm_case(dtype, out, M, N, K, layout, b_order, sparse, seed=0):
    A, Bt = synth.make(NAME_OF[dtype], M=M, N=N, K=K, seed=seed)
    Pn = oracle.prune(A, dtype)
    Bmath = np.ascontiguousarray(Bt.T)                      # K x N
    ref = oracle.gemm(Pn, Bmath, dtype)
    Bd = to_gpu(Bt, dtype) if b_order == "k" else to_gpu(Bmath, dtype)
    if sparse:
        V, meta = sp24.sp24_compress(to_gpu(A, dtype), layout=layout)
        D = sp24.sp24_spmm(V, meta, Bd, OUT_DT[out], b_order=b_order, layout=layout)
    else:
        D = sp24.sp24_gemm_dense(to_gpu(Pn, dtype), Bd, OUT_DT[out], b_order=b_order)
    torch.cuda.synchronize()
    if dtype == "i8":
        assert np.array_equal(D.cpu().numpy(), ref), (dtype, M, N, K, layout, b_order, sparse)
    else:
        e = rel_err(out_to_f64(D), ref)
        assert e <= REL_TOL, (dtype, out, M, N, K, layout, b_order, sparse, e)
        if out == "f32":
            # fp32 accumulation: every partial sum is bounded by sum_k |p||b|, each of the K adds errs by <= 2^-24 of it
            scale = np.abs(oracle.to_double(Pn, dtype)) @ np.abs(oracle.to_double(Bmath, dtype))
            assert (np.abs(out_to_f64(D) - ref) <= K * 2.0 ** -24 * scale + 1e-30).all()


@pytest.mark.parametrize("case", MM_CASES)
@pytest.mark.parametrize("b_order", ["k", "n"])
def test_spmm_canonical_matches_oracle(case, b_order):
    run_mm_case(*case, layout="canonical", b_order=b_order, sparse=True)


@pytest.mark.parametrize("case", [c for c in MM_CASES if c[2] % 32 == 0 and c[4] % 64 == 0])
def test_spmm_tiled_matches_oracle(case):
    run_mm_case(*case, layout="tiled", b_order="k", sparse=True)


TILED_CASES = [
    # several workgroup tiles plus ragged edges; the last three are large enough for the 256x256 tile
    ("i8", "i32", 320, 300, 256),
    ("bf16", "bf16", 512, 520, 192),
    ("f16", "f32", 192, 1000, 128),
    ("i8", "i32", 4096, 3300, 128),
    ("bf16", "f32", 3520, 4100, 64),
    ("f16", "f16", 4096, 3328, 128),
    ("i8", "i32", 4096, 3328, 640),       # whole 256x256 tiles: pipelined kernel, 5 steps
    ("bf16", "bf16", 3328, 4096, 448),    # 7 steps
    ("f16", "f32", 4096, 3328, 64),       # a single step
    # more tiles than compute units (several rounds of workgroups), interior and edge tiles
    ("i8", "i32", 4352, 4000, 384),       # 17 x 16 tiles of 256x256, ragged N, 3 steps
    ("bf16", "bf16", 4384, 4001, 128),    # 18 x 16 tiles, ragged M, odd N (no 16-byte stores), 2 steps
    ("f16", "f32", 2400, 2500, 192),      # sparse: 19 x 20 tiles of 128x128, two workgroups to a unit; dense: 10 x 10 tiles of 256x256; ragged both ways, 3 steps
    ("f16", "f32", 3040, 3300, 192),      # 12 x 13 tiles of 256x256: fewer than compute units, ragged both ways
    ("i8", "i32", 3008, 2800, 256),       # 12 x 11 tiles of 256x256: just past what 128x128 tiles cover in one round
]


@pytest.mark.parametrize("case", TILED_CASES)
def test_spmm_tiled_kernels_match_oracle(case):
    run_mm_case(*case, layout="tiled", b_order="k", sparse=True, seed=2)


@pytest.mark.parametrize("case", TILED_CASES)
def test_dense_tiled_kernels_match_oracle(case):
    run_mm_case(*case, layout="canonical", b_order="k", sparse=False, seed=3)


FEW_ROWS_CASES = [
    # fewer rows than a 128x128 tile, down to one: the tiled kernels compute the missing rows on a valid one and store none of them
    ("f16", "f32", 1, 96, 128),
    ("i8", "i32", 8, 304, 256),
    ("bf16", "bf16", 33, 520, 192),
    ("i8", "i32", 48, 128, 640),
    ("f16", "f16", 32, 1000, 128),        # one row block: also in the tiled layout
    ("bf16", "f32", 31, 4104, 64),
]


@pytest.mark.parametrize("case", FEW_ROWS_CASES)
@pytest.mark.parametrize("b_order", ["k", "n"])
def test_products_with_few_rows_match_oracle(case, b_order):
    run_mm_case(*case, layout="canonical", b_order=b_order, sparse=True, seed=12)
    run_mm_case(*case, layout="canonical", b_order=b_order, sparse=False, seed=13)
    if case[2] % 32 == 0:
        run_mm_case(*case, layout="tiled", b_order=b_order, sparse=True, seed=14)


FEW_COLUMNS_CASES = [
    # N <= 32 where the tiled kernels run instead of the streaming one (very many rows), and products small both ways
    ("bf16", "bf16", 24704, 1, 64),       # 193 tiles of 128 rows: sparse and dense 16-bit, a single column
    ("f16", "f32", 24704, 7, 128),
    ("i8", "i32", 20608, 12, 128),        # 161 tiles: the dense 8-bit product (N > 8); the sparse one streams
    ("bf16", "f32", 11008, 24, 192),      # N > 16 from 86 tiles on
    ("i8", "i32", 11136, 32, 256),
    ("f16", "f16", 16, 16, 256),          # fewer than 32 rows and columns
    ("i8", "i32", 8, 31, 128),
]


@pytest.mark.parametrize("case", FEW_COLUMNS_CASES)
def test_products_with_few_columns_on_the_tiled_kernels_match_oracle(case):
    run_mm_case(*case, layout="canonical", b_order="k", sparse=True, seed=15)
    run_mm_case(*case, layout="canonical", b_order="k", sparse=False, seed=16)
    if case[2] % 32 == 0:
        run_mm_case(*case, layout="tiled", b_order="k", sparse=True, seed=17)
    if case[3] * (1 if case[0] == "i8" else 2) % 16 == 0:
        run_mm_case(*case, layout="canonical", b_order="n", sparse=True, seed=18)
        run_mm_case(*case, layout="canonical", b_order="n", sparse=False, seed=19)


NMAJOR_CASES = [
    # B stored N-major (element (k, n) at B[k*ldb + n]) on the tiled kernels: transposing LDS reads
    ("i8", "i32", 320, 304, 256),         # 128x128 tiles, ragged N (a whole number of 16-byte chunks)
    ("bf16", "bf16", 512, 520, 192),
    ("f16", "f32", 192, 1000, 128),
    ("i8", "i32", 4096, 3328, 640),       # 256x256 tiles, 5 steps
    ("bf16", "bf16", 3328, 4096, 448),
    ("f16", "f16", 4096, 3320, 128),      # ragged N on the eight-wavefront shape
    ("i8", "i32", 4352, 4000, 384),
    ("i8", "i32", 320, 300, 256),         # N not a whole number of chunks: the general kernel
]


@pytest.mark.parametrize("case", NMAJOR_CASES)
def test_spmm_n_major_b_matches_oracle(case):
    run_mm_case(*case, layout="tiled", b_order="n", sparse=True, seed=6)


@pytest.mark.parametrize("case", NMAJOR_CASES)
def test_dense_n_major_b_matches_oracle(case):
    run_mm_case(*case, layout="canonical", b_order="n", sparse=False, seed=7)


@pytest.mark.parametrize("dtype,out,M,N,K", [("i8", "i32", 256, 384, 256), ("bf16", "bf16", 4096, 3328, 128), ("f16", "f32", 128, 16, 512)])
@pytest.mark.parametrize("b_order", ["k", "n"])
def test_leading_dimensions_larger_than_the_rows(dtype, out, M, N, K, b_order):
    """A, B and D as windows of wider buffers (lda > K, ldb > K or N, ldd > N): tiled, skinny and dense kernels."""
    A, Bt = synth.make(NAME_OF[dtype], M=M, N=N, K=K, seed=11)
    Pn = oracle.prune(A, dtype)
    ref = oracle.gemm(Pn, np.ascontiguousarray(Bt.T), dtype)
    pad = 64
    Bsrc = to_gpu(Bt, dtype) if b_order == "k" else to_gpu(np.ascontiguousarray(Bt.T), dtype)
    Bbuf = torch.zeros((Bsrc.shape[0], Bsrc.shape[1] + pad), dtype=Bsrc.dtype, device="cuda")
    Bbuf[:, :Bsrc.shape[1]] = Bsrc
    Bv = Bbuf[:, :Bsrc.shape[1]]
    Abuf = torch.zeros((M, K + pad), dtype=Bsrc.dtype, device="cuda")
    Abuf[:, :K] = to_gpu(Pn, dtype)
    V, meta = sp24.sp24_compress(to_gpu(A, dtype), layout="tiled")
    for sparse in (True, False):
        Dbuf = torch.full((M, N + pad), 7, dtype=OUT_DT[out], device="cuda")
        Dv = Dbuf[:, :N]
        if sparse:
            sp24.sp24_spmm(V, meta, Bv, OUT_DT[out], b_order=b_order, layout="tiled", out=Dv)
        else:
            sp24.sp24_gemm_dense(Abuf[:, :K], Bv, OUT_DT[out], b_order=b_order, out=Dv)
        torch.cuda.synchronize()
        assert (Dbuf[:, N:] == 7).all()                       # nothing written past the rows
        if dtype == "i8":
            assert np.array_equal(Dv.cpu().numpy(), ref)
        else:
            assert rel_err(out_to_f64(Dv.contiguous()), ref) <= REL_TOL


@pytest.mark.parametrize("case", TILED_CASES[:9] + [("i8", "i32", 4352, 4000, 384), ("bf16", "f32", 300, 200, 192)])
def test_spmm_canonical_layout_on_the_tiled_kernels(case):
    """The row-major compressed pair feeds the tiled kernels directly (ragged M included)."""
    run_mm_case(*case, layout="canonical", b_order="k", sparse=True, seed=8)


RAGGED_K_CASES = [
    # K not a whole number of 128-byte steps: the last step is filled up with zeros
    ("i8", "i32", 256, 320, 192, "tiled"),        # half a step (one 64-column tile)
    ("i8", "i32", 4096, 3328, 320, "tiled"),      # the same on 256x256 tiles
    ("i8", "i32", 160, 200, 160, "canonical"),    # a quarter step, ragged M and N
    ("i8", "i32", 128, 128, 96, "canonical"),     # a single, partial step
    ("bf16", "bf16", 256, 264, 96, "canonical"),  # 16-bit: K % 64 = 32
    ("f16", "f32", 192, 128, 224, "canonical"),
    ("f16", "f16", 128, 256, 208, "canonical"),   # K % 32 = 16: sparse runs the general kernel, dense the tiled one
]


@pytest.mark.parametrize("case", RAGGED_K_CASES)
@pytest.mark.parametrize("b_order", ["k", "n"])
def test_partial_last_step(case, b_order):
    dtype, out, M, N, K, layout = case
    run_mm_case(dtype, out, M, N, K, layout=layout, b_order=b_order, sparse=True, seed=12)
    run_mm_case(dtype, out, M, N, K, layout="canonical", b_order=b_order, sparse=False, seed=13)


SKINNY_CASES = [
    ("bf16", "bf16", 256, 16, 1024),
    ("f16", "f32", 96, 7, 576),       # ragged N, K split unevenly over the wavefronts
    ("i8", "i32", 128, 32, 2112),
    ("bf16", "f32", 64, 1, 64),
]


@pytest.mark.parametrize("case", SKINNY_CASES)
def test_skinny_kernels_match_oracle(case):
    run_mm_case(*case, layout="tiled", b_order="k", sparse=True, seed=4)
    run_mm_case(*case, layout="canonical", b_order="k", sparse=True, seed=9)
    run_mm_case(case[0], case[1], case[2] + 13, case[3], case[4], layout="canonical", b_order="k", sparse=True, seed=10)   # ragged M
    run_mm_case(*case, layout="canonical", b_order="k", sparse=False, seed=5)


@pytest.mark.parametrize("case", MM_CASES)
def test_dense_gemm_matches_oracle(case):
    run_mm_case(*case, layout="canonical", b_order="k", sparse=False)
    run_mm_case(*case, layout="canonical", b_order="n", sparse=False, seed=1)


def test_all_equal_rows_and_identity_operand():
    # ties everywhere in A; B = identity returns the pruned matrix itself
    M = K = N = 64
    A = np.full((M, K), 0x3C00, dtype=np.uint16)
    V, meta = sp24.sp24_compress(to_gpu(A, "f16"))
    eye = synth.to_bits(np.eye(K), "f16")
    D = sp24.sp24_spmm(V, meta, to_gpu(eye, "f16"), torch.float32)
    want = oracle.to_double(oracle.prune(A, "f16"), "f16")
    assert np.array_equal(out_to_f64(D), want)


def test_empty_problem_is_a_no_op():
    A = torch.empty((0, 64), dtype=torch.float16, device="cuda")
    assert sp24.sp24_prune(A).shape == (0, 64)
    V, meta = sp24.sp24_compress(A)
    B = torch.zeros((16, 64), dtype=torch.float16, device="cuda")
    assert sp24.sp24_spmm(V, meta, B, torch.float32).shape == (0, 16)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("out", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("shape", [(64, 64, 64, True), (64, 64, 64, False), (256, 320, 128, False)])   # the general kernel (B rows unaligned), the tiled kernel
def test_special_values_reach_the_output_as_ieee_conversion_gives_them(dtype, out, shape):
    """Small integers (sums exact in any order), a NaN weight, infinities and sums beyond the 16-bit ranges: the stored
    result is the exact sum converted once, round to nearest even -- NaN stays NaN, overflow becomes infinity."""
    M, N, K, general = shape
    rng = np.random.default_rng(31)
    A = rng.integers(-3, 4, size=(M, K)).astype(np.float64)
    B = rng.integers(-4, 5, size=(K, N)).astype(np.float64)
    A[5, 0:4] = [np.nan, 1.0, 0.0, 0.0]                  # a kept NaN: the whole row of D is NaN
    A[9, 0:4] = [3.0e4, 3.0e4, 0.0, 0.0]                 # products around 1e5: beyond fp16, inside bf16 and fp32
    B[0, :] = 4.0
    B[1, :] = 4.0
    A[12, 8:12] = [np.inf, 0.0, 0.0, 2.0]                # an infinite weight: row 12 of D is +-inf by the sign of B's row 8
    B[8, :] = np.where(np.arange(N) % 2 == 0, 3.0, -2.0)  # (an infinity in B instead would meet the zeros that the dense
    #                                                      product multiplies and the sparse one skips: 0 * inf differs)
    Abits, Bbits = synth.to_bits(A, dtype), synth.to_bits(np.ascontiguousarray(B.T), dtype)      # B stored K-major
    P = oracle.prune(Abits, dtype)
    V, meta = sp24.sp24_compress(to_gpu(Abits, dtype))
    Bd = unaligned_rows(to_gpu(Bbits, dtype)) if general else to_gpu(Bbits, dtype)
    D = sp24.sp24_spmm(V, meta, Bd, OUT_DT[out])
    Dd = sp24.sp24_gemm_dense(to_gpu(P, dtype), Bd, OUT_DT[out])
    torch.cuda.synchronize()
    with np.errstate(invalid="ignore", over="ignore"):
        ref = oracle.gemm(P, synth.to_bits(B, dtype), dtype)                                      # fp64
    want = torch.from_numpy(ref).to(torch.float32).to(OUT_DT[out])   # every finite sum here is exact in fp32
    for got in (D, Dd):
        g = got.cpu()
        assert torch.equal(torch.isnan(g), torch.isnan(want))
        assert torch.equal(torch.nan_to_num(g.float(), nan=0.0), torch.nan_to_num(want.float(), nan=0.0))
    assert torch.isnan(D[5]).all() and torch.isinf(D[12]).all() and D[12, 0] > 0 and D[12, 1] < 0
    if out == "f16":
        assert torch.isinf(D[9]).all()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("shape", [(64, 64, 64, True), (64, 16, 128, False), (256, 320, 128, False)])   # general (B rows unaligned), skinny and tiled kernels
def test_removed_positions_take_no_part_in_the_sum(dtype, shape):
    """Sec. 3.2: the products with removed weights are skipped, not computed -- an infinity in B opposite a removed
    position leaves the result finite (the dense product of the pruned matrix has 0 * inf = NaN there)."""
    M, N, K, general = shape
    rng = np.random.default_rng(37)
    A = rng.integers(1, 4, size=(M, K)).astype(np.float64) * rng.choice([-1.0, 1.0], size=(M, K))
    B = rng.integers(-4, 5, size=(K, N)).astype(np.float64)
    A[:, 20] = 0.0                                        # three non-zeros beside it in the group: always removed
    A[:, 21] = 0.0                                        # ... and so is this one: the group keeps columns 22, 23
    Binf = B.copy()
    Binf[20, :] = np.inf
    Binf[21, :] = np.nan
    Abits = synth.to_bits(A, dtype)
    for layout in ("canonical", "tiled"):
        if layout == "tiled" and (M % 32 or K % 64):
            continue
        V, meta = sp24.sp24_compress(to_gpu(Abits, dtype), layout=layout)
        Bd = to_gpu(synth.to_bits(np.ascontiguousarray(Binf.T), dtype), dtype)
        D = sp24.sp24_spmm(V, meta, unaligned_rows(Bd) if general else Bd, torch.float32, layout=layout)
        torch.cuda.synchronize()
        ref = oracle.gemm(oracle.prune(Abits, dtype), synth.to_bits(B, dtype), dtype)     # the finite B: rows 20, 21 never count
        assert torch.equal(D.cpu(), torch.from_numpy(ref).to(torch.float32)), (dtype, shape, layout)


def test_int8_product_with_minus_128_in_both_operands():
    """-128 has no positive counterpart in int8: its products (+16384 with itself, -16256 with 127) must come out of
    the integer matrix instructions exactly, in the general, the streaming and both tiled kernels."""
    rng = np.random.default_rng(91)
    pool = np.array([-128, -128, -127, 127, -1, 0, 1, 64], dtype=np.int8)
    for M, N, K, layout, general in ((33, 17, 64, "canonical", True), (33, 17, 64, "canonical", False), (64, 16, 256, "tiled", False),
                                     (256, 160, 384, "tiled", False), (128, 128, 128, "canonical", False), (3840, 3840, 128, "tiled", False)):
        A, Bt = rng.choice(pool, size=(M, K)), rng.choice(pool, size=(N, K))
        Ad, Bd = to_gpu(A, "i8"), to_gpu(Bt, "i8")
        if general:
            Bd = unaligned_rows(Bd)
        V, meta = sp24.sp24_compress(Ad, layout=layout)
        D = sp24.sp24_spmm(V, meta, Bd, torch.int32, layout=layout)
        Dd = sp24.sp24_gemm_dense(sp24.sp24_prune(Ad), Bd, torch.int32)
        torch.cuda.synchronize()
        rows = np.arange(M) if M < 1000 else np.unique(np.concatenate([[0, 255, 256, M - 1], rng.integers(0, M, 10)]))
        ref = oracle.gemm(oracle.prune(np.ascontiguousarray(A[rows]), "i8"), np.ascontiguousarray(Bt.T), "i8")
        assert np.array_equal(D.cpu().numpy()[rows], ref), (M, N, K)
        assert np.array_equal(Dd.cpu().numpy()[rows], ref), (M, N, K)
        assert (np.abs(ref) >= 16384).any()
