"""GPU parity of the channel-permutation operations (Sec. 4.1 Step 2, Fig. 6) against the CPU oracle: the column
gather bit-exact, the retained magnitude to 1e-12 relative (its terms are exact doubles, only their order of
addition differs: the sum of n non-negative terms is off by at most n * 2^-53 relative, n < 2^14 per partial sum
and 2^11 partial sums)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2104_08378_amd import sp24, synth
from util import to_bits, to_gpu
from test_gpu_parity import NAME_OF, adversarial

pytestmark = pytest.mark.gpu

# rows x columns: one wavefront pass, ragged passes, a row longer than one LDS region (> 16 KiB), many workgroups
SHAPES = [(1, 32), (5, 96), (37, 160), (130, 1056), (3, 16416), (9000, 64)]


def dev_perm(perm):
    return torch.from_numpy(np.ascontiguousarray(perm, dtype=np.int32)).cuda()


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_permute_columns_bit_exact(dtype):
    for i, (M, K) in enumerate(SHAPES):
        A = adversarial(dtype, M, K, 70 + i) if i == 2 else synth.make(NAME_OF[dtype], M=M, N=16, K=K, seed=60 + i)[0]
        rng = np.random.default_rng(80 + i)
        perm = rng.permutation(K).astype(np.int32)
        Ad = to_gpu(A, dtype)
        P = sp24.sp24_permute_columns(Ad, dev_perm(perm))
        back = sp24.sp24_permute_columns(P, dev_perm(np.argsort(perm)))
        torch.cuda.synchronize()
        assert np.array_equal(to_bits(P), oracle.permute_columns(A, perm, dtype)), (dtype, M, K)
        assert np.array_equal(to_bits(back), A)
    # rows with a pitch larger than K, on both sides; an entry outside 0..K-1 reads column 0
    M, K = 33, 96
    A = synth.make(NAME_OF[dtype], M=M, N=16, K=K, seed=66)[0]
    big = torch.zeros((M, K + 32), dtype=to_gpu(A, dtype).dtype, device="cuda")
    big[:, :K] = to_gpu(A, dtype)
    out = torch.zeros((M, K + 64), dtype=big.dtype, device="cuda")
    perm = np.random.default_rng(9).permutation(K).astype(np.int32)
    sp24.sp24_permute_columns(big[:, :K], dev_perm(perm), out=out[:, :K])
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(out[:, :K]), A[:, perm])
    assert not to_bits(out[:, K:]).any()
    wild = perm.copy()
    wild[5], wild[17] = -3, K
    P = sp24.sp24_permute_columns(to_gpu(A, dtype), dev_perm(wild))
    torch.cuda.synchronize()
    safe = wild.copy()
    safe[[5, 17]] = 0
    assert np.array_equal(to_bits(P), A[:, safe])


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_permute_rows_bit_exact(dtype):
    for i, (M, K) in enumerate(SHAPES):
        A = synth.make(NAME_OF[dtype], M=M, N=16, K=K, seed=110 + i)[0]
        perm = np.random.default_rng(120 + i).permutation(M).astype(np.int32)
        P = sp24.sp24_permute_rows(to_gpu(A, dtype), dev_perm(perm))
        torch.cuda.synchronize()
        assert np.array_equal(to_bits(P), oracle.permute_rows(A, perm, dtype)), (dtype, M, K)
    # pitched rows on both sides; an entry outside 0..M-1 reads row 0
    M, K = 37, 96
    A = synth.make(NAME_OF[dtype], M=M, N=16, K=K, seed=116)[0]
    big = torch.zeros((M, K + 32), dtype=to_gpu(A, dtype).dtype, device="cuda")
    big[:, :K] = to_gpu(A, dtype)
    out = torch.zeros((M, K + 64), dtype=big.dtype, device="cuda")
    perm = np.random.default_rng(19).permutation(M).astype(np.int32)
    perm[4] = M + 3
    sp24.sp24_permute_rows(big[:, :K], dev_perm(perm), out=out[:, :K])
    torch.cuda.synchronize()
    safe = perm.copy()
    safe[4] = 0
    assert np.array_equal(to_bits(out[:, :K]), A[safe])
    assert not to_bits(out[:, K:]).any()


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_retained_magnitude_matches_the_oracle(dtype):
    for i, (M, K) in enumerate(SHAPES):
        A = synth.make(NAME_OF[dtype], M=M, N=16, K=K, seed=90 + i)[0]
        if i == 2:   # ties, signed zeros, -128 (no NaN or infinity: a finite total to compare)
            A = adversarial(dtype, M, K, 75)
            if dtype != "i8":
                finite = (A & 0x7FFF) < (0x7C00 if dtype == "f16" else 0x7F80)
                A = np.where(finite, A, np.uint16(0x3C00 if dtype == "f16" else 0x3F80)).astype(np.uint16)
        rng = np.random.default_rng(100 + i)
        perm = rng.permutation(K).astype(np.int32)
        Ad = to_gpu(A, dtype)
        plain = sp24.sp24_retained_magnitude(Ad)
        ordered = sp24.sp24_retained_magnitude(Ad, dev_perm(perm))
        # the same number by another route on the GPU: prune the gathered matrix, add up |p| in float64
        via = sp24.sp24_prune(sp24.sp24_permute_columns(Ad, dev_perm(perm))).to(torch.float64).abs().sum()
        torch.cuda.synchronize()
        assert plain.item() == pytest.approx(oracle.retained_magnitude(A, dtype), rel=1e-12), (dtype, M, K)
        assert ordered.item() == pytest.approx(oracle.retained_magnitude(A, dtype, perm=perm), rel=1e-12), (dtype, M, K)
        assert ordered.item() == pytest.approx(via.item(), rel=1e-12)
    # int8 totals are integers below 2^53: exact whatever the order
    A = synth.make("square_i8", M=257, N=16, K=1056, seed=7)[0]
    got = sp24.sp24_retained_magnitude(to_gpu(A, "i8")).item()
    assert got == oracle.retained_magnitude(A, "i8")
    # a kept NaN makes the total NaN; an empty matrix gives 0 and overwrites what the cell held
    if dtype != "i8":
        N = synth.make(NAME_OF[dtype], M=8, N=16, K=64, seed=3)[0].copy()
        N[3, 10] = 0x7E00 if dtype == "f16" else 0x7FC0
        assert np.isnan(sp24.sp24_retained_magnitude(to_gpu(N, dtype)).item())
    cell = torch.full((1,), 5.0, dtype=torch.float64, device="cuda")
    sp24.sp24_retained_magnitude(to_gpu(A, "i8")[:0], out=cell)
    assert cell.item() == 0.0


def test_joint_permutation_leaves_the_dense_product_unchanged():
    """Sec. 4.1 Step 2: columns of A and rows of B (the columns of a K-major B) permuted alike -- same product.  Exact
    for int8; checked on the GPU's own dense product."""
    M, N, K = 96, 64, 256
    A, Bt = synth.make("square_i8", M=M, N=N, K=K, seed=12)
    perm = dev_perm(np.random.default_rng(13).permutation(K))
    Ad, Bd = to_gpu(A, "i8"), to_gpu(Bt, "i8")
    D0 = sp24.sp24_gemm_dense(Ad, Bd, torch.int32)
    D1 = sp24.sp24_gemm_dense(sp24.sp24_permute_columns(Ad, perm), sp24.sp24_permute_columns(Bd, perm), torch.int32)
    torch.cuda.synchronize()
    assert torch.equal(D0, D1)
    assert np.array_equal(D0.cpu().numpy(), oracle.gemm(A, np.ascontiguousarray(Bt.T), "i8"))


# --- the search for a column order: the order found must equal the oracle's entry for entry -------------------
# rows x columns: K/4 a power of two and not (groups that sit out rounds); fewer rows than lanes, a ragged last pass
# over the rows, several passes
SEARCH_SHAPES = [(40, 32), (300, 48), (256, 64), (1000, 96), (17, 160), (2100, 128)]


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_permute_search_order_equals_the_oracle(dtype):
    for i, (M, K) in enumerate(SEARCH_SHAPES):
        if dtype == "i8" and K % 32:
            K += 16                                             # int8 needs K % 32 == 0; 48 -> 64 etc. keeps a mix of group counts
        A = adversarial(dtype, M, K, 170 + i) if i in (1, 4) else synth.make(NAME_OF[dtype], M=M, N=16, K=K, seed=160 + i)[0]
        Ad = to_gpu(A, dtype)
        for sweeps in (1, 2):
            got = sp24.sp24_permute_search(Ad, sweeps=sweeps)
            torch.cuda.synchronize()
            want = oracle.permute_search(A, dtype, sweeps=sweeps)
            assert np.array_equal(got.cpu().numpy(), want), (dtype, M, K, sweeps)
        # the figure of merit does not fall (both evaluated on the GPU), and the order is a permutation
        before = float(sp24.sp24_retained_magnitude(Ad).cpu()[0])
        after = float(sp24.sp24_retained_magnitude(Ad, got).cpu()[0])
        assert sorted(got.cpu().tolist()) == list(range(K))
        if not np.isnan(before):
            assert after >= before * (1 - 1e-12)


def test_permute_search_starts_from_a_given_order_and_takes_pitched_rows():
    dtype, M, K = "bf16", 500, 96
    A = synth.make(NAME_OF[dtype], M=M, N=16, K=K, seed=181)[0]
    rng = np.random.default_rng(182)
    start = rng.permutation(K).astype(np.int32)
    big = torch.zeros((M, K + 40), dtype=torch.bfloat16, device="cuda")
    big[:, :K] = to_gpu(A, dtype)
    perm = dev_perm(start)
    out = sp24.sp24_permute_search(big[:, :K], sweeps=2, perm=perm)
    torch.cuda.synchronize()
    assert out.data_ptr() == perm.data_ptr()                    # refined in place
    assert np.array_equal(out.cpu().numpy(), oracle.permute_search(A, dtype, sweeps=2, perm=start))
    # zero sweeps and an empty matrix leave the order alone
    perm2 = dev_perm(start)
    sp24.sp24_permute_search(to_gpu(A, dtype), sweeps=0, perm=perm2)
    sp24.sp24_permute_search(to_gpu(A, dtype)[:0], sweeps=3, perm=perm2)
    torch.cuda.synchronize()
    assert np.array_equal(perm2.cpu().numpy(), start)


def test_permute_search_ties_heavy_int8_and_equal_columns():
    # few distinct magnitudes: most ways tie and the first must win; all columns equal: nothing moves
    rng = np.random.default_rng(183)
    A = rng.integers(-2, 3, size=(700, 128)).astype(np.int8)
    got = sp24.sp24_permute_search(to_gpu(A, "i8"), sweeps=2)
    E = np.full((64, 64), 7, dtype=np.int8)
    same = sp24.sp24_permute_search(to_gpu(E, "i8"), sweeps=1)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.permute_search(A, "i8", sweeps=2))
    assert np.array_equal(same.cpu().numpy(), np.arange(64))


def test_permute_search_leaves_the_sparse_product_path_consistent():
    # the order found, applied to the weights' columns and to the K-major second operand alike, gives a pruned
    # product that the oracle reproduces from the same permuted operands (Sec. 4.1: the result of the layer is kept)
    dtype, M, K, N = "i8", 128, 256, 64
    A, Bt = synth.make(NAME_OF[dtype], M=M, N=N, K=K, seed=184)
    Ad, Bd = to_gpu(A, dtype), to_gpu(Bt, dtype)
    perm = sp24.sp24_permute_search(Ad, sweeps=1)
    Ap, Bp = sp24.sp24_permute_columns(Ad, perm), sp24.sp24_permute_columns(Bd, perm)
    V, meta = sp24.sp24_compress(Ap, layout="tiled")
    D = sp24.sp24_spmm(V, meta, Bp, torch.int32, layout="tiled")
    torch.cuda.synchronize()
    p = perm.cpu().numpy()
    ref = oracle.gemm(oracle.prune(np.ascontiguousarray(A[:, p]), dtype), np.ascontiguousarray(Bt[:, p].T), dtype)
    assert np.array_equal(D.cpu().numpy(), ref)
