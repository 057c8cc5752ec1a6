"""GPU parity for the 8-bit float input type (4 exponent bits, bias 7, 3 fraction bits, no infinities) through
every operation: prune / compress / decompress and the mask operations bit-exact, products within the tolerance of
the other float types (fp32 accumulation of exact products), the retained magnitude, the searches."""
import numpy as np
import pytest
import torch

import oracle
from paper_2104_08378_amd import sp24, synth
from util import out_to_f64, tiled_from_canonical, to_bits, to_gpu
from test_gpu_parity import REL_TOL, rel_err

pytestmark = pytest.mark.gpu

# Tolerance of the 8-bit float products.  The products themselves are exact (4-bit significands), but the matrix
# instruction adds the products of one instruction in a single aligned sum that keeps fewer bits below its largest
# term than an fp32 addition would: measured on this chip, errors of up to 2^-16.5 of sum |p||b| with fp32 output.
# Against outputs that cancel to nearly nothing that is more than 1e-2 of the floored denominator the other types
# use, so the criterion gets a second, absolute term: |gpu - ref| <= 1e-2 * max(|ref|, 1e-3 rms) + 2^-15 sum |p||b|.
F8_ABS = 2.0 ** -15
WORST = {"ratio": 0.0}


def f8_close(got, ref, P, Bt):
    mags = np.abs(oracle.to_double(P, "f8")) @ np.abs(oracle.to_double(Bt, "f8")).T
    floor = 1e-3 * np.sqrt(np.mean(ref * ref)) + 1e-300
    err = np.abs(got - ref)
    WORST["ratio"] = max(WORST["ratio"], float(np.max(err / np.maximum(mags, 1e-300))))
    return bool((err <= REL_TOL * np.maximum(np.abs(ref), floor) + F8_ABS * mags).all())


def draw(M, K, sigma, seed):
    return synth.normal_bits((M, K), sigma, "f8", seed, 9, 0)


def adversarial_f8(M, K, seed):
    """Ties, both zeros, subnormals, the largest finite value and the NaN pattern in either sign."""
    pool = np.array([0x00, 0x80, 0x01, 0x81, 0x38, 0xB8, 0x39, 0x08, 0x7E, 0xFE, 0x7F, 0xFF], dtype=np.uint8)
    return np.random.default_rng(seed).choice(pool, size=(M, K))


@pytest.mark.parametrize("kind", ["normal", "adversarial"])
def test_f8_prune_compress_decompress_bit_exact(kind):
    for i, (M, K) in enumerate([(1, 32), (5, 64), (33, 96), (64, 64), (96, 192), (257, 1056)]):
        A = draw(M, K, 1.0, i) if kind == "normal" else adversarial_f8(M, K, i)
        Ad = to_gpu(A, "f8")
        P = sp24.sp24_prune(Ad)
        V, meta = sp24.sp24_compress(Ad)
        P2 = sp24.sp24_decompress(V, meta)
        torch.cuda.synchronize()
        oP = oracle.prune(A, "f8")
        oV, ometa = oracle.compress(A, "f8")
        assert np.array_equal(to_bits(P), oP), (kind, M, K)
        assert np.array_equal(to_bits(V), oV) and np.array_equal(to_bits(meta), ometa), (kind, M, K)
        assert np.array_equal(to_bits(P2), oP)
        if M % 32 == 0 and K % 64 == 0:
            Vt, mt = sp24.sp24_compress(Ad, layout="tiled")
            Pt = sp24.sp24_decompress(Vt, mt, layout="tiled")
            wantV, wantmeta = tiled_from_canonical(oV, ometa, "f8")
            assert np.array_equal(to_bits(Vt), wantV) and np.array_equal(to_bits(mt), wantmeta), (kind, M, K)
            assert np.array_equal(to_bits(Pt), oP)
            # the pattern of this matrix on other weights (Sec. 4.1 Step 3)
            W = draw(M, K, 0.5, 50 + i)
            Wd = to_gpu(W, "f8")
            assert np.array_equal(to_bits(sp24.sp24_mask_apply(Wd, mt, layout="tiled")), oracle.mask_apply(W, ometa, "f8"))
            wantVm, _ = tiled_from_canonical(oracle.compress_masked(W, ometa, "f8"), ometa, "f8")
            assert np.array_equal(to_bits(sp24.sp24_compress_masked(Wd, mt, layout="tiled")), wantVm)


# M, N, K, layout, b_order: the general kernel (ragged), the streaming kernel, 128x128 tiles, 256x256 tiles (more than
# 200 of them), a ragged K tail on the tiled kernel, an N-major second operand
PRODUCTS = [
    (33, 17, 96, "canonical", "k"),
    (64, 16, 512, "tiled", "k"),
    (256, 192, 320, "tiled", "k"),
    (128, 128, 256, "canonical", "k"),
    (3840, 3840, 256, "tiled", "k"),
    (128, 96, 224, "canonical", "k"),
    (192, 160, 256, "tiled", "n"),
]


@pytest.mark.parametrize("case", PRODUCTS)
@pytest.mark.parametrize("out", [torch.float32, torch.bfloat16, torch.float16])
def test_f8_products_against_the_oracle(case, out):
    M, N, K, layout, bo = case
    if out != torch.float32 and M > 1000:
        pytest.skip("the large shape once")
    A, Bt = draw(M, K, 0.5, M + N), synth.normal_bits((N, K), 1.0, "f8", M + K, 9, 1)
    Ad, Bd = to_gpu(A, "f8"), to_gpu(Bt, "f8")
    if bo == "n":
        Bd = Bd.view(torch.uint8).t().contiguous().view(torch.float8_e4m3fn)
    V, meta = sp24.sp24_compress(Ad, layout=layout)
    P = sp24.sp24_prune(Ad)
    D = sp24.sp24_spmm(V, meta, Bd, out, b_order=bo, layout=layout)
    Dd = sp24.sp24_gemm_dense(P, Bd, out, b_order=bo)
    torch.cuda.synchronize()
    if M > 1000:                                                  # sampled rows of the large shape
        rows = np.unique(np.concatenate([[0, 255, 256, M - 1], np.random.default_rng(1).integers(0, M, 12)]))
    else:
        rows = np.arange(M)
    Pr = oracle.prune(np.ascontiguousarray(A[rows]), "f8")
    ref = oracle.gemm(Pr, np.ascontiguousarray(Bt.T), "f8")
    for got in (D, Dd):
        assert f8_close(out_to_f64(got)[rows], ref, Pr, Bt), (case, WORST)
    if out == torch.float32:
        # with fp32 output the absolute term alone holds the error (no output rounding)
        mags = np.abs(oracle.to_double(Pr, "f8")) @ np.abs(oracle.to_double(Bt, "f8")).T
        assert (np.abs(out_to_f64(D)[rows] - ref) <= F8_ABS * mags + 1e-30).all()
    print("worst |err| / sum|p||b| so far: 2^%.1f" % np.log2(max(WORST["ratio"], 1e-300)))


def test_f8_every_pattern_through_the_matrix_instruction():
    # each of the 254 finite patterns (and both zeros) times 1.0 and times 0.5, one per output: the instruction reads
    # the format exactly as the oracle's decoder does (exponent bias, subnormals, no infinities)
    vals = np.array([b for b in range(256) if b & 0x7F != 0x7F], dtype=np.uint8)
    M, K, N = 64, 64, 32
    A = np.zeros((M, K), dtype=np.uint8)
    for i, b in enumerate(vals):
        A[i % M, 4 * (i // M)] = b                              # one non-zero per group: survives pruning untouched
    Bt = np.zeros((N, K), dtype=np.uint8)
    for n in range(N):
        Bt[n, :] = 0x38 if n % 2 == 0 else 0x30                 # 1.0 / 0.5 in every row of B
    Ad, Bd = to_gpu(A, "f8"), to_gpu(Bt, "f8")
    for layout in ("canonical", "tiled"):
        V, meta = sp24.sp24_compress(Ad, layout=layout)
        D = sp24.sp24_spmm(V, meta, Bd, torch.float32, layout=layout)
        Dd = sp24.sp24_gemm_dense(sp24.sp24_prune(Ad), Bd, torch.float32)
        torch.cuda.synchronize()
        ref = oracle.gemm(A, np.ascontiguousarray(Bt.T), "f8")   # A is already 2:4
        assert np.array_equal(out_to_f64(D), ref) and np.array_equal(out_to_f64(Dd), ref)


def test_f8_nan_propagates_from_kept_positions():
    A = draw(64, 64, 1.0, 77)
    A[3, 8] = 0x7F                                              # NaN ranks highest: kept
    Bt = synth.normal_bits((32, 64), 1.0, "f8", 78, 9, 1)
    V, meta = sp24.sp24_compress(to_gpu(A, "f8"), layout="tiled")
    D = sp24.sp24_spmm(V, meta, to_gpu(Bt, "f8"), torch.float32, layout="tiled")
    torch.cuda.synchronize()
    Dn = out_to_f64(D)
    assert np.isnan(Dn[3]).all() and not np.isnan(np.delete(Dn, 3, axis=0)).any()


def test_f8_other_operations():
    M, K = 96, 128
    A = draw(M, K, 1.0, 80)
    Ad = to_gpu(A, "f8")
    # row-and-column pruning, column gather, figure of merit, search, split product, convolution
    assert np.array_equal(to_bits(sp24.sp24_prune_transposable(Ad)), oracle.prune_transposable(A, "f8"))
    Aadv = adversarial_f8(M, K, 81)
    Aadv[Aadv & 0x7F == 0x7F] = 0x7E                            # (the tie order of the 4x4 search is pinned for finite values)
    assert np.array_equal(to_bits(sp24.sp24_prune_transposable(to_gpu(Aadv, "f8"))), oracle.prune_transposable(Aadv, "f8"))
    perm = np.random.default_rng(82).permutation(K).astype(np.int32)
    pd = torch.from_numpy(perm).cuda()
    assert np.array_equal(to_bits(sp24.sp24_permute_columns(Ad, pd)), oracle.permute_columns(A, perm, "f8"))
    for pp, hp in ((None, None), (pd, perm)):
        got = float(sp24.sp24_retained_magnitude(Ad, pp).cpu()[0])
        assert got == pytest.approx(oracle.retained_magnitude(A, "f8", perm=hp), rel=1e-12)
    An = A.copy()
    An[5, 3] = 0xFF
    assert np.isnan(float(sp24.sp24_retained_magnitude(to_gpu(An, "f8")).cpu()[0]))
    found = sp24.sp24_permute_search(Ad, sweeps=2)
    torch.cuda.synchronize()
    assert np.array_equal(found.cpu().numpy(), oracle.permute_search(A, "f8", sweeps=2))
    found = sp24.sp24_permute_search(to_gpu(An, "f8"), sweeps=1)
    torch.cuda.synchronize()
    assert np.array_equal(found.cpu().numpy(), oracle.permute_search(An, "f8", sweeps=1))
    # split product: few tiles, long K
    M2, N2, K2 = 256, 96, 4096
    A2, B2 = draw(M2, K2, 0.5, 83), synth.normal_bits((N2, K2), 1.0, "f8", 84, 9, 1)
    assert sp24.sp24_splitk_workspace_bytes(M2, N2, K2, torch.float8_e4m3fn) > 0
    V, meta = sp24.sp24_compress(to_gpu(A2, "f8"), layout="tiled")
    D = sp24.sp24_spmm_splitk(V, meta, to_gpu(B2, "f8"), torch.float32, layout="tiled")
    torch.cuda.synchronize()
    ref = oracle.gemm(oracle.prune(A2, "f8"), np.ascontiguousarray(B2.T), "f8")
    assert f8_close(out_to_f64(D), ref, oracle.prune(A2, "f8"), B2)
    # convolution as an implicit GEMM: 3x3, pad 1, 384 channels (three 128-byte chunks of channels per filter tap)
    C, R, S = 384, 3, 3
    W = draw(128, R * S * C, 0.5, 85)
    X = synth.normal_bits((2, 9, 9, C), 1.0, "f8", 86, 9, 1)
    Vc, mc = sp24.sp24_compress(to_gpu(W, "f8"), layout="tiled")
    Dc = sp24.sp24_spmm_conv2d(Vc, mc, to_gpu(X, "f8").view(2, 9, 9, C), torch.float32, R, S, (1, 1), (1, 1), layout="tiled")
    torch.cuda.synchronize()
    refc = oracle.conv2d(oracle.prune(W, "f8"), X, "f8", R, S, (1, 1), (1, 1))
    Bcol = synth.im2col_nhwc(X.reshape(2, 9, 9, C), R, S, 1)    # the same second operand as a matrix, for the magnitudes
    assert f8_close(out_to_f64(Dc), refc, oracle.prune(W, "f8"), Bcol)


def test_f8_rejected_where_it_does_not_apply():
    A = to_gpu(draw(64, 64, 1.0, 90), "f8")
    V, meta = sp24.sp24_compress(A)
    B = to_gpu(draw(32, 64, 1.0, 91), "f8")
    with pytest.raises(sp24.Sp24Error) as e:
        sp24.sp24_spmm(V, meta, B, torch.int32)                 # integer output is for int8 inputs
    assert e.value.status == 4
    with pytest.raises(sp24.Sp24Error):
        sp24.sp24_prune(to_gpu(draw(8, 48, 1.0, 92), "f8"))     # K % 32
