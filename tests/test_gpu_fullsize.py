"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times (tiled
layout, K-major B, the workload's output type): compress is compared bit for bit on the whole matrix, the
sparse and dense products on sampled rows x columns that the oracle computes one by one."""
import numpy as np
import pytest
import torch

import oracle
from paper_2104_08378_amd import sp24, synth
from util import OUT_DT, out_to_f64, tiled_from_canonical, to_bits, to_gpu

pytestmark = pytest.mark.gpu


def rel_err(got, ref, rms):
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-3 * rms + 1e-300)))


@pytest.mark.parametrize("name", ["tiny_f16", "ffn_bf16", "conv3x3_f16", "square_i8", "skinny_bf16"])
def test_full_size_workload(name):
    w = synth.WORKLOADS[name]
    dt, M, K, N = w["dtype"], w["M"], w["K"], w["N"]
    A, Bt = synth.make(name)
    Ad, Bd = to_gpu(A, dt), to_gpu(Bt, dt)
    V, meta = sp24.sp24_compress(Ad, layout="tiled")
    P = sp24.sp24_prune(Ad)
    D = sp24.sp24_spmm(V, meta, Bd, OUT_DT[w["out"]], layout="tiled")
    Dd = sp24.sp24_gemm_dense(P, Bd, OUT_DT[w["out"]])
    torch.cuda.synchronize()

    # compression of the whole matrix, bit for bit (through the documented permutation)
    oV, ometa = oracle.compress(A, dt)
    wantV, wantmeta = tiled_from_canonical(oV, ometa, dt)
    assert np.array_equal(to_bits(V), wantV)
    assert np.array_equal(to_bits(meta), wantmeta)
    del wantV, wantmeta, oV, ometa
    # and back: the whole decompressed matrix is the whole pruned matrix, both from the oracle and from sp24_prune
    P2 = sp24.sp24_decompress(V, meta, layout="tiled")
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(P2), oracle.prune(A, dt))
    assert torch.equal(P2.view(torch.uint8), P.view(torch.uint8))
    del P2

    # sampled outputs: corners, tile edges and random picks
    rng = np.random.default_rng(7)
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 255, 256 % M, M - 1], rng.integers(0, M, 40)])) % M
    cols = np.unique(np.concatenate([[0, 1, 31, 32 % N, 255 % N, 256 % N, N - 1], rng.integers(0, N, 56)])) % N
    rows, cols = np.unique(rows), np.unique(cols)
    Prows = oracle.prune(np.ascontiguousarray(A[rows]), dt)
    assert np.array_equal(to_bits(P)[rows], Prows)
    ref = oracle.gemm(Prows, np.ascontiguousarray(Bt[cols].T), dt)
    for got_t in (D, Dd):
        got = got_t[torch.as_tensor(rows, device="cuda")][:, torch.as_tensor(cols, device="cuda")]
        if dt == "i8":
            assert np.array_equal(got.cpu().numpy(), ref), name
        else:
            rms = float(np.sqrt(np.mean(ref * ref)))
            assert rel_err(out_to_f64(got), ref, rms) <= 1e-2, name


@pytest.mark.parametrize("dt,out,M,N,K", [("bf16", "bf16", 32000, 1, 4096), ("bf16", "bf16", 32000, 32, 4096),
                                          ("i8", "i32", 32000, 16, 4096), ("f16", "f32", 11008, 24, 4096)])
def test_full_size_tall_products_with_few_columns(dt, out, M, N, K):
    """The output projection of a language model on a handful of tokens: N <= 32 with so many rows that the tiled
    kernels run instead of the streaming one (the 8-bit sparse product at N <= 16 stays with the streaming kernel)."""
    A, Bt = synth.make({"bf16": "ffn_bf16", "f16": "tiny_f16", "i8": "square_i8"}[dt], M=M, N=N, K=K, seed=41)
    Ad, Bd = to_gpu(A, dt), to_gpu(Bt, dt)
    V, meta = sp24.sp24_compress(Ad, layout="tiled")
    P = sp24.sp24_prune(Ad)
    D = sp24.sp24_spmm(V, meta, Bd, OUT_DT[out], layout="tiled")
    Dd = sp24.sp24_gemm_dense(P, Bd, OUT_DT[out])
    torch.cuda.synchronize()
    rng = np.random.default_rng(43)
    rows = np.unique(np.concatenate([[0, 31, 32, 127, 128, M - 129, M - 128, M - 1], rng.integers(0, M, 120)]))
    ref = oracle.gemm(oracle.prune(np.ascontiguousarray(A[rows]), dt), np.ascontiguousarray(Bt.T), dt)
    for got_t in (D, Dd):
        got = got_t[torch.as_tensor(rows, device="cuda")]
        if dt == "i8":
            assert np.array_equal(got.cpu().numpy(), ref)
        else:
            rms = float(np.sqrt(np.mean(ref * ref)))
            assert rel_err(out_to_f64(got), ref, rms) <= 1e-2
    if dt == "i8":
        assert torch.equal(D, Dd)


def test_full_size_convolution_without_im2col():
    """conv3x3_f16 as its title says, an implicit GEMM on the NHWC activations: sampled filters x pixels against
    the oracle's direct convolution of whole images (the images that hold the sampled pixels)."""
    w = synth.WORKLOADS["conv3x3_f16"]
    dt, M = w["dtype"], w["M"]
    A, _ = synth.make("conv3x3_f16", N=196)            # the filter matrix depends on M and K only
    X = synth.conv_activations()                       # [64, 14, 14, 256]
    n_img = X.shape[0]
    Ad, Xd = to_gpu(A, dt), to_gpu(X, dt)
    V, meta = sp24.sp24_compress(Ad, layout="tiled")
    P = sp24.sp24_prune(Ad)
    D = sp24.sp24_spmm_conv2d(V, meta, Xd, OUT_DT[w["out"]], 3, 3, (1, 1), (1, 1), layout="tiled")
    Dd = sp24.sp24_conv2d_dense(P, Xd, OUT_DT[w["out"]], 3, 3, (1, 1), (1, 1))
    torch.cuda.synchronize()
    assert tuple(D.shape) == (M, w["N"])
    rng = np.random.default_rng(8)
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 127, 128, M - 1], rng.integers(0, M, 30)]))
    imgs = [0, 17, n_img - 1]
    Prows = oracle.prune(np.ascontiguousarray(A[rows]), dt)
    for img in imgs:
        ref = oracle.conv2d(Prows, np.ascontiguousarray(X[img:img + 1]), dt, 3, 3, (1, 1), (1, 1))      # [rows, 196]
        rms = float(np.sqrt(np.mean(ref * ref)))
        for got_t in (D, Dd):
            got = got_t[torch.as_tensor(rows, device="cuda")][:, img * 196:(img + 1) * 196]
            assert rel_err(out_to_f64(got), ref, rms) <= 1e-2, img


def test_full_size_quantised_product():
    """square_i8 with the quantised path's epilogue (int8 output): sampled rows x columns, bit for bit."""
    w = synth.WORKLOADS["square_i8"]
    M, K, N = w["M"], w["K"], w["N"]
    A, Bt = synth.make("square_i8")
    rng = np.random.default_rng(12)
    w_scale = rng.uniform(2e-5, 9e-5, size=M).astype(np.float32)
    bias = rng.normal(0.0, 0.3, size=M).astype(np.float32)
    x_scale, inv_y = np.float32(0.02), 40.0
    Ad, Bd = to_gpu(A, "i8"), to_gpu(Bt, "i8")
    V, meta = sp24.sp24_compress(Ad, layout="tiled")
    ws, bs = torch.from_numpy(w_scale).cuda(), torch.from_numpy(bias).cuda()
    D = sp24.sp24_spmm_i8_scaled(V, meta, Bd, torch.int8, ws, x_scale, bs, True, inv_y, layout="tiled")
    Dd = sp24.sp24_gemm_dense_i8_scaled(sp24.sp24_prune(Ad), Bd, torch.int8, ws, x_scale, bs, True, inv_y)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 31, 32, 255, 256, M - 1], rng.integers(0, M, 30)]))
    cols = np.unique(np.concatenate([[0, 31, 32, 255, 256, N - 1], rng.integers(0, N, 40)]))
    Prows = oracle.prune(np.ascontiguousarray(A[rows]), "i8")
    acc = oracle.gemm(Prows, np.ascontiguousarray(Bt[cols].T), "i8")
    want = oracle.requant(acc, w_scale[rows], x_scale, inv_y, bias[rows], True)
    for got_t in (D, Dd):
        got = got_t[torch.as_tensor(rows, device="cuda")][:, torch.as_tensor(cols, device="cuda")].cpu().numpy()
        assert np.array_equal(got, want)
    assert len(np.unique(want)) > 30


def test_full_size_int8_sparse_equals_dense_of_pruned_everywhere():
    """Every one of the 8192 x 8192 outputs: the sparse product of the compressed matrix and the dense product of the
    pruned matrix are the same integers (Sec. 3.2, Fig. 2: the sparse operation skips only multiplications by
    zero), compared on the GPU -- a misplaced tile anywhere would show.  Sampled outputs of both are checked
    against the oracle above."""
    A, Bt = synth.make("square_i8")
    Ad, Bd = to_gpu(A, "i8"), to_gpu(Bt, "i8")
    V, meta = sp24.sp24_compress(Ad, layout="tiled")
    D = sp24.sp24_spmm(V, meta, Bd, torch.int32, layout="tiled")
    Dd = sp24.sp24_gemm_dense(sp24.sp24_prune(Ad), Bd, torch.int32)
    torch.cuda.synchronize()
    assert torch.equal(D, Dd)
    assert int(D.abs().max()) > 100000                           # not trivially equal


def test_full_size_search_for_a_column_order():
    """The search on the matrix bench.py --extras times it on (square_i8's A, 8192 x 8192): the whole order equals
    the oracle's on the first 512 rows (all 8192 columns: eleven rounds of 1024 pairs of groups); on all rows the
    order is a permutation, keeps no less magnitude than before, and every pair of groups of the last round is
    optimal among its 35 ways by the oracle's figure of merit on those eight columns (the order depends on every
    row, so the oracle cannot reproduce it from a sample of rows)."""
    A, _ = synth.make("square_i8")
    M, K = A.shape
    Ad = to_gpu(A, "i8")
    top = np.ascontiguousarray(A[:512])
    got_top = sp24.sp24_permute_search(to_gpu(top, "i8"), sweeps=1)
    perm = sp24.sp24_permute_search(Ad, sweeps=1)
    before = float(sp24.sp24_retained_magnitude(Ad).cpu()[0])
    after = float(sp24.sp24_retained_magnitude(Ad, perm).cpu()[0])
    torch.cuda.synchronize()
    assert np.array_equal(got_top.cpu().numpy(), oracle.permute_search(top, "i8", sweeps=1))
    p = perm.cpu().numpy()
    assert sorted(p.tolist()) == list(range(K))
    assert after >= before
    assert after == oracle.retained_magnitude(A, "i8", perm=p)          # int8: every sum is an exact integer
    # the last round pairs group g (bit 10 clear) with g + 1024
    from itertools import combinations
    rng = np.random.default_rng(11)
    G = K // 4
    for g in rng.choice([g for g in range(G) if not g & (G // 2)], size=24, replace=False):
        h = g + G // 2
        cols = np.concatenate([p[4 * g:4 * g + 4], p[4 * h:4 * h + 4]])
        sub = np.ascontiguousarray(A[:, cols])
        kept = oracle.retained_magnitude(sub, "i8")
        for rest in combinations(range(1, 8), 3):
            first = (0,) + rest
            other = tuple(i for i in range(8) if i not in first)
            way = np.array(first + other, dtype=np.int32)
            assert oracle.retained_magnitude(sub, "i8", perm=way) <= kept, (g, way)
