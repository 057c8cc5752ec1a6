"""GPU parity of the products with the inner dimension split across workgroups (Sec. 3.2, Fig. 2: the same
product, for shapes with few output tiles): against the CPU oracle on the same seeded inputs, to the bar of the
unsplit products -- int8 bit-exact, floating results within 1e-2 relative of the fp64 oracle and, for fp32 output,
within the bound of K fp32 additions -- and against the unsplit entry points."""
import numpy as np
import pytest
import torch

import oracle
from paper_2104_08378_amd import sp24, synth
from test_gpu_parity import NAME_OF, REL_TOL, rel_err
from util import OUT_DT, out_to_f64, to_gpu

pytestmark = pytest.mark.gpu

IN_DT = {"f16": torch.float16, "bf16": torch.bfloat16, "i8": torch.int8}

CASES = [
    # dtype, out, M, N, K, layout, B order -- every one a shape that is split (asserted below)
    ("i8", "i32", 1024, 64, 8192, "tiled", "k"),        # 64 steps in 8 slices
    ("i8", "i32", 1000, 100, 6176, "canonical", "k"),   # ragged M and N; a partial last step (in the last slice)
    ("bf16", "bf16", 512, 96, 3104, "canonical", "k"),  # 48 steps and half a step
    ("f16", "f32", 256, 256, 4096, "tiled", "n"),       # N-major B
    ("bf16", "f32", 2048, 128, 4096, "tiled", "k"),     # 16 tiles
    ("bf16", "f16", 256, 64, 3200, "tiled", "k"),       # 50 steps: slices of 7, ..., 7 and 1
    ("i8", "i32", 192, 48, 8192, "canonical", "n"),     # one ragged tile column, N-major B
    ("f16", "f16", 128, 65, 4096, "canonical", "k"),    # odd N: rows of the partial images padded to 68
    ("bf16", "bf16", 4096, 64, 8192, "tiled", "k"),     # 32 tiles, 128 steps
    ("bf16", "bf16", 320, 40, 4096, "canonical", "k"),  # ragged M and N
    ("i8", "i32", 32, 256, 4096, "tiled", "k"),         # one row block: two tiles with 96 rows never stored
    ("f16", "f32", 8, 200, 4096, "canonical", "n"),     # fewer rows than a row block
    # N <= 32: the streaming kernel, slices of whole 64-column tiles
    ("bf16", "bf16", 1024, 16, 8192, "tiled", "k"),     # 32 row blocks, 4 slices
    ("i8", "i32", 512, 32, 16384, "canonical", "k"),    # 16 row blocks, 8 slices
    ("f16", "f32", 96, 7, 8192, "canonical", "k"),      # ragged N; 3 row blocks
    ("i8", "i32", 2048, 1, 12352, "tiled", "k"),        # N = 1; 193 tiles: uneven slices
    ("f16", "f16", 128, 16, 8208, "canonical", "k"),    # K % 64 = 16: the dense product has a partial last tile, the sparse one is not split
]


def operands(dtype, M, N, K, layout, b_order, seed):
    A, Bt = synth.make(NAME_OF[dtype], M=M, N=N, K=K, seed=seed)
    Pn = oracle.prune(A, dtype)
    Bmath = np.ascontiguousarray(Bt.T)
    Bd = to_gpu(Bt, dtype) if b_order == "k" else to_gpu(Bmath, dtype)
    V, meta = sp24.sp24_compress(to_gpu(A, dtype), layout=layout)
    return Pn, Bmath, Bd, V, meta


@pytest.mark.parametrize("case", CASES)
def test_split_products_match_oracle_and_the_unsplit_products(case):
    dtype, out, M, N, K, layout, b_order = case
    assert sp24.sp24_splitk_workspace_bytes(M, N, K, IN_DT[dtype]) > 0
    Pn, Bmath, Bd, V, meta = operands(dtype, M, N, K, layout, b_order, seed=21)
    ref = oracle.gemm(Pn, Bmath, dtype)
    Pd = to_gpu(Pn, dtype)
    for sparse in (True, False):
        if sparse:
            D = sp24.sp24_spmm_splitk(V, meta, Bd, OUT_DT[out], b_order=b_order, layout=layout)
            D2 = sp24.sp24_spmm_splitk(V, meta, Bd, OUT_DT[out], b_order=b_order, layout=layout)
            U = sp24.sp24_spmm(V, meta, Bd, OUT_DT[out], b_order=b_order, layout=layout)
        else:
            D = sp24.sp24_gemm_dense_splitk(Pd, Bd, OUT_DT[out], b_order=b_order)
            D2 = sp24.sp24_gemm_dense_splitk(Pd, Bd, OUT_DT[out], b_order=b_order)
            U = sp24.sp24_gemm_dense(Pd, Bd, OUT_DT[out], b_order=b_order)
        torch.cuda.synchronize()
        assert torch.equal(D.view(torch.uint8), D2.view(torch.uint8)), (case, sparse)     # the same from call to call
        if dtype == "i8":
            assert np.array_equal(D.cpu().numpy(), ref), (case, sparse)
            assert torch.equal(D, U), (case, sparse)
        else:
            e = rel_err(out_to_f64(D), ref)
            assert e <= REL_TOL, (case, sparse, e)
            scale = np.abs(oracle.to_double(Pn, dtype)) @ np.abs(oracle.to_double(Bmath, dtype))
            if out == "f32":
                assert (np.abs(out_to_f64(D) - ref) <= K * 2.0 ** -24 * scale + 1e-30).all()
            # against the unsplit product: two roundings to the output type and two fp32 summation orders apart
            ulp = {"f32": 2.0 ** -23, "f16": 2.0 ** -10, "bf16": 2.0 ** -7}[out]
            assert (np.abs(out_to_f64(D) - out_to_f64(U)) <= 2 * K * 2.0 ** -24 * scale + ulp * np.abs(ref) + 1e-30).all(), (case, sparse)


def test_workspace_contents_are_ignored_and_a_workspace_serves_calls_of_different_shapes():
    big = ("i8", "i32", 1024, 64, 8192, "tiled", "k")
    small = ("bf16", "f32", 256, 64, 3200, "tiled", "k")
    need = max(sp24.sp24_splitk_workspace_bytes(c[2], c[3], c[4], IN_DT[c[0]]) for c in (big, small))
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")     # NaN bit patterns / -1
    for dtype, out, M, N, K, layout, b_order in (big, small, big):
        Pn, Bmath, Bd, V, meta = operands(dtype, M, N, K, layout, b_order, seed=22)
        ref = oracle.gemm(Pn, Bmath, dtype)
        D = sp24.sp24_spmm_splitk(V, meta, Bd, OUT_DT[out], b_order=b_order, layout=layout, workspace=ws)
        torch.cuda.synchronize()
        used = sp24.sp24_splitk_workspace_bytes(M, N, K, IN_DT[dtype])
        assert not bool((ws[:used] == 0xFF).all())                      # the partial products went through it
        if dtype == "i8":
            assert np.array_equal(D.cpu().numpy(), ref)
        else:
            assert rel_err(out_to_f64(D), ref) <= REL_TOL
        ws.fill_(0xFF)


@pytest.mark.parametrize("dtype,out,M,N,K", [("bf16", "bf16", 512, 16, 1024), ("i8", "i32", 16, 32, 4096), ("f16", "f32", 256, 256, 128)])
def test_shapes_that_are_not_split_take_the_unsplit_path(dtype, out, M, N, K):
    """Workspace size 0: the call is the unsplit product, bit for bit, and needs no workspace."""
    assert sp24.sp24_splitk_workspace_bytes(M, N, K, IN_DT[dtype]) == 0
    Pn, Bmath, Bd, V, meta = operands(dtype, M, N, K, "canonical", "k", seed=23)
    L = sp24.lib()
    D = torch.empty((M, N), dtype=OUT_DT[out], device="cuda")
    st = L.sp24_spmm_splitk(V.data_ptr(), meta.data_ptr(), Bd.data_ptr(), D.data_ptr(), M, N, K, K, N, sp24._DT[V.dtype],
                            sp24._DT[D.dtype], 0, sp24.CANONICAL, None, 0, None)
    assert st == 0
    U = sp24.sp24_spmm(V, meta, Bd, OUT_DT[out])
    torch.cuda.synchronize()
    assert torch.equal(D.view(torch.uint8), U.view(torch.uint8))


@pytest.mark.parametrize("dtype,out,M,N,K", [("bf16", "bf16", 8192, 64, 8192), ("i8", "i32", 8192, 128, 8192), ("bf16", "bf16", 512, 32, 16384)])
def test_split_products_at_the_sizes_bench_times(dtype, out, M, N, K):
    """The shapes of bench.py --few-tiles, tiled layout, K-major B: sampled rows x columns that the oracle computes one by one."""
    assert sp24.sp24_splitk_workspace_bytes(M, N, K, IN_DT[dtype]) > 0
    A, Bt = synth.make(NAME_OF[dtype], M=M, N=N, K=K, seed=31)
    Ad, Bd = to_gpu(A, dtype), to_gpu(Bt, dtype)
    V, meta = sp24.sp24_compress(Ad, layout="tiled")
    P = sp24.sp24_prune(Ad)
    D = sp24.sp24_spmm_splitk(V, meta, Bd, OUT_DT[out], layout="tiled")
    Dd = sp24.sp24_gemm_dense_splitk(P, Bd, OUT_DT[out])
    torch.cuda.synchronize()
    rng = np.random.default_rng(9)
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 127, 128, M - 1], rng.integers(0, M, 40)]))
    cols = np.unique(np.concatenate([[0, 1, 31, N - 1], rng.integers(0, N, 24)]))
    Prows = oracle.prune(np.ascontiguousarray(A[rows]), dtype)
    ref = oracle.gemm(Prows, np.ascontiguousarray(Bt[cols].T), dtype)
    for got_t in (D, Dd):
        got = got_t[torch.as_tensor(rows, device="cuda")][:, torch.as_tensor(cols, device="cuda")]
        if dtype == "i8":
            assert np.array_equal(got.cpu().numpy(), ref)
        else:
            assert rel_err(out_to_f64(got), ref) <= REL_TOL
