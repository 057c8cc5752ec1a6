"""sp24_spmm_splitk_static -- the split product for callers that cannot allocate, with its partial products in the
library's own static device array -- against sp24_spmm_splitk with a caller's workspace: same kernels, same slice
order, so the results must be equal bit for bit; and against the oracle to the bar of the other products.  Calls
follow one another on one stream and share the array: a larger problem first, then smaller ones."""
import numpy as np
import pytest
import torch

import oracle
from paper_2104_08378_amd import sp24
from util import out_to_f64, to_bits, to_gpu

pytestmark = pytest.mark.gpu


def _draw(rng, rows, cols, dt, sigma):
    if dt == "i8":
        return rng.integers(-127, 128, size=(rows, cols), dtype=np.int8)
    x = rng.normal(0.0, sigma, size=(rows, cols)).astype(np.float32)
    t = torch.from_numpy(x).to(torch.bfloat16 if dt == "bf16" else torch.float16)
    return t.view(torch.int16).numpy().view(np.uint16)


def _case(rng, M, N, K, dt, out, layout):
    A, Bt = _draw(rng, M, K, dt, 0.05), _draw(rng, N, K, dt, 1.0)
    Ad, Bd = to_gpu(A, dt), to_gpu(Bt, dt)
    V, meta = sp24.sp24_compress(Ad, layout=layout)
    need = sp24.sp24_splitk_workspace_bytes(M, N, K, Ad.dtype)
    return A, Bt, V, meta, Bd, need


# (M, N, K, type, output type, layout): every one is split (the second and later ones need less scratch than the first)
CASES = [
    (1024, 256, 4096, "bf16", torch.bfloat16, "tiled"),       # needs exactly the 8 MiB the array holds
    (256, 256, 8192, "i8", torch.int32, "tiled"),
    (256, 96, 4096, "f16", torch.float32, "canonical"),
    (512, 32, 8192, "bf16", torch.float32, "tiled"),          # the streaming kernel's split
]


def test_static_scratch_equals_workspace_variant_on_calls_in_a_row():
    rng = np.random.default_rng(11)
    needs = []
    for M, N, K, dt, out_dt, layout in CASES:
        A, Bt, V, meta, Bd, need = _case(rng, M, N, K, dt, out_dt, layout)
        assert 0 < need <= sp24.STATIC_SCRATCH_BYTES, (M, N, K, need)
        needs.append(need)
        D_static = torch.full((M, N), -7, dtype=out_dt, device="cuda")
        D_ws = torch.full((M, N), -9, dtype=out_dt, device="cuda")
        sp24.sp24_spmm_splitk_static(V, meta, Bd, out_dt, layout=layout, out=D_static)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        sp24.sp24_spmm_splitk(V, meta, Bd, out_dt, layout=layout, workspace=ws, out=D_ws)
        torch.cuda.synchronize()
        assert np.array_equal(to_bits(D_static), to_bits(D_ws)), (M, N, K, dt)
        # and against the oracle on sampled rows (whole rows, so every column tile is hit)
        rows = np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, 6)]))
        P = oracle.prune(np.ascontiguousarray(A[rows]), dt)
        ref = oracle.gemm(P, np.ascontiguousarray(Bt.T), dt)
        got = out_to_f64(D_static)[rows]
        if dt == "i8":
            assert np.array_equal(got, ref.astype(np.float64))
        else:
            floor = 1e-3 * np.sqrt(np.mean(ref * ref))
            assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor)) <= 1e-2
    assert needs[1] < needs[0]                                # the second call is the smaller one


def test_static_scratch_twice_on_the_same_problem_and_unsplit_shapes():
    rng = np.random.default_rng(12)
    M, N, K, dt, out_dt, layout = CASES[1]
    A, Bt, V, meta, Bd, need = _case(rng, M, N, K, dt, out_dt, layout)
    D1 = sp24.sp24_spmm_splitk_static(V, meta, Bd, out_dt, layout=layout)
    D2 = sp24.sp24_spmm_splitk_static(V, meta, Bd, out_dt, layout=layout)
    torch.cuda.synchronize()
    assert torch.equal(D1, D2)
    # a shape that is not split runs as the plain product
    A, Bt, V, meta, Bd, need = _case(rng, 1024, 1024, 256, "bf16", torch.bfloat16, "tiled")
    assert need == 0
    D = sp24.sp24_spmm_splitk_static(V, meta, Bd, torch.bfloat16, layout="tiled")
    Dp = sp24.sp24_spmm(V, meta, Bd, torch.bfloat16, layout="tiled")
    torch.cuda.synchronize()
    assert torch.equal(D, Dp)


def test_static_scratch_refuses_what_does_not_fit():
    M, N, K = 8192, 128, 8192
    need = sp24.sp24_splitk_workspace_bytes(M, N, K, torch.bfloat16)
    assert need > sp24.STATIC_SCRATCH_BYTES
    V = torch.zeros((M, K // 2), dtype=torch.bfloat16, device="cuda")
    meta = torch.zeros((M, K // 8), dtype=torch.uint8, device="cuda")
    B = torch.zeros((N, K), dtype=torch.bfloat16, device="cuda")
    D = torch.full((M, N), 3.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sp24.Sp24Error) as e:
        sp24.sp24_spmm_splitk_static(V, meta, B, torch.bfloat16, layout="tiled", out=D)
    assert e.value.status == 7
    torch.cuda.synchronize()
    assert bool((D == 3.0).all())                             # nothing was launched
