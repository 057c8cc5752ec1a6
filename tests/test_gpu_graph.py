"""The whole path under HIP graph capture and replay: the library launches on the caller's stream, allocates
nothing and synchronises nothing, so a launch-bound sequence (the 256-cubed configuration spends its time in
launch latency) can be recorded once and replayed.  Every replay, on inputs changed in place in between and with
eager work and synchronisations between the replays, must reproduce the eager result bit for bit."""
import numpy as np
import pytest
import torch

from paper_2104_08378_amd import sp24, synth
from util import to_gpu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,dtype,out", [("tiny_f16", "f16", torch.float32), ("square_i8", "i8", torch.int32)])
def test_path_replays_from_a_graph(name, dtype, out):
    M, N, K = 256, 256, 256
    sets = [tuple(to_gpu(x, dtype) for x in synth.make(name, M=M, N=N, K=K, seed=40 + i)) for i in range(3)]
    A, Bt = sets[0][0].clone(), sets[0][1].clone()
    V = torch.empty((M, K // 2), dtype=A.dtype, device="cuda")
    meta = torch.empty((M, K // 8), dtype=torch.uint8, device="cuda")
    P = torch.empty_like(A)
    D, Dd = torch.empty((M, N), dtype=out, device="cuda"), torch.empty((M, N), dtype=out, device="cuda")
    total = torch.empty(1, dtype=torch.float64, device="cuda")

    def path():
        sp24.sp24_compress(A, layout="tiled", out=(V, meta))
        sp24.sp24_decompress(V, meta, layout="tiled", out=P)
        sp24.sp24_spmm(V, meta, Bt, out, layout="tiled", out=D)
        sp24.sp24_gemm_dense(P, Bt, out, out=Dd)
        sp24.sp24_retained_magnitude(A, out=total)

    path()                                   # first calls outside the capture (one-time kernel attributes)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            path()
    torch.cuda.synchronize()
    for a, b in sets[1:] + sets[:1]:
        A.copy_(a)
        Bt.copy_(b)
        path()                               # eager, on the new inputs
        torch.cuda.synchronize()
        want = [t.clone() for t in (V, meta, P, D, Dd, total)]
        for t in (V, meta, P, D, Dd, total):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((V, meta, P, D, Dd), want):
            assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8))
        assert total.item() == pytest.approx(want[5].item(), rel=1e-12)
        if dtype == "i8":
            assert torch.equal(D, Dd)        # sparse and dense products of the same pruned matrix: exact in int32


@pytest.mark.parametrize("name,dtype,out", [("ffn_bf16", "bf16", torch.bfloat16), ("square_i8", "i8", torch.int32)])
def test_split_product_replays_from_a_graph(name, dtype, out):
    """The two kernels of a split product and their workspace, recorded once; the workspace is scrambled between replays."""
    M, N, K = 256, 64, 8192
    sets = [tuple(to_gpu(x, dtype) for x in synth.make(name, M=M, N=N, K=K, seed=50 + i)) for i in range(3)]
    A, Bt = sets[0][0].clone(), sets[0][1].clone()
    need = sp24.sp24_splitk_workspace_bytes(M, N, K, A.dtype)
    assert need > 0
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    V = torch.empty((M, K // 2), dtype=A.dtype, device="cuda")
    meta = torch.empty((M, K // 8), dtype=torch.uint8, device="cuda")
    D = torch.empty((M, N), dtype=out, device="cuda")

    def path():
        sp24.sp24_compress(A, layout="tiled", out=(V, meta))
        sp24.sp24_spmm_splitk(V, meta, Bt, out, layout="tiled", workspace=ws, out=D)

    path()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            path()
    torch.cuda.synchronize()
    for a, b in sets[1:] + sets[:1]:
        A.copy_(a)
        Bt.copy_(b)
        path()
        torch.cuda.synchronize()
        want = D.clone()
        D.zero_()
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(D.view(torch.uint8), want.view(torch.uint8))
