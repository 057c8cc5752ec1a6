"""The Python binding refuses what the C ABI cannot see: a result tensor of the wrong shape or type, metadata of the
wrong size, operands of different types, a compressed array that is not contiguous.  (The ABI takes raw pointers and
leading dimensions; a smaller tensor behind the pointer would be written past its end.)"""
import pytest
import torch

from paper_2104_08378_amd import sp24

pytestmark = pytest.mark.gpu


def _operands(M=64, K=128, N=64, dt=torch.float16):
    g = torch.Generator(device="cuda").manual_seed(5)
    A = torch.randn((M, K), device="cuda", generator=g).to(dt)
    B = torch.randn((N, K), device="cuda", generator=g).to(dt)
    V, meta = sp24.sp24_compress(A)
    return A, B, V, meta


def test_result_tensor_must_match():
    A, B, V, meta = _operands()
    good = torch.empty((64, 64), dtype=torch.float32, device="cuda")
    sp24.sp24_spmm(V, meta, B, torch.float32, out=good)
    wide = torch.empty((64, 96), dtype=torch.float32, device="cuda")
    sp24.sp24_spmm(V, meta, B, torch.float32, out=wide[:, :64])          # a view with a longer row stride is fine
    for bad in (torch.empty((32, 64), dtype=torch.float32, device="cuda"), torch.empty((64, 32), dtype=torch.float32, device="cuda"),
                torch.empty((64, 64), dtype=torch.float16, device="cuda")):
        with pytest.raises(ValueError):
            sp24.sp24_spmm(V, meta, B, torch.float32, out=bad)
        with pytest.raises(ValueError):
            sp24.sp24_gemm_dense(A, B, torch.float32, out=bad)
        with pytest.raises(ValueError):
            sp24.sp24_spmm_splitk(V, meta, B, torch.float32, out=bad)
    for fn in (sp24.sp24_prune, sp24.sp24_prune_transposable):
        with pytest.raises(ValueError):
            fn(A, out=torch.empty((32, 128), dtype=A.dtype, device="cuda"))
    with pytest.raises(ValueError):
        sp24.sp24_decompress(V, meta, out=torch.empty((64, 64), dtype=A.dtype, device="cuda"))
    with pytest.raises(ValueError):
        sp24.sp24_mask_apply(A, meta, out=torch.empty((64, 64), dtype=A.dtype, device="cuda"))


def test_compressed_pair_and_types_must_match():
    A, B, V, meta = _operands()
    with pytest.raises(ValueError):
        sp24.sp24_spmm(V, meta[:32], B, torch.float32)                     # too little metadata
    with pytest.raises(ValueError):
        sp24.sp24_decompress(V, meta[:, ::2])                             # not contiguous
    with pytest.raises(ValueError):
        sp24.sp24_spmm(V[:, ::2], meta, B[:, :64], torch.float32)         # V not contiguous
    with pytest.raises(ValueError):
        sp24.sp24_spmm(V, meta, B.to(torch.bfloat16), torch.float32)      # B of another type
    with pytest.raises(ValueError):
        sp24.sp24_gemm_dense(A, B.to(torch.int8), torch.float32)
    with pytest.raises(ValueError):
        sp24.sp24_mask_apply(A, meta[:8])
    with pytest.raises(ValueError):
        sp24.sp24_compress_masked(A, meta, out=torch.empty((64, 32), dtype=A.dtype, device="cuda"))
    with pytest.raises(ValueError):
        sp24.sp24_compress(A, out=(torch.empty((64, 64), dtype=A.dtype, device="cuda"), meta[:8]))
