"""GPU parity of the quantised path's fused epilogue (int8 products with per-row weight scale, per-tensor
activation scale, bias, ReLU): int8 output bit-exact against the oracle's binary32 re-quantisation of the exact
int32 product; floating outputs against the oracle's double evaluation, within the rounding of the binary32
epilogue (3 ulp of the largest term) plus one rounding to the output type."""
import numpy as np
import pytest
import torch

import oracle
from paper_2104_08378_amd import sp24, synth
from util import OUT_DT, out_to_f64, to_gpu

pytestmark = pytest.mark.gpu

CASES = [
    # M, N, K, layout                     -- kernel that serves it
    (45, 70, 96, "canonical"),            # 128x128 tile, ragged both ways, fewer rows than a tile
    (64, 200, 128, "tiled"),
    (8, 300, 128, "canonical"),           # fewer rows than a row block
    (11136, 24, 128, "tiled"),            # N <= 32 on the tiled kernels (many rows)
    (128, 16, 2112, "tiled"),             # skinny (N <= 32)
    (320, 300, 256, "tiled"),             # 128x128 tiles, ragged N
    (4096, 3328, 256, "tiled"),           # 256x256 tiles, eight wavefronts
]


def make(M, N, K, seed):
    A, Bt = synth.make("square_i8", M=M, N=N, K=K, seed=seed)
    rng = np.random.default_rng([seed, 5])
    w_scale = rng.uniform(4e-4, 2e-3, size=M).astype(np.float32)
    bias = rng.normal(0.0, 0.5, size=M).astype(np.float32)
    return A, Bt, w_scale, bias, np.float32(0.021)


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("sparse", [True, False])
def test_int8_output_is_bit_exact(case, sparse):
    M, N, K, layout = case
    A, Bt, w_scale, bias, x_scale = make(M, N, K, 3)
    Pn = oracle.prune(A, "i8")
    acc = oracle.gemm(Pn, np.ascontiguousarray(Bt.T), "i8")
    ws, bs = torch.from_numpy(w_scale).cuda(), torch.from_numpy(bias).cuda()
    Bd = to_gpu(Bt, "i8")
    for use_bias, relu, inv_y in [(True, False, 11.0), (False, True, 29.5), (True, True, 70.0)]:
        b_np, b_t = (bias, bs) if use_bias else (None, None)
        if sparse:
            V, meta = sp24.sp24_compress(to_gpu(A, "i8"), layout=layout)
            D = sp24.sp24_spmm_i8_scaled(V, meta, Bd, torch.int8, ws, x_scale, b_t, relu, inv_y, layout=layout)
        else:
            D = sp24.sp24_gemm_dense_i8_scaled(to_gpu(Pn, "i8"), Bd, torch.int8, ws, x_scale, b_t, relu, inv_y)
        torch.cuda.synchronize()
        want = oracle.requant(acc, w_scale, x_scale, inv_y, b_np, relu)
        got = D.cpu().numpy()
        assert np.array_equal(got, want), (case, sparse, use_bias, relu, inv_y, int((got != want).sum()))
        assert got.min() == -128 or relu or inv_y < 20          # the larger output scales saturate
        assert len(np.unique(got)) > 20


@pytest.mark.parametrize("sparse", [True, False])
def test_int8_output_from_the_general_kernel_is_bit_exact(sparse):
    """Rows of B that are not 16-byte aligned (a view with a leading dimension of K + 4): the general kernel."""
    M, N, K = 45, 70, 96
    A, Bt, w_scale, bias, x_scale = make(M, N, K, 6)
    Pn = oracle.prune(A, "i8")
    acc = oracle.gemm(Pn, np.ascontiguousarray(Bt.T), "i8")
    ws, bs = torch.from_numpy(w_scale).cuda(), torch.from_numpy(bias).cuda()
    wide = torch.zeros((N, K + 4), dtype=torch.int8, device="cuda")
    wide[:, :K] = to_gpu(Bt, "i8")
    Bd = wide[:, :K]
    if sparse:
        V, meta = sp24.sp24_compress(to_gpu(A, "i8"))
        D = sp24.sp24_spmm_i8_scaled(V, meta, Bd, torch.int8, ws, x_scale, bs, True, 29.5)
    else:
        D = sp24.sp24_gemm_dense_i8_scaled(to_gpu(Pn, "i8"), Bd, torch.int8, ws, x_scale, bs, True, 29.5)
    torch.cuda.synchronize()
    assert np.array_equal(D.cpu().numpy(), oracle.requant(acc, w_scale, x_scale, 29.5, bias, True))


@pytest.mark.parametrize("case", CASES[:6])
@pytest.mark.parametrize("out", ["f32", "f16", "bf16"])
def test_float_outputs_match_the_double_epilogue(case, out):
    M, N, K, layout = case
    A, Bt, w_scale, bias, x_scale = make(M, N, K, 4)
    Pn = oracle.prune(A, "i8")
    acc = oracle.gemm(Pn, np.ascontiguousarray(Bt.T), "i8")
    ws, bs = torch.from_numpy(w_scale).cuda(), torch.from_numpy(bias).cuda()
    V, meta = sp24.sp24_compress(to_gpu(A, "i8"), layout=layout)
    Bd = to_gpu(Bt, "i8")
    rel_out = {"f32": 0.0, "f16": 2.0 ** -11, "bf16": 2.0 ** -8}[out]
    for relu in (False, True):
        ref = oracle.dequant(acc, w_scale, x_scale, bias, relu)
        # |y error| <= 3 * 2^-24 * (|acc| s + |bias|) from the binary32 scale product, conversion and fused multiply-add
        terms = np.abs(acc) * (w_scale.astype(np.float64) * float(x_scale))[:, None] + np.abs(bias.astype(np.float64))[:, None]
        bound = 3 * 2.0 ** -24 * terms + rel_out * (np.abs(ref) + 3 * 2.0 ** -24 * terms) + 1e-30
        for D in (sp24.sp24_spmm_i8_scaled(V, meta, Bd, OUT_DT[out], ws, x_scale, bs, relu, layout=layout),
                  sp24.sp24_gemm_dense_i8_scaled(to_gpu(Pn, "i8"), Bd, OUT_DT[out], ws, x_scale, bs, relu)):
            torch.cuda.synchronize()
            err = np.abs(out_to_f64(D) - ref)
            assert (err <= bound).all(), (case, out, relu, float((err / bound).max()))


def test_unit_scales_reproduce_the_clamped_integer_product():
    M, N, K = 64, 96, 64
    rng = np.random.default_rng(9)
    A = rng.integers(-3, 4, size=(M, K), dtype=np.int8)
    Bt = rng.integers(-3, 4, size=(N, K), dtype=np.int8)
    V, meta = sp24.sp24_compress(to_gpu(A, "i8"))
    ones = torch.ones(M, dtype=torch.float32, device="cuda")
    D8 = sp24.sp24_spmm_i8_scaled(V, meta, to_gpu(Bt, "i8"), torch.int8, ones, 1.0)
    D32 = sp24.sp24_spmm(V, meta, to_gpu(Bt, "i8"), torch.int32)
    torch.cuda.synchronize()
    assert torch.equal(D8.to(torch.int32), D32.clamp(-128, 127))


@pytest.mark.parametrize("geom", [
    # M, n_img, H, W, C, R, S, pad, stride, layout
    (33, 3, 5, 5, 32, 3, 3, (1, 1), (1, 1), "canonical"),      # general kernel
    (256, 4, 10, 10, 128, 3, 3, (1, 1), (1, 1), "tiled"),      # tiled kernel, implicit gather
    (128, 2, 9, 9, 128, 3, 3, (0, 1), (2, 1), "tiled"),
])
def test_quantised_convolution_int8_output_is_bit_exact(geom):
    M, n_img, H, W, C, R, S, pad, stride, layout = geom
    rng = np.random.default_rng([31, M])
    A = rng.integers(-127, 128, size=(M, R * S * C), dtype=np.int8)
    X = rng.integers(-127, 128, size=(n_img, H, W, C), dtype=np.int8)
    w_scale = rng.uniform(4e-4, 2e-3, size=M).astype(np.float32)          # one per output channel
    bias = rng.normal(0.0, 0.5, size=M).astype(np.float32)
    x_scale, inv_y = np.float32(0.018), 23.0
    Pn = oracle.prune(A, "i8")
    acc = oracle.conv2d(Pn, X, "i8", R, S, pad, stride)
    want = oracle.requant(acc, w_scale, x_scale, inv_y, bias, True)
    ws, bs = torch.from_numpy(w_scale).cuda(), torch.from_numpy(bias).cuda()
    V, meta = sp24.sp24_compress(to_gpu(A, "i8"), layout=layout)
    Xd = to_gpu(X, "i8")
    D = sp24.sp24_spmm_conv2d_i8_scaled(V, meta, Xd, torch.int8, R, S, ws, x_scale, bs, True, inv_y, pad, stride, layout=layout)
    Dd = sp24.sp24_conv2d_dense_i8_scaled(to_gpu(Pn, "i8"), Xd, torch.int8, R, S, ws, x_scale, bs, True, inv_y, pad, stride)
    torch.cuda.synchronize()
    assert np.array_equal(D.cpu().numpy(), want)
    assert np.array_equal(Dd.cpu().numpy(), want)
    ref = oracle.dequant(acc, w_scale, x_scale, bias, True)
    Df = sp24.sp24_spmm_conv2d_i8_scaled(V, meta, Xd, torch.float32, R, S, ws, x_scale, bs, True, 1.0, pad, stride, layout=layout)
    torch.cuda.synchronize()
    assert np.allclose(out_to_f64(Df), ref, rtol=1e-6, atol=1e-5)
