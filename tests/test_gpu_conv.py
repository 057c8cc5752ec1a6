"""GPU parity of the implicit-GEMM convolution entry points against the CPU oracle's direct convolution
(same bar as the products: int8 bit-exact, floating point within max relative error 1e-2 of the fp64 result)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2104_08378_amd import sp24, synth
from util import OUT_DT, out_to_f64, to_gpu

pytestmark = pytest.mark.gpu
REL_TOL = 1e-2


def rel_err(got, ref):
    floor = 1e-3 * np.sqrt(np.mean(ref * ref)) + 1e-300
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor)))


def make_inputs(dtype, M, n_img, H, W, C, K, seed):
    rng = np.random.default_rng([seed, 77])
    if dtype == "i8":
        A = rng.integers(-127, 128, size=(M, K), dtype=np.int8)
        X = rng.integers(-127, 128, size=(n_img, H, W, C), dtype=np.int8)
    else:
        A = synth.to_bits(rng.standard_normal((M, K)) * 0.05, dtype)
        X = synth.to_bits(np.maximum(rng.standard_normal((n_img, H, W, C)), 0.0), dtype)   # ReLU activations
    return A, X


CASES = [
    # dtype, out, M, n_img, H, W, C, R, S, pad, stride, layout        -- kernel that serves it
    ("f16", "f32", 40, 2, 6, 5, 16, 3, 3, (1, 1), (1, 1), "canonical"),     # general
    ("bf16", "bf16", 64, 1, 7, 9, 32, 3, 2, (0, 1), (2, 1), "tiled"),      # general (N = 27 < 32)
    ("i8", "i32", 33, 3, 5, 5, 32, 3, 3, (1, 1), (1, 1), "canonical"),      # general, ragged M
    ("i8", "i32", 64, 2, 6, 6, 64, 3, 3, (2, 2), (1, 1), "tiled"),          # general (C*1 = 64 bytes < a step), pad > needed
    ("f16", "f16", 128, 3, 12, 12, 64, 3, 3, (1, 1), (1, 1), "tiled"),      # 3x3 patch kernel (sparse), one chunk of channels, ragged N = 432
    ("f16", "f16", 96, 5, 9, 11, 192, 3, 3, (1, 1), (1, 1), "tiled"),       # patch kernel: three chunks, ragged M (three row blocks), N = 495
    ("bf16", "f32", 160, 40, 4, 4, 256, 3, 3, (1, 1), (1, 1), "tiled"),     # patch kernel: four chunks, a tile spans eight images, ragged M
    ("i8", "i32", 128, 3, 16, 8, 384, 3, 3, (0, 1), (1, 1), "tiled"),       # patch kernel: no vertical padding (output images shorter than input), int8, three chunks
    ("i8", "i32", 128, 3, 13, 9, 384, 3, 3, (0, 0), (1, 1), "tiled"),       # no padding at all: a patch may span 222 pixels, the 256-pixel patch kernel
    ("f16", "f16", 128, 1, 56, 56, 64, 3, 3, (1, 1), (1, 1), "tiled"),      # 56 pixels wide: patches of 242 pixels (the 256-pixel kernel), ragged N = 3136
    ("bf16", "f32", 96, 2, 36, 20, 256, 3, 3, (1, 1), (1, 1), "tiled"),     # 20 wide and 36 tall, patches of 170 pixels, four chunks
    ("f16", "f32", 128, 2, 20, 20, 128, 3, 3, (1, 0), (1, 1), "tiled"),     # patch kernel: padding on one axis only, two chunks, output rows shorter than input, patch of up to 186 pixels
    ("f16", "f16", 32, 2, 12, 12, 128, 3, 3, (1, 1), (1, 1), "tiled"),      # patch kernel with a single row block of filters
    ("bf16", "f32", 24, 2, 10, 10, 64, 3, 3, (1, 1), (1, 1), "canonical"),  # fewer filters than a row block: the tiled kernel
    ("bf16", "bf16", 256, 1, 24, 24, 320, 3, 3, (1, 1), (1, 1), "tiled"),   # patch kernel: five chunks, one image larger than a tile
    ("f16", "f16", 128, 2, 30, 30, 64, 3, 3, (0, 0), (1, 1), "tiled"),      # 3x3 but a patch would span 260 pixels: the general tiled kernel
    ("f16", "f16", 256, 300, 8, 8, 64, 3, 3, (1, 1), (1, 1), "tiled"),      # patch kernel, 300 tiles: more workgroups than compute units, two on some
    ("bf16", "f32", 192, 2, 11, 13, 128, 2, 3, (1, 0), (2, 1), "tiled"),    # tiled, two steps per tap, strides, ragged N = 132
    ("i8", "i32", 256, 4, 10, 10, 128, 3, 3, (1, 1), (1, 1), "tiled"),      # patch kernel int8, one chunk (dense: tiled, 9 steps)
    ("f16", "f32", 128, 2, 8, 8, 256, 1, 1, (0, 0), (1, 1), "tiled"),       # pointwise: the plain product's kernels (N = 128: tiled)
    ("i8", "i32", 64, 1, 4, 4, 256, 1, 1, (0, 0), (1, 1), "tiled"),         # pointwise on 16 pixels: the streaming kernel
    ("bf16", "bf16", 256, 8, 16, 16, 512, 1, 1, (0, 0), (1, 1), "canonical"),  # pointwise, 2048 pixels, canonical layout
    ("f16", "f16", 128, 2, 9, 9, 128, 1, 1, (0, 0), (2, 2), "tiled"),       # 1x1 with stride 2: still a gather
    ("bf16", "bf16", 64, 5, 9, 7, 64, 5, 3, (2, 1), (3, 2), "tiled"),       # 5x3 filter, stride 3x2
    ("f16", "f16", 2048, 64, 10, 10, 64, 3, 3, (1, 1), (1, 1), "tiled"),    # sparse: 16 x 50 tiles through the 3x3 kernel; dense: 8 x 25 tiles of 256x256
    ("f16", "f16", 2048, 64, 20, 20, 64, 3, 3, (1, 1), (2, 2), "tiled"),    # stride 2: 8 x 25 tiles of 256x256 (eight-wavefront shape), sparse and dense
]


def run_case(dtype, out, M, n_img, H, W, C, R, S, pad, stride, layout, sparse, seed):
    K = R * S * C
    A, X = make_inputs(dtype, M, n_img, H, W, C, K, seed)
    Pn = oracle.prune(A, dtype)
    ref = oracle.conv2d(Pn, X, dtype, R, S, pad, stride)
    Xd = to_gpu(X, dtype)
    if sparse:
        V, meta = sp24.sp24_compress(to_gpu(A, dtype), layout=layout)
        D = sp24.sp24_spmm_conv2d(V, meta, Xd, OUT_DT[out], R, S, pad, stride, layout=layout)
    else:
        D = sp24.sp24_conv2d_dense(to_gpu(Pn, dtype), Xd, OUT_DT[out], R, S, pad, stride)
    torch.cuda.synchronize()
    assert tuple(D.shape) == ref.shape
    if dtype == "i8":
        assert np.array_equal(D.cpu().numpy(), ref), (dtype, M, n_img, H, W, C, R, S, pad, stride, layout, sparse)
    else:
        e = rel_err(out_to_f64(D), ref)
        assert e <= REL_TOL, (dtype, out, M, n_img, H, W, C, R, S, pad, stride, layout, sparse, e)


@pytest.mark.parametrize("case", CASES)
def test_sparse_convolution_matches_oracle(case):
    run_case(*case, sparse=True, seed=1)


@pytest.mark.parametrize("case", CASES)
def test_dense_convolution_matches_oracle(case):
    run_case(*case, sparse=False, seed=2)


def test_convolution_equals_product_with_materialised_im2col():
    # the workload's own recipe: both routes through the library give the same fp16 bits where the K order agrees
    A, Bt = synth.make("conv3x3_f16", M=128, N=196 * 3, K=9 * 64)
    X = synth.conv_activations(0, 3, 64)
    V, meta = sp24.sp24_compress(to_gpu(A, "f16"), layout="tiled")
    d1 = sp24.sp24_spmm_conv2d(V, meta, to_gpu(X, "f16"), torch.float32, 3, 3, (1, 1), (1, 1), layout="tiled")
    d2 = sp24.sp24_spmm(V, meta, to_gpu(Bt, "f16"), torch.float32, layout="tiled")
    torch.cuda.synchronize()
    assert torch.equal(d1, d2)


def test_empty_convolution():
    V = torch.empty((0, 72), dtype=torch.float16, device="cuda")
    meta = torch.empty((0, 18), dtype=torch.uint8, device="cuda")
    X = torch.zeros((2, 4, 4, 16), dtype=torch.float16, device="cuda")
    D = sp24.sp24_spmm_conv2d(V, meta, X, torch.float32, 3, 3, (1, 1), (1, 1))
    assert tuple(D.shape) == (0, 32)
