"""Seeded synthetic inputs shared by the tests, the smoke check and bench.py.

Holds no part of the 2:4 method (no pruning, packing or products): only random
draws, one rounding to the storage type, and the im2col gather that shapes the
convolution workload.  16-bit floats are returned as ``uint16`` bit patterns,
int8 as ``int8``.  The five workloads mirror transformer and CNN layer shapes
(Sec. 3.2: N = batch x sequence; Sec. 4.2: conv inner dimension C*R*S).
"""
import numpy as np

WORKLOADS = {
    # name: dtype, M, K, N, out dtype
    "tiny_f16": dict(id=1, dtype="f16", M=256, K=256, N=256, out="f32"),
    "ffn_bf16": dict(id=2, dtype="bf16", M=4096, K=1024, N=8192, out="bf16"),
    "conv3x3_f16": dict(id=3, dtype="f16", M=256, K=2304, N=12544, out="f16"),
    "square_i8": dict(id=4, dtype="i8", M=8192, K=8192, N=8192, out="i32"),
    "skinny_bf16": dict(id=5, dtype="bf16", M=8192, K=8192, N=16, out="bf16"),
}


def f64_to_f16_bits(x):
    """Round-to-nearest-even to IEEE binary16, returned as uint16 bits."""
    return np.asarray(x, dtype=np.float64).astype(np.float16).view(np.uint16)


def f64_to_bf16_bits(x):
    """Round-to-nearest-even to bfloat16 via the binary32 bit pattern."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    out = rounded.astype(np.uint16)
    nan = np.isnan(f)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def f64_to_f8_bits(x):
    """Round-to-nearest-even to the 8-bit float with 4 exponent bits (bias 7) and 3 fraction bits (no infinities,
    largest finite value 448); values beyond it saturate to +-448, NaN becomes the one NaN pattern.  uint8 bits."""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(np.where(np.isnan(x), 0.0, x)), 448.0)
    e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.clip(e, -6, 8)                                  # exponent of the binade the value is rounded in
    q = np.rint(a / np.exp2(e - 3))                        # in units of the binade's spacing; rint rounds half to even
    v = np.minimum(q * np.exp2(e - 3), 448.0)              # q = 16 moves up one binade by itself
    e2 = np.clip(np.floor(np.log2(np.where(v > 0, v, 1.0))), -6, 8)
    normal = v >= 2.0 ** -6
    frac = np.where(normal, np.rint((v / np.exp2(e2) - 1.0) * 8.0), np.rint(v * 512.0)).astype(np.uint8)
    expo = np.where(normal, e2 + 7, 0).astype(np.uint8)
    bits = (expo << 3) | frac
    bits = np.where(np.signbit(x), bits | 0x80, bits).astype(np.uint8)
    return np.where(np.isnan(x), np.uint8(0x7F), bits).astype(np.uint8)


def to_bits(x, dtype):
    if dtype == "f16":
        return f64_to_f16_bits(x)
    if dtype == "bf16":
        return f64_to_bf16_bits(x)
    if dtype == "f8":
        return f64_to_f8_bits(x)
    raise ValueError(dtype)


def _rng(seed, config_id, tensor_id):
    return np.random.default_rng([seed, config_id, tensor_id])


def normal_bits(shape, sigma, dtype, seed, config_id, tensor_id):
    return to_bits(_rng(seed, config_id, tensor_id).standard_normal(shape) * sigma, dtype)


def int8_uniform(shape, seed, config_id, tensor_id):
    return _rng(seed, config_id, tensor_id).integers(-127, 128, size=shape, dtype=np.int8)


def im2col_nhwc(x, R=3, S=3, pad=1):
    """x: [batch, H, W, C] -> [batch*H*W, R*S*C], k = (r*S + s)*C + c, stride 1."""
    b, H, W, C = x.shape
    xp = np.zeros((b, H + 2 * pad, W + 2 * pad, C), dtype=x.dtype)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    cols = np.empty((b, H, W, R * S, C), dtype=x.dtype)
    for r in range(R):
        for s in range(S):
            cols[:, :, :, r * S + s, :] = xp[:, r:r + H, s:s + W, :]
    return cols.reshape(b * H * W, R * S * C)


def conv_activations(seed=0, n_img=64, C=256):
    """NHWC activations of the conv3x3_f16 workload, [n_img, 14, 14, C] fp16 bits: ReLU of a standard
    normal draw (about half exact zeros)."""
    cid = WORKLOADS["conv3x3_f16"]["id"]
    return f64_to_f16_bits(np.maximum(_rng(seed, cid, 1).standard_normal((n_img, 14, 14, C)), 0.0))


def make(name, seed=0, M=None, N=None, K=None):
    """Return (A [M,K], Bt [N,K]) for a named workload; Bt is the second operand
    stored K-contiguous (one row per token / output pixel).  M, N, K may be
    overridden to cut a smaller problem of the same distribution."""
    w = WORKLOADS[name]
    cid, dt = w["id"], w["dtype"]
    M = w["M"] if M is None else M
    N = w["N"] if N is None else N
    K = w["K"] if K is None else K
    if name == "tiny_f16":
        A = normal_bits((M, K), 1.0, dt, seed, cid, 0)
        Bt = normal_bits((N, K), 1.0, dt, seed, cid, 1)
    elif name in ("ffn_bf16", "skinny_bf16"):
        A = normal_bits((M, K), 0.02, dt, seed, cid, 0)
        Bt = normal_bits((N, K), 1.0, dt, seed, cid, 1)
    elif name == "conv3x3_f16":
        C = K // 9
        if C * 9 != K or N % 196:
            raise ValueError("conv workload needs K = 9*C and N = batch*14*14")
        A = normal_bits((M, K), 0.05, dt, seed, cid, 0)
        Bt = im2col_nhwc(conv_activations(seed, N // 196, C))
    elif name == "square_i8":
        A = int8_uniform((M, K), seed, cid, 0)
        Bt = int8_uniform((N, K), seed, cid, 1)
    else:
        raise KeyError(name)
    return np.ascontiguousarray(A), np.ascontiguousarray(Bt)
