"""sp24 oracle -- TEST INFRASTRUCTURE ONLY (never part of the product path).

Thin ctypes access to ``sp24_oracle.c``: a plain scalar CPU statement of
prune / compress / decompress / product for 2:4 structured sparsity, written
from the paper (Sec. 3.1, Sec. 3.2, Sec. 4.1 Step 2).  Only tests, the smoke
check and the benchmark's cpu_baseline leg may import this package; it shares
nothing with the GPU library and does not import it.

Arrays are numpy: 16-bit floats travel as ``uint16`` bit patterns, int8 as
``int8``.  ``dtype`` is one of "f16", "bf16", "i8", "f8" (the 8-bit float with 4 exponent
and 3 fraction bits, as ``uint8`` bit patterns).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sp24_oracle.c")
_LIB = os.path.join(_HERE, "libsp24_oracle.so")
_TYPES = {"f16": 0, "bf16": 1, "i8": 2, "f8": 3}
_lib = None
_decode_tables = {}


def build(force=False):
    """Compile the C oracle with gcc (OpenMP over rows of the product only)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-std=c11", "-ffp-contract=off", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_long, ctypes.c_int
        lib.sp24o_prune.argtypes = [vp, vp, i64, i64, i32]
        lib.sp24o_compress.argtypes = [vp, vp, vp, i64, i64, i32]
        lib.sp24o_decompress.argtypes = [vp, vp, vp, i64, i64, i32]
        lib.sp24o_gemm_f64.argtypes = [vp, vp, vp, i64, i64, i64, i32]
        lib.sp24o_gemm_i32.argtypes = [vp, vp, vp, i64, i64, i64]
        lib.sp24o_conv2d_f64.argtypes = [vp, vp, vp] + [i64] * 11 + [i32]
        lib.sp24o_conv2d_i32.argtypes = [vp, vp, vp] + [i64] * 11
        lib.sp24o_prune_transposable.argtypes = [vp, vp, i64, i64, i32]
        lib.sp24o_mask_apply.argtypes = [vp, vp, vp, i64, i64, i32]
        lib.sp24o_compress_masked.argtypes = [vp, vp, vp, i64, i64, i32]
        lib.sp24o_permute_columns.argtypes = [vp, vp, vp, i64, i64, i32]
        lib.sp24o_permute_rows.argtypes = [vp, vp, vp, i64, i64, i32]
        lib.sp24o_retained_magnitude.argtypes = [vp, vp, i64, i64, i32, vp]
        lib.sp24o_permute_search.argtypes = [vp, vp, i64, i64, i32, i32]
        f32 = ctypes.c_float
        lib.sp24o_dequant_f64.argtypes = [vp, vp, i64, i64, vp, f32, vp, i32]
        lib.sp24o_requant_i8.argtypes = [vp, vp, i64, i64, vp, f32, vp, i32, f32]
        lib.sp24o_f16_to_double.argtypes = [ctypes.c_uint16]
        lib.sp24o_f16_to_double.restype = ctypes.c_double
        lib.sp24o_bf16_to_double.argtypes = [ctypes.c_uint16]
        lib.sp24o_bf16_to_double.restype = ctypes.c_double
        lib.sp24o_f8_to_double.argtypes = [ctypes.c_uint8]
        lib.sp24o_f8_to_double.restype = ctypes.c_double
        _lib = lib
    return _lib


def _np_dtype(dtype):
    return np.int8 if dtype == "i8" else np.uint8 if dtype == "f8" else np.uint16


def _check(a, dtype, ndim=2):
    if a.dtype != _np_dtype(dtype) or a.ndim != ndim or not a.flags.c_contiguous:
        raise ValueError(f"expected C-contiguous {ndim}-d {_np_dtype(dtype).__name__} array")


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def prune(A, dtype):
    """Sec. 4.1 Step 2: zero the two smallest-magnitude entries of every group of 4."""
    _check(A, dtype)
    M, K = A.shape
    P = np.empty_like(A)
    rc = _load().sp24o_prune(_ptr(A), _ptr(P), M, K, _TYPES[dtype])
    if rc:
        raise ValueError(f"oracle prune failed ({rc}): K must be a multiple of 4")
    return P


def compress(A, dtype):
    """Sec. 3.1: (V [M,K/2], meta [M,K/8] uint8) in the canonical packing."""
    _check(A, dtype)
    M, K = A.shape
    if K % 8:
        raise ValueError("K must be a multiple of 8")
    V = np.empty((M, K // 2), dtype=A.dtype)
    meta = np.empty((M, K // 8), dtype=np.uint8)
    rc = _load().sp24o_compress(_ptr(A), _ptr(V), _ptr(meta), M, K, _TYPES[dtype])
    if rc:
        raise ValueError(f"oracle compress failed ({rc})")
    return V, meta


def decompress(V, meta, dtype):
    """Inverse of compress: scatter the kept values, +0 elsewhere."""
    _check(V, dtype)
    M, K2 = V.shape
    K = 2 * K2
    if meta.dtype != np.uint8 or meta.shape != (M, K // 8) or not meta.flags.c_contiguous:
        raise ValueError("meta must be C-contiguous uint8 [M, K/8]")
    P = np.empty((M, K), dtype=V.dtype)
    rc = _load().sp24o_decompress(_ptr(V), _ptr(meta), _ptr(P), M, K, _TYPES[dtype])
    if rc:
        raise ValueError(f"oracle decompress failed ({rc}): illegal metadata code")
    return P


def prune_transposable(A, dtype):
    """Sec. 6: a 2:4 pattern along rows and along columns -- per aligned 4x4 block the pattern with two kept entries
    in every row and column that retains the most magnitude (exhaustive search; ties to the first pattern)."""
    _check(A, dtype)
    P = np.empty_like(A)
    rc = _load().sp24o_prune_transposable(_ptr(A), _ptr(P), A.shape[0], A.shape[1], _TYPES[dtype])
    if rc:
        raise ValueError("oracle prune_transposable: M and K must be multiples of 4")
    return P


def _check_meta(W, meta):
    M, K = W.shape
    if meta.dtype != np.uint8 or meta.shape != (M, K // 8) or not meta.flags.c_contiguous:
        raise ValueError("meta must be C-contiguous uint8 [M, K/8]")


def mask_apply(W, meta, dtype):
    """Sec. 4.1 Step 3: W with every position that the metadata does not record set to +0."""
    _check(W, dtype)
    _check_meta(W, meta)
    P = np.empty_like(W)
    rc = _load().sp24o_mask_apply(_ptr(W), _ptr(meta), _ptr(P), W.shape[0], W.shape[1], _TYPES[dtype])
    if rc:
        raise ValueError(f"oracle mask_apply failed ({rc})")
    return P


def compress_masked(W, meta, dtype):
    """The compressed values of W at the positions the metadata records (no new selection)."""
    _check(W, dtype)
    _check_meta(W, meta)
    V = np.empty((W.shape[0], W.shape[1] // 2), dtype=W.dtype)
    rc = _load().sp24o_compress_masked(_ptr(W), _ptr(meta), _ptr(V), W.shape[0], W.shape[1], _TYPES[dtype])
    if rc:
        raise ValueError(f"oracle compress_masked failed ({rc})")
    return V


def permute_columns(A, perm, dtype):
    """Sec. 4.1 Step 2 (channel permutations): the matrix with its columns in the order perm, P[:, k] = A[:, perm[k]]."""
    _check(A, dtype)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    if perm.shape != (A.shape[1],):
        raise ValueError("perm must hold K entries")
    P = np.empty_like(A)
    rc = _load().sp24o_permute_columns(_ptr(A), _ptr(perm), _ptr(P), A.shape[0], A.shape[1], _TYPES[dtype])
    if rc:
        raise ValueError(f"oracle permute_columns: perm is not a permutation of 0..K-1 ({rc})")
    return P


def permute_rows(A, perm, dtype):
    """Sec. 4.1 Step 2, the producing layer's side: the matrix with its rows in the order perm, P[m] = A[perm[m]]."""
    _check(A, dtype)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    if perm.shape != (A.shape[0],):
        raise ValueError("perm must hold M entries")
    P = np.empty_like(A)
    rc = _load().sp24o_permute_rows(_ptr(A), _ptr(perm), _ptr(P), A.shape[0], A.shape[1], _TYPES[dtype])
    if rc:
        raise ValueError(f"oracle permute_rows: perm is not a permutation of 0..M-1 ({rc})")
    return P


def retained_magnitude(A, dtype, perm=None):
    """Fig. 6: the total magnitude that 2:4 pruning keeps when the groups of four are taken in the column order perm."""
    _check(A, dtype)
    out = np.zeros(1, dtype=np.float64)
    if perm is not None:
        perm = np.ascontiguousarray(perm, dtype=np.int32)
        if perm.shape != (A.shape[1],):
            raise ValueError("perm must hold K entries")
    rc = _load().sp24o_retained_magnitude(_ptr(A), _ptr(perm) if perm is not None else None, A.shape[0], A.shape[1],
                                          _TYPES[dtype], _ptr(out))
    if rc:
        raise ValueError(f"oracle retained_magnitude failed ({rc})")
    return float(out[0])


def permute_search(A, dtype, sweeps=1, perm=None):
    """Sec. 4.1 Step 2 (the search the paper defers): a column order, found by a bounded pairwise exchange between
    groups of four starting from perm (default: the columns as they are), under which 2:4 pruning keeps at least as
    much magnitude.  Returns the new order (int32 [K])."""
    _check(A, dtype)
    K = A.shape[1]
    perm = np.arange(K, dtype=np.int32) if perm is None else np.array(perm, dtype=np.int32)
    if perm.shape != (K,):
        raise ValueError("perm must hold K entries")
    rc = _load().sp24o_permute_search(_ptr(A), _ptr(perm), A.shape[0], K, _TYPES[dtype], int(sweeps))
    if rc:
        raise ValueError(f"oracle permute_search failed ({rc})")
    return perm


def gemm(P, B, dtype):
    """Sec. 3.2 / Fig. 2 by definition: D = P @ B with B [K,N] row-major.

    Returns float64 [M,N] for f16/bf16 (exact conversion, double accumulation)
    and int32 for i8.
    """
    _check(P, dtype)
    _check(B, dtype)
    M, K = P.shape
    K2, N = B.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    lib = _load()
    if dtype == "i8":
        D = np.empty((M, N), dtype=np.int32)
        lib.sp24o_gemm_i32(_ptr(P), _ptr(B), _ptr(D), M, N, K)
    else:
        D = np.empty((M, N), dtype=np.float64)
        lib.sp24o_gemm_f64(_ptr(P), _ptr(B), _ptr(D), M, N, K, _TYPES[dtype])
    return D


def conv2d(P, X, dtype, R, S, pad=(0, 0), stride=(1, 1)):
    """Convolution of the NHWC input X [n_img,H,W,C] with the filter bank P [M, R*S*C] (column
    k = (r*S + s)*C + c; Sec. 4.2: inner dimension C x R x S), written out directly with zero padding.
    Returns [M, n_img*OH*OW]: float64 for f16/bf16, int32 for i8."""
    _check(P, dtype)
    if X.ndim != 4 or not X.flags.c_contiguous or X.dtype != P.dtype:
        raise ValueError("X must be a C-contiguous [n_img,H,W,C] array of the filter's storage type")
    n_img, H, W, C = X.shape
    M, K = P.shape
    if K != R * S * C:
        raise ValueError("filter columns must number R*S*C")
    (ph, pw), (sh, sw) = pad, stride
    OH, OW = (H + 2 * ph - R) // sh + 1, (W + 2 * pw - S) // sw + 1
    lib = _load()
    geom = (M, n_img, H, W, C, R, S, ph, pw, sh, sw)
    if dtype == "i8":
        D = np.empty((M, n_img * OH * OW), dtype=np.int32)
        rc = lib.sp24o_conv2d_i32(_ptr(P), _ptr(X), _ptr(D), *geom)
    else:
        D = np.empty((M, n_img * OH * OW), dtype=np.float64)
        rc = lib.sp24o_conv2d_f64(_ptr(P), _ptr(X), _ptr(D), *geom, _TYPES[dtype])
    if rc:
        raise ValueError("oracle conv2d: illegal geometry")
    return D


def _scales(acc, w_scale, bias):
    if acc.dtype != np.int32 or acc.ndim != 2 or not acc.flags.c_contiguous:
        raise ValueError("acc must be a C-contiguous int32 matrix")
    w = np.ascontiguousarray(w_scale, dtype=np.float32)
    if w.shape != (acc.shape[0],):
        raise ValueError("one weight scale per row")
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    if b is not None and b.shape != w.shape:
        raise ValueError("one bias per row")
    return w, b


def dequant(acc, w_scale, x_scale, bias=None, relu=False):
    """Epilogue of the quantised path in double: acc * (w_scale[m] * x_scale) + bias[m], optional ReLU (Sec. 5:
    per-row weight scales, per-tensor activation scale)."""
    w, b = _scales(acc, w_scale, bias)
    Y = np.empty(acc.shape, dtype=np.float64)
    _load().sp24o_dequant_f64(_ptr(acc), _ptr(Y), acc.shape[0], acc.shape[1], _ptr(w), float(np.float32(x_scale)),
                              None if b is None else _ptr(b), int(bool(relu)))
    return Y


def requant(acc, w_scale, x_scale, inv_y_scale, bias=None, relu=False):
    """The same epilogue re-quantised to int8 with a per-tensor output scale, the rounding decision taken in
    binary32 (one product for the scale, one fused multiply-add, one product, round half to even, clamp)."""
    w, b = _scales(acc, w_scale, bias)
    Q = np.empty(acc.shape, dtype=np.int8)
    _load().sp24o_requant_i8(_ptr(acc), _ptr(Q), acc.shape[0], acc.shape[1], _ptr(w), float(np.float32(x_scale)),
                             None if b is None else _ptr(b), int(bool(relu)), float(np.float32(inv_y_scale)))
    return Q


def spmm(V, meta, B, dtype):
    """The sparse product as the paper defines it: the dense product of the
    decompressed first operand (Fig. 2)."""
    return gemm(decompress(V, meta, dtype), B, dtype)


def to_double(bits, dtype):
    """Exact value of 16-bit patterns (or int8) as float64, element by element."""
    if dtype == "i8":
        return bits.astype(np.float64)
    if dtype == "f8":
        if dtype not in _decode_tables:
            _decode_tables[dtype] = np.array([_load().sp24o_f8_to_double(b) for b in range(256)], dtype=np.float64)
        return _decode_tables[dtype][np.asarray(bits, dtype=np.uint8)]
    if dtype not in _decode_tables:   # the C decoder applied once to each of the 65536 patterns
        fn = _load().sp24o_f16_to_double if dtype == "f16" else _load().sp24o_bf16_to_double
        _decode_tables[dtype] = np.array([fn(b) for b in range(65536)], dtype=np.float64)
    return _decode_tables[dtype][np.asarray(bits, dtype=np.uint16)]


def threads():
    return int(_load().sp24o_threads())


def set_threads(n):
    """Use n OpenMP threads from now on; returns the previous count."""
    return int(_load().sp24o_set_threads(int(n)))
