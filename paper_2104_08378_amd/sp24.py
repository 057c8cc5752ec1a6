"""Python binding of libsp24.so: argument marshalling only.

Each function mirrors the C entry point of the same name (``include/sp24.h``):
it checks that the tensors live on the GPU, allocates the outputs with torch,
passes raw device pointers and the current HIP stream, and raises on a non-zero
status.  Every arithmetic step runs in the library's HIP kernels; there is no
fallback: if ``libsp24.so`` is not built the import of the symbols fails loudly.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsp24.so")

F16, BF16, I8, F32, I32, F8 = 0, 1, 2, 3, 4, 5
CANONICAL, TILED = 0, 1
B_KMAJOR, B_NMAJOR = 0, 1

_DT = {torch.float16: F16, torch.bfloat16: BF16, torch.int8: I8, torch.float32: F32, torch.int32: I32, torch.float8_e4m3fn: F8}
_LAYOUT = {"canonical": CANONICAL, "tiled": TILED}
_lib = None


class Sp24Error(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib():
    """Load libsp24.so (built by ``python -m paper_2104_08378_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2104_08378_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.sp24_values_bytes.argtypes = [i64, i64, i32]
        L.sp24_values_bytes.restype = ctypes.c_size_t
        L.sp24_meta_bytes.argtypes = [i64, i64, i32, i32]
        L.sp24_meta_bytes.restype = ctypes.c_size_t
        L.sp24_prune.argtypes = [vp, vp, i64, i64, i64, i64, i32, vp]
        L.sp24_compress.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, vp]
        L.sp24_decompress.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, vp]
        L.sp24_prune_transposable.argtypes = [vp, vp, i64, i64, i64, i64, i32, vp]
        L.sp24_mask_apply.argtypes = [vp, vp, vp, i64, i64, i64, i64, i32, i32, vp]
        L.sp24_compress_masked.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, vp]
        L.sp24_permute_columns.argtypes = [vp, vp, vp, i64, i64, i64, i64, i32, vp]
        L.sp24_permute_rows.argtypes = [vp, vp, vp, i64, i64, i64, i64, i32, vp]
        L.sp24_retained_magnitude.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp]
        L.sp24_permute_search.argtypes = [vp, vp, i64, i64, i64, i32, i32, vp]
        L.sp24_permute_search.restype = i32
        L.sp24_spmm.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i32, i32, i32, i32, vp]
        L.sp24_gemm_dense.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i64, i32, i32, i32, vp]
        L.sp24_splitk_workspace_bytes.argtypes = [i64, i64, i64, i32]
        L.sp24_splitk_workspace_bytes.restype = ctypes.c_size_t
        L.sp24_spmm_splitk.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i32, i32, i32, i32, vp, ctypes.c_size_t, vp]
        L.sp24_spmm_splitk_static.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i32, i32, i32, i32, vp]
        L.sp24_gemm_dense_splitk.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i64, i32, i32, i32, vp, ctypes.c_size_t, vp]
        L.sp24_spmm_conv2d.argtypes = [vp, vp, vp, vp] + [i64] * 5 + [i32] * 6 + [i64, i32, i32, i32, vp]
        L.sp24_conv2d_dense.argtypes = [vp, vp, vp] + [i64] * 5 + [i32] * 6 + [i64, i64, i32, i32, vp]
        f32 = ctypes.c_float
        L.sp24_spmm_i8_scaled.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, vp, f32, vp, i32, f32, i32, i32, i32, vp]
        L.sp24_gemm_dense_i8_scaled.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i64, vp, f32, vp, i32, f32, i32, i32, vp]
        L.sp24_spmm_conv2d_i8_scaled.argtypes = [vp, vp, vp, vp] + [i64] * 5 + [i32] * 6 + [i64, vp, f32, vp, i32, f32, i32, i32, vp]
        L.sp24_conv2d_dense_i8_scaled.argtypes = [vp, vp, vp] + [i64] * 5 + [i32] * 6 + [i64, i64, vp, f32, vp, i32, f32, i32, vp]
        L.sp24_status_string.argtypes = [i32]
        L.sp24_status_string.restype = ctypes.c_char_p
        for name in ("sp24_prune_transposable", "sp24_mask_apply", "sp24_compress_masked", "sp24_prune", "sp24_compress", "sp24_decompress", "sp24_spmm", "sp24_gemm_dense", "sp24_spmm_conv2d",
                     "sp24_conv2d_dense", "sp24_spmm_i8_scaled", "sp24_gemm_dense_i8_scaled",
                     "sp24_spmm_conv2d_i8_scaled", "sp24_conv2d_dense_i8_scaled", "sp24_spmm_splitk", "sp24_gemm_dense_splitk", "sp24_spmm_splitk_static"):
            getattr(L, name).restype = i32
        _lib = L
    return _lib


def status_string(status):
    return lib().sp24_status_string(int(status)).decode()


def sp24_values_bytes(M, K, dtype):
    return lib().sp24_values_bytes(M, K, _DT[dtype])


def sp24_meta_bytes(M, K, dtype, layout="canonical"):
    return lib().sp24_meta_bytes(M, K, _DT[dtype], _LAYOUT[layout])


def _stream():
    """torch's current stream on the current device, as the raw hipStream_t (the two private calls are what
    torch.cuda.current_stream() itself ends in; going through the Stream object costs 3 us a call, a third of the
    time of a small launch)."""
    try:
        return ctypes.c_void_p(torch._C._cuda_getCurrentRawStream(torch._C._cuda_getDevice()))
    except AttributeError:
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, name):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    return t


def _rowmajor(t, name):
    _dev(t, name)
    if t.dim() != 2 or (t.stride(1) != 1 and t.shape[1] > 1):      # (the stride of a dimension of size 1 means nothing)
        raise ValueError(f"{name} must be 2-d with unit column stride")
    return t


def _ld(t):
    """Leading dimension of a row-major matrix in elements; a single row may carry any stride."""
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


def _out(out, shape, dtype, device, name="out"):
    """The result tensor: a new one, or the caller's, which must have exactly the result's shape and type (the C ABI
    sees a pointer and a row stride only, so a smaller tensor would be written past its end)."""
    if out is None:
        return torch.empty(shape, dtype=dtype, device=device)
    _rowmajor(out, name)
    if tuple(out.shape) != tuple(shape) or out.dtype != dtype:
        raise ValueError(f"{name} must be a {tuple(shape)} tensor of {dtype}, got {tuple(out.shape)} of {out.dtype}")
    return out


def _compressed(V, meta):
    """The compressed pair as sp24_compress returns it: V [M, K/2] contiguous, meta M*K/8 contiguous bytes."""
    _dev(V, "V"), _dev(meta, "meta")
    if V.dim() != 2 or not V.is_contiguous():
        raise ValueError("V must be a contiguous 2-d tensor [M, K/2]")
    if V.dtype not in (torch.float16, torch.bfloat16, torch.int8, torch.float8_e4m3fn):
        raise ValueError("V must be float16, bfloat16, int8 or float8_e4m3fn")
    M, K = V.shape[0], V.shape[1] * 2
    _meta_arg(meta, M, K)
    return M, K


def _meta_arg(meta, M, K):
    _dev(meta, "meta")
    if not meta.is_contiguous() or meta.numel() * meta.element_size() != M * (K // 8):
        raise ValueError("meta must be contiguous and hold M*K/8 bytes")


def _same_type(B, ref, name="B"):
    if B.dtype != ref.dtype:
        raise ValueError(f"{name} must have the first operand's type {ref.dtype}, got {B.dtype}")


def _check(status, where):
    if status != 0:
        raise Sp24Error(status, where)


def sp24_prune(A, out=None):
    """P = A with the two smallest-magnitude entries of each group of 4 zeroed; out may be A."""
    _rowmajor(A, "A")
    M, K = A.shape
    P = _out(out, (M, K), A.dtype, A.device)
    _check(lib().sp24_prune(A.data_ptr(), P.data_ptr(), M, K, A.stride(0), P.stride(0), _DT[A.dtype], _stream()),
           "sp24_prune")
    return P


def sp24_compress(A, layout="canonical", out=None):
    """Return (V, meta): V [M, K/2] of A's dtype, meta uint8 [M, K/8] (both flat-permuted for "tiled")."""
    _rowmajor(A, "A")
    M, K = A.shape
    if out is None:
        V = torch.empty((M, K // 2), dtype=A.dtype, device=A.device)
        meta = torch.empty((M, K // 8), dtype=torch.uint8, device=A.device)
    else:
        V, meta = _dev(out[0], "V"), _dev(out[1], "meta")
        if (V.numel() != M * (K // 2) or V.dtype != A.dtype or meta.numel() * meta.element_size() != M * (K // 8)
                or not V.is_contiguous() or not meta.is_contiguous()):
            raise ValueError("out buffers must be contiguous and hold M*K/2 values and M*K/8 metadata bytes")
    _check(lib().sp24_compress(A.data_ptr(), V.data_ptr(), meta.data_ptr(), M, K, A.stride(0), _DT[A.dtype],
                               _LAYOUT[layout], _stream()), "sp24_compress")
    return V, meta


def sp24_decompress(V, meta, layout="canonical", out=None):
    M, K = _compressed(V, meta)
    P = _out(out, (M, K), V.dtype, V.device)
    _check(lib().sp24_decompress(V.data_ptr(), meta.data_ptr(), P.data_ptr(), M, K, P.stride(0), _DT[V.dtype],
                                 _LAYOUT[layout], _stream()), "sp24_decompress")
    return P


def sp24_prune_transposable(A, out=None):
    """2:4 along rows and along columns: per 4x4 block the two-per-row-and-column pattern that keeps the most magnitude."""
    _rowmajor(A, "A")
    M, K = A.shape
    P = _out(out, (M, K), A.dtype, A.device)
    _check(lib().sp24_prune_transposable(A.data_ptr(), P.data_ptr(), M, K, A.stride(0), P.stride(0), _DT[A.dtype], _stream()),
           "sp24_prune_transposable")
    return P


def _perm_arg(perm, K):
    _dev(perm, "perm")
    if perm.dtype != torch.int32 or perm.dim() != 1 or perm.numel() != K or not perm.is_contiguous():
        raise ValueError("perm must be a contiguous int32 device tensor with one entry per column (row)")
    return perm


def sp24_permute_columns(A, perm, out=None):
    """The matrix with its columns in the order perm: out[:, k] = A[:, perm[k]]."""
    _rowmajor(A, "A")
    M, K = A.shape
    _perm_arg(perm, K)
    P = _out(out, (M, K), A.dtype, A.device)
    _check(lib().sp24_permute_columns(A.data_ptr(), perm.data_ptr(), P.data_ptr(), M, K, A.stride(0), P.stride(0), _DT[A.dtype],
                                      _stream()), "sp24_permute_columns")
    return P


def sp24_permute_rows(A, perm, out=None):
    """The matrix with its rows in the order perm: out[m] = A[perm[m]]."""
    _rowmajor(A, "A")
    M, K = A.shape
    _perm_arg(perm, M)
    P = _out(out, (M, K), A.dtype, A.device)
    _check(lib().sp24_permute_rows(A.data_ptr(), perm.data_ptr(), P.data_ptr(), M, K, A.stride(0), P.stride(0), _DT[A.dtype],
                                   _stream()), "sp24_permute_rows")
    return P


def sp24_retained_magnitude(A, perm=None, out=None):
    """Total magnitude that 2:4 pruning keeps with the groups of four formed in the column order perm (a 1-element
    float64 device tensor; no synchronisation)."""
    _rowmajor(A, "A")
    M, K = A.shape
    if perm is not None:
        _perm_arg(perm, K)
    total = torch.empty(1, dtype=torch.float64, device=A.device) if out is None else _dev(out, "out")
    if total.dtype != torch.float64 or total.numel() != 1:
        raise ValueError("out must be one float64")
    _check(lib().sp24_retained_magnitude(A.data_ptr(), perm.data_ptr() if perm is not None else None, total.data_ptr(), M, K,
                                         A.stride(0), _DT[A.dtype], _stream()), "sp24_retained_magnitude")
    return total


def sp24_permute_search(A, sweeps=1, perm=None):
    """Search for a column order under which 2:4 pruning keeps more magnitude, starting from ``perm`` (refined in
    place; default: a new tensor holding 0, 1, 2, ...).  Returns the int32 device tensor of K column numbers."""
    _rowmajor(A, "A")
    M, K = A.shape
    if perm is None:
        perm = torch.arange(K, dtype=torch.int32, device=A.device)
    _perm_arg(perm, K)
    _check(lib().sp24_permute_search(A.data_ptr(), perm.data_ptr(), M, K, A.stride(0), _DT[A.dtype], int(sweeps), _stream()),
           "sp24_permute_search")
    return perm


def sp24_mask_apply(W, meta, layout="canonical", out=None):
    """W with every position that the metadata does not record set to +0 (the pattern is kept, not re-selected)."""
    _rowmajor(W, "W")
    M, K = W.shape
    _meta_arg(meta, M, K)
    P = _out(out, (M, K), W.dtype, W.device)
    _check(lib().sp24_mask_apply(W.data_ptr(), meta.data_ptr(), P.data_ptr(), M, K, W.stride(0), P.stride(0), _DT[W.dtype],
                                 _LAYOUT[layout], _stream()), "sp24_mask_apply")
    return P


def sp24_compress_masked(W, meta, layout="canonical", out=None):
    """Compressed values of W at the positions the metadata records."""
    _rowmajor(W, "W")
    M, K = W.shape
    _meta_arg(meta, M, K)
    V = torch.empty((M, K // 2), dtype=W.dtype, device=W.device) if out is None else _dev(out, "out")
    if V.numel() != M * (K // 2) or V.dtype != W.dtype or not V.is_contiguous():
        raise ValueError("out must be contiguous and hold M*K/2 values of W's type")
    _check(lib().sp24_compress_masked(W.data_ptr(), meta.data_ptr(), V.data_ptr(), M, K, W.stride(0), _DT[W.dtype],
                                      _LAYOUT[layout], _stream()), "sp24_compress_masked")
    return V


def _b_args(B, b_order):
    _rowmajor(B, "B")
    if b_order == "k":      # B given as [N, K]: one row per column of the math operand
        N, K = B.shape
        return N, K, B_KMAJOR
    if b_order == "n":      # B given as [K, N]
        K, N = B.shape
        return N, K, B_NMAJOR
    raise ValueError("b_order must be 'k' or 'n'")


def sp24_spmm(V, meta, B, out_dtype, b_order="k", layout="canonical", out=None):
    """D [M, N] = decompress(V, meta) @ B.  B is [N, K] for b_order "k", [K, N] for "n"."""
    M, K = _compressed(V, meta)
    N, Kb, bo = _b_args(B, b_order)
    if Kb != K:
        raise ValueError("inner dimensions differ")
    _same_type(B, V)
    D = _out(out, (M, N), out_dtype, V.device)
    _check(lib().sp24_spmm(V.data_ptr(), meta.data_ptr(), B.data_ptr(), D.data_ptr(), M, N, K, _ld(B),
                           D.stride(0), _DT[V.dtype], _DT[D.dtype], bo, _LAYOUT[layout], _stream()), "sp24_spmm")
    return D


def sp24_gemm_dense(A, B, out_dtype, b_order="k", out=None):
    """D [M, N] = A @ B on the dense matrix cores (speedup denominator)."""
    _rowmajor(A, "A")
    M, K = A.shape
    N, Kb, bo = _b_args(B, b_order)
    if Kb != K:
        raise ValueError("inner dimensions differ")
    _same_type(B, A)
    D = _out(out, (M, N), out_dtype, A.device)
    _check(lib().sp24_gemm_dense(A.data_ptr(), B.data_ptr(), D.data_ptr(), M, N, K, A.stride(0), _ld(B),
                                 D.stride(0), _DT[A.dtype], _DT[D.dtype], bo, _stream()), "sp24_gemm_dense")
    return D


def sp24_splitk_workspace_bytes(M, N, K, dtype):
    """Bytes of workspace the split-K products need for this shape (0: they would not split it)."""
    return lib().sp24_splitk_workspace_bytes(M, N, K, _DT[dtype])


def _workspace(workspace, M, N, K, dtype, device):
    need = sp24_splitk_workspace_bytes(M, N, K, dtype)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=device)
    _dev(workspace, "workspace")
    if not workspace.is_contiguous():
        raise ValueError("workspace must be contiguous")
    return workspace, workspace.numel() * workspace.element_size()


def sp24_spmm_splitk(V, meta, B, out_dtype, b_order="k", layout="canonical", workspace=None, out=None):
    """sp24_spmm with the inner dimension split across workgroups (shapes with few output tiles); ``workspace``: a
    device tensor of at least sp24_splitk_workspace_bytes(...) bytes, allocated here when None."""
    M, K = _compressed(V, meta)
    N, Kb, bo = _b_args(B, b_order)
    if Kb != K:
        raise ValueError("inner dimensions differ")
    _same_type(B, V)
    ws, ws_bytes = _workspace(workspace, M, N, K, V.dtype, V.device)
    D = _out(out, (M, N), out_dtype, V.device)
    _check(lib().sp24_spmm_splitk(V.data_ptr(), meta.data_ptr(), B.data_ptr(), D.data_ptr(), M, N, K, _ld(B), D.stride(0),
                                  _DT[V.dtype], _DT[D.dtype], bo, _LAYOUT[layout], ws.data_ptr(), ws_bytes, _stream()), "sp24_spmm_splitk")
    return D


STATIC_SCRATCH_BYTES = 8 << 20     # SP24_STATIC_SCRATCH_BYTES of the header


def sp24_spmm_splitk_static(V, meta, B, out_dtype, b_order="k", layout="canonical", out=None):
    """sp24_spmm_splitk with the partial products in the library's own static device array (no workspace, nothing
    allocated by the call itself when ``out`` is given); raises Sp24Error with status 7 for shapes whose split needs
    more than STATIC_SCRATCH_BYTES."""
    M, K = _compressed(V, meta)
    N, Kb, bo = _b_args(B, b_order)
    if Kb != K:
        raise ValueError("inner dimensions differ")
    _same_type(B, V)
    D = _out(out, (M, N), out_dtype, V.device)
    _check(lib().sp24_spmm_splitk_static(V.data_ptr(), meta.data_ptr(), B.data_ptr(), D.data_ptr(), M, N, K, _ld(B), D.stride(0),
                                         _DT[V.dtype], _DT[D.dtype], bo, _LAYOUT[layout], _stream()), "sp24_spmm_splitk_static")
    return D


def sp24_gemm_dense_splitk(A, B, out_dtype, b_order="k", workspace=None, out=None):
    """sp24_gemm_dense with the inner dimension split across workgroups."""
    _rowmajor(A, "A")
    M, K = A.shape
    N, Kb, bo = _b_args(B, b_order)
    if Kb != K:
        raise ValueError("inner dimensions differ")
    _same_type(B, A)
    ws, ws_bytes = _workspace(workspace, M, N, K, A.dtype, A.device)
    D = _out(out, (M, N), out_dtype, A.device)
    _check(lib().sp24_gemm_dense_splitk(A.data_ptr(), B.data_ptr(), D.data_ptr(), M, N, K, A.stride(0), _ld(B), D.stride(0),
                                        _DT[A.dtype], _DT[D.dtype], bo, ws.data_ptr(), ws_bytes, _stream()), "sp24_gemm_dense_splitk")
    return D


def _conv_args(X, K, R, S, pad, stride):
    _dev(X, "X")
    if X.dim() != 4 or not X.is_contiguous():
        raise ValueError("X must be a contiguous NHWC tensor [n_img, H, W, C]")
    n_img, H, W, C = X.shape
    if K != R * S * C:
        raise ValueError("the filter matrix must have R*S*C columns")
    (ph, pw), (sh, sw) = pad, stride
    OH, OW = (H + 2 * ph - R) // sh + 1, (W + 2 * pw - S) // sw + 1
    return (n_img, H, W, C, R, S, ph, pw, sh, sw), n_img * max(OH, 0) * max(OW, 0)


def sp24_spmm_conv2d(V, meta, X, out_dtype, R, S, pad=(0, 0), stride=(1, 1), layout="canonical", out=None):
    """D [M, n_img*OH*OW] = decompress(V, meta) applied as a bank of M filters to the NHWC input X, with no
    im2col matrix in memory.  Filter column k = (r*S + s)*C + c."""
    M, K = _compressed(V, meta)
    geom, N = _conv_args(X, K, R, S, pad, stride)
    _same_type(X, V, "X")
    D = _out(out, (M, N), out_dtype, V.device)
    _check(lib().sp24_spmm_conv2d(V.data_ptr(), meta.data_ptr(), X.data_ptr(), D.data_ptr(), M, *geom, D.stride(0),
                                  _DT[V.dtype], _DT[D.dtype], _LAYOUT[layout], _stream()), "sp24_spmm_conv2d")
    return D


def sp24_conv2d_dense(A, X, out_dtype, R, S, pad=(0, 0), stride=(1, 1), out=None):
    """The same convolution with the dense filter matrix A [M, R*S*C] on the dense matrix cores."""
    _rowmajor(A, "A")
    M, K = A.shape
    geom, N = _conv_args(X, K, R, S, pad, stride)
    _same_type(X, A, "X")
    D = _out(out, (M, N), out_dtype, A.device)
    _check(lib().sp24_conv2d_dense(A.data_ptr(), X.data_ptr(), D.data_ptr(), M, *geom, A.stride(0), D.stride(0),
                                   _DT[A.dtype], _DT[D.dtype], _stream()), "sp24_conv2d_dense")
    return D


def _scale_args(M, w_scale, bias):
    _dev(w_scale, "w_scale")
    if w_scale.dtype != torch.float32 or w_scale.numel() != M or not w_scale.is_contiguous():
        raise ValueError("w_scale must be a contiguous float32 vector with one entry per row")
    if bias is not None:
        _dev(bias, "bias")
        if bias.dtype != torch.float32 or bias.numel() != M or not bias.is_contiguous():
            raise ValueError("bias must be a contiguous float32 vector with one entry per row")
    return w_scale.data_ptr(), (bias.data_ptr() if bias is not None else None)


def sp24_spmm_i8_scaled(V, meta, B, out_dtype, w_scale, x_scale, bias=None, relu=False, inv_y_scale=1.0, b_order="k",
                        layout="canonical", out=None):
    """int8 sparse product with the quantised path's epilogue fused into the store: per-row weight scale,
    per-tensor activation scale, optional bias and ReLU; out_dtype int8 (re-quantised by inv_y_scale) or a float type."""
    M, K = _compressed(V, meta)
    N, Kb, bo = _b_args(B, b_order)
    if Kb != K:
        raise ValueError("inner dimensions differ")
    _same_type(B, V)
    ws, bs = _scale_args(M, w_scale, bias)
    D = _out(out, (M, N), out_dtype, V.device)
    _check(lib().sp24_spmm_i8_scaled(V.data_ptr(), meta.data_ptr(), B.data_ptr(), D.data_ptr(), M, N, K, _ld(B), D.stride(0),
                                     ws, float(x_scale), bs, int(bool(relu)), float(inv_y_scale), _DT[D.dtype], bo, _LAYOUT[layout],
                                     _stream()), "sp24_spmm_i8_scaled")
    return D


def sp24_gemm_dense_i8_scaled(A, B, out_dtype, w_scale, x_scale, bias=None, relu=False, inv_y_scale=1.0, b_order="k", out=None):
    """The same epilogue on the dense int8 product."""
    _rowmajor(A, "A")
    M, K = A.shape
    N, Kb, bo = _b_args(B, b_order)
    if Kb != K:
        raise ValueError("inner dimensions differ")
    _same_type(B, A)
    ws, bs = _scale_args(M, w_scale, bias)
    D = _out(out, (M, N), out_dtype, A.device)
    _check(lib().sp24_gemm_dense_i8_scaled(A.data_ptr(), B.data_ptr(), D.data_ptr(), M, N, K, A.stride(0), _ld(B), D.stride(0),
                                           ws, float(x_scale), bs, int(bool(relu)), float(inv_y_scale), _DT[D.dtype], bo, _stream()),
           "sp24_gemm_dense_i8_scaled")
    return D


def sp24_spmm_conv2d_i8_scaled(V, meta, X, out_dtype, R, S, w_scale, x_scale, bias=None, relu=False, inv_y_scale=1.0,
                               pad=(0, 0), stride=(1, 1), layout="canonical", out=None):
    """int8 sparse convolution (implicit GEMM) with the quantised path's epilogue; w_scale per output channel."""
    M, K = _compressed(V, meta)
    geom, N = _conv_args(X, K, R, S, pad, stride)
    _same_type(X, V, "X")
    ws, bs = _scale_args(M, w_scale, bias)
    D = _out(out, (M, N), out_dtype, V.device)
    _check(lib().sp24_spmm_conv2d_i8_scaled(V.data_ptr(), meta.data_ptr(), X.data_ptr(), D.data_ptr(), M, *geom, D.stride(0), ws,
                                            float(x_scale), bs, int(bool(relu)), float(inv_y_scale), _DT[D.dtype], _LAYOUT[layout],
                                            _stream()), "sp24_spmm_conv2d_i8_scaled")
    return D


def sp24_conv2d_dense_i8_scaled(A, X, out_dtype, R, S, w_scale, x_scale, bias=None, relu=False, inv_y_scale=1.0, pad=(0, 0),
                                stride=(1, 1), out=None):
    """The same with the dense int8 filter matrix."""
    _rowmajor(A, "A")
    M, K = A.shape
    geom, N = _conv_args(X, K, R, S, pad, stride)
    _same_type(X, A, "X")
    ws, bs = _scale_args(M, w_scale, bias)
    D = _out(out, (M, N), out_dtype, A.device)
    _check(lib().sp24_conv2d_dense_i8_scaled(A.data_ptr(), X.data_ptr(), D.data_ptr(), M, *geom, A.stride(0), D.stride(0), ws,
                                             float(x_scale), bs, int(bool(relu)), float(inv_y_scale), _DT[D.dtype], _stream()),
           "sp24_conv2d_dense_i8_scaled")
    return D
