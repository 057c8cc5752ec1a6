// Internal launch entry points shared by the C-ABI layer (api.hip).
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/sp24.h"
#include "common.hpp"

namespace sp24 {

sp24_status launch_prune(const void* A, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, sp24_dtype t, hipStream_t st);
sp24_status launch_compress(const void* A, void* V, void* meta, int64_t M, int64_t K, int64_t lda, sp24_dtype t, sp24_layout l, hipStream_t st);
sp24_status launch_prune_transposable(const void* A, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, sp24_dtype t, hipStream_t st);
sp24_status launch_mask_apply(const void* W, const void* meta, void* P, int64_t M, int64_t K, int64_t ldw, int64_t ldp, sp24_dtype t,
                              sp24_layout l, hipStream_t st);
sp24_status launch_permute_columns(const void* A, const void* perm, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, sp24_dtype t,
                                   hipStream_t st);
sp24_status launch_permute_rows(const void* A, const void* perm, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, sp24_dtype t,
                                hipStream_t st);
sp24_status launch_retained_magnitude(const void* A, const void* perm, double* out, int64_t M, int64_t K, int64_t lda, sp24_dtype t,
                                      hipStream_t st);
sp24_status launch_permute_search(const void* A, int32_t* perm, int64_t M, int64_t K, int64_t lda, sp24_dtype t, int sweeps, hipStream_t st);
sp24_status launch_compress_masked(const void* W, const void* meta, void* V, int64_t M, int64_t K, int64_t ldw, sp24_dtype t,
                                   sp24_layout l, hipStream_t st);
sp24_status launch_decompress(const void* V, const void* meta, void* P, int64_t M, int64_t K, int64_t ldp, sp24_dtype t, sp24_layout l, hipStream_t st);

// Geometry of a convolution read as an implicit GEMM (Sec. 3.2: convolutions are GEMM-like operations; Sec. 4.2:
// inner dimension C x R x S): the second operand is never formed, element (k, n) of it is
//   X[img][oy*stride_h - pad_h + r][ox*stride_w - pad_w + s][c]   (zero outside the image)
// with k = (r*S + s)*C + c and n = (img*OH + oy)*OW + ox, X being NHWC.
struct ConvGeom {
    int on;                 // 0: plain matrix B
    int H, W, C, R, S, pad_h, pad_w, stride_h, stride_w, OH, OW;
};

// Problem description for the matrix-multiply kernels.  For the sparse product
// A = V and lda is unused; for the dense product meta is null.
struct MmArgs {
    const void* A;      // V (sparse) or dense A
    const void* meta;   // sparse only
    const void* B;
    void* D;
    int64_t M, N, K;
    int64_t lda, ldb, ldd; // elements
    sp24_dtype in, out;
    sp24_border bo;
    sp24_layout layout;    // sparse only
    bool sparse;
    ConvGeom conv;         // conv.on: B is the NHWC input X, N = n_img*OH*OW, K = R*S*C, bo / ldb unused
    Epilogue epi;          // epi.on: int8 inputs, scaled / re-quantised output (out = I8, F16, BF16 or F32)
    // K split across workgroups (tiled kernels only; k_slices > 1): slice s covers slice_steps whole 128-byte steps
    // from s * slice_steps on and writes its partial product, in the accumulator type, to image s of D
    // (M rows of ldd values each); out must then be F32 or I32, and conv and epi off.
    int k_slices, slice_steps;
};

// General kernel: any M, N; both layouts; both B orders.  One wavefront per 32x32 tile of D.
sp24_status launch_mm_simple(const MmArgs& a, hipStream_t st);

// Streaming kernel for N <= 32; returns false in *handled when the problem does not fit it.
sp24_status launch_mm_skinny(const MmArgs& a, hipStream_t st, bool* handled);

// Tiled kernels for large shapes; return false in *handled when the shape does not fit them.
sp24_status launch_mm_tiled(const MmArgs& a, hipStream_t st, bool* handled);

// D [M, N] (type out) = the sum, in slice order, of `slices` partial products (float or int32, M rows of ldw values
// each, images M * ldw values apart).
sp24_status launch_splitk_reduce(const void* partial, int slices, int64_t M, int64_t N, int64_t ldw, void* D, int64_t ldd, bool integer,
                                 sp24_dtype out, hipStream_t st);

} // namespace sp24
