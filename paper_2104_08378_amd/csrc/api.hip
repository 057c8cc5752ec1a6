// C ABI of libsp24: argument validation on the host, then kernel selection.
// Nothing here allocates, synchronises or touches the current device.
#include <atomic>

#include "common.hpp"
#include "launch.hpp"

using namespace sp24;

// Memory of the library's own for sp24_spmm_splitk_static, whose callers cannot allocate or pass a workspace: the
// partial products of the split product live here instead.  Every GPU the library runs on holds its own copy of
// the array until the process ends.  In host code the array's name stands for the symbol, it is not a device
// address: the address on the current device comes from hipGetSymbolAddress (static_scratch() below), and only
// that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[SP24_STATIC_SCRATCH_BYTES];

namespace {

bool is_input_type(sp24_dtype t) { return t == SP24_F16 || t == SP24_BF16 || t == SP24_I8 || t == SP24_F8; }
bool is_layout(sp24_layout l) { return l == SP24_LAYOUT_CANONICAL || l == SP24_LAYOUT_TILED; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Dimension rule of Sec. 3.2 / Sec. 4.2 on the inner dimension.
bool k_legal(int64_t K, sp24_dtype t) { return K > 0 && K % (esize_of(t) == 1 ? 32 : 16) == 0; }

bool layout_fits(int64_t M, int64_t K, sp24_layout l)
{
    return l == SP24_LAYOUT_CANONICAL || (M % 32 == 0 && K % 64 == 0);
}

bool out_legal(sp24_dtype in, sp24_dtype out, bool scaled)
{
    if (scaled) return in == SP24_I8 && (out == SP24_I8 || out == SP24_F32 || out == SP24_F16 || out == SP24_BF16);
    if (in == SP24_I8) return out == SP24_I32;
    return out == SP24_F32 || out == SP24_F16 || out == SP24_BF16;
}

// a matrix of `rows` rows, `cols` used columns, leading dimension ld (elements of size es);
// vec16: rows must start on 16-byte boundaries (the streaming kernels use 16-byte accesses),
// otherwise natural element alignment is enough.
sp24_status check_matrix(const void* p, int64_t rows, int64_t cols, int64_t ld, int es, bool vec16 = true)
{
    if (rows == 0) return SP24_OK;
    if (!p) return SP24_ERR_NULL;
    if (ld < cols) return SP24_ERR_SHAPE;
    if (vec16 ? (!aligned16(p) || (ld * es) % 16 != 0) : (reinterpret_cast<uintptr_t>(p) % es != 0)) return SP24_ERR_ALIGN;
    return SP24_OK;
}

bool ranges_overlap(const void* a, size_t na, const void* b, size_t nb)
{
    uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y + nb && y < x + na;
}

} // namespace

extern "C" {

size_t sp24_values_bytes(int64_t M, int64_t K, sp24_dtype t)
{
    if (!is_input_type(t) || M < 0 || !k_legal(K, t)) return 0;
    return (size_t)M * (size_t)(K / 2) * (size_t)esize_of(t);
}

size_t sp24_meta_bytes(int64_t M, int64_t K, sp24_dtype t, sp24_layout l)
{
    if (!is_input_type(t) || !is_layout(l) || M < 0 || !k_legal(K, t) || !layout_fits(M, K, l)) return 0;
    return (size_t)M * (size_t)(K / 8);
}

sp24_status sp24_prune(const void* A, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, sp24_dtype t, void* stream)
{
    if (!is_input_type(t)) return SP24_ERR_DTYPE;
    if (M < 0 || !k_legal(K, t)) return SP24_ERR_SHAPE;
    int es = esize_of(t);
    sp24_status s = check_matrix(A, M, K, lda, es);
    if (s != SP24_OK) return s;
    s = check_matrix(P, M, K, ldp, es);
    if (s != SP24_OK) return s;
    if (M > 0 && A == P && lda != ldp) return SP24_ERR_SHAPE;
    if (M > 0 && A != P) {
        size_t na = ((size_t)(M - 1) * lda + K) * es, np = ((size_t)(M - 1) * ldp + K) * es;
        if (ranges_overlap(A, na, P, np)) return SP24_ERR_SHAPE;
    }
    return launch_prune(A, P, M, K, lda, ldp, t, static_cast<hipStream_t>(stream));
}

sp24_status sp24_compress(const void* A, void* V, void* meta, int64_t M, int64_t K, int64_t lda, sp24_dtype t,
                          sp24_layout l, void* stream)
{
    if (!is_input_type(t)) return SP24_ERR_DTYPE;
    if (!is_layout(l)) return SP24_ERR_LAYOUT;
    if (M < 0 || !k_legal(K, t)) return SP24_ERR_SHAPE;
    if (!layout_fits(M, K, l)) return SP24_ERR_LAYOUT;
    int es = esize_of(t);
    sp24_status s = check_matrix(A, M, K, lda, es);
    if (s != SP24_OK) return s;
    if (M == 0) return SP24_OK;
    if (!V || !meta) return SP24_ERR_NULL;
    if (!aligned16(V) || !aligned16(meta)) return SP24_ERR_ALIGN;
    size_t na = ((size_t)(M - 1) * lda + K) * es;
    if (ranges_overlap(A, na, V, sp24_values_bytes(M, K, t)) || ranges_overlap(A, na, meta, sp24_meta_bytes(M, K, t, l)))
        return SP24_ERR_SHAPE;
    return launch_compress(A, V, meta, M, K, lda, t, l, static_cast<hipStream_t>(stream));
}

sp24_status sp24_decompress(const void* V, const void* meta, void* P, int64_t M, int64_t K, int64_t ldp, sp24_dtype t,
                            sp24_layout l, void* stream)
{
    if (!is_input_type(t)) return SP24_ERR_DTYPE;
    if (!is_layout(l)) return SP24_ERR_LAYOUT;
    if (M < 0 || !k_legal(K, t)) return SP24_ERR_SHAPE;
    if (!layout_fits(M, K, l)) return SP24_ERR_LAYOUT;
    int es = esize_of(t);
    sp24_status s = check_matrix(P, M, K, ldp, es);
    if (s != SP24_OK) return s;
    if (M == 0) return SP24_OK;
    if (!V || !meta) return SP24_ERR_NULL;
    if (!aligned16(V) || !aligned16(meta)) return SP24_ERR_ALIGN;
    size_t np = ((size_t)(M - 1) * ldp + K) * es;
    if (ranges_overlap(P, np, V, sp24_values_bytes(M, K, t)) || ranges_overlap(P, np, meta, sp24_meta_bytes(M, K, t, l)))
        return SP24_ERR_SHAPE;
    return launch_decompress(V, meta, P, M, K, ldp, t, l, static_cast<hipStream_t>(stream));
}

sp24_status sp24_prune_transposable(const void* A, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, sp24_dtype t, void* stream)
{
    if (!is_input_type(t)) return SP24_ERR_DTYPE;
    if (M < 0 || M % 4 != 0 || !k_legal(K, t)) return SP24_ERR_SHAPE;
    int es = esize_of(t);
    sp24_status s = check_matrix(A, M, K, lda, es);
    if (s != SP24_OK) return s;
    s = check_matrix(P, M, K, ldp, es);
    if (s != SP24_OK) return s;
    if (M > 0 && A == P && lda != ldp) return SP24_ERR_SHAPE;
    if (M > 0 && A != P) {
        size_t na = ((size_t)(M - 1) * lda + K) * es, np = ((size_t)(M - 1) * ldp + K) * es;
        if (ranges_overlap(A, na, P, np)) return SP24_ERR_SHAPE;
    }
    return launch_prune_transposable(A, P, M, K, lda, ldp, t, static_cast<hipStream_t>(stream));
}

sp24_status sp24_mask_apply(const void* W, const void* meta, void* P, int64_t M, int64_t K, int64_t ldw, int64_t ldp, sp24_dtype t,
                            sp24_layout l, void* stream)
{
    if (!is_input_type(t)) return SP24_ERR_DTYPE;
    if (!is_layout(l)) return SP24_ERR_LAYOUT;
    if (M < 0 || !k_legal(K, t)) return SP24_ERR_SHAPE;
    if (!layout_fits(M, K, l)) return SP24_ERR_LAYOUT;
    int es = esize_of(t);
    sp24_status s = check_matrix(W, M, K, ldw, es);
    if (s != SP24_OK) return s;
    s = check_matrix(P, M, K, ldp, es);
    if (s != SP24_OK) return s;
    if (M == 0) return SP24_OK;
    if (!meta) return SP24_ERR_NULL;
    if (!aligned16(meta)) return SP24_ERR_ALIGN;
    if (W == P && ldw != ldp) return SP24_ERR_SHAPE;
    size_t nw = ((size_t)(M - 1) * ldw + K) * es, np = ((size_t)(M - 1) * ldp + K) * es;
    if (W != P && ranges_overlap(W, nw, P, np)) return SP24_ERR_SHAPE;
    if (ranges_overlap(P, np, meta, sp24_meta_bytes(M, K, t, l))) return SP24_ERR_SHAPE;
    return launch_mask_apply(W, meta, P, M, K, ldw, ldp, t, l, static_cast<hipStream_t>(stream));
}

sp24_status sp24_compress_masked(const void* W, const void* meta, void* V, int64_t M, int64_t K, int64_t ldw, sp24_dtype t,
                                 sp24_layout l, void* stream)
{
    if (!is_input_type(t)) return SP24_ERR_DTYPE;
    if (!is_layout(l)) return SP24_ERR_LAYOUT;
    if (M < 0 || !k_legal(K, t)) return SP24_ERR_SHAPE;
    if (!layout_fits(M, K, l)) return SP24_ERR_LAYOUT;
    int es = esize_of(t);
    sp24_status s = check_matrix(W, M, K, ldw, es);
    if (s != SP24_OK) return s;
    if (M == 0) return SP24_OK;
    if (!V || !meta) return SP24_ERR_NULL;
    if (!aligned16(V) || !aligned16(meta)) return SP24_ERR_ALIGN;
    size_t nw = ((size_t)(M - 1) * ldw + K) * es, nv = sp24_values_bytes(M, K, t);
    if (ranges_overlap(W, nw, V, nv) || ranges_overlap(V, nv, meta, sp24_meta_bytes(M, K, t, l))) return SP24_ERR_SHAPE;
    return launch_compress_masked(W, meta, V, M, K, ldw, t, l, static_cast<hipStream_t>(stream));
}

sp24_status sp24_permute_columns(const void* A, const int32_t* perm, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp,
                                 sp24_dtype t, void* stream)
{
    if (!is_input_type(t)) return SP24_ERR_DTYPE;
    if (M < 0 || !k_legal(K, t) || K > 0x7FFFFFFF) return SP24_ERR_SHAPE;
    int es = esize_of(t);
    sp24_status s = check_matrix(A, M, K, lda, es);
    if (s != SP24_OK) return s;
    s = check_matrix(P, M, K, ldp, es);
    if (s != SP24_OK) return s;
    if (M == 0) return SP24_OK;
    if (!perm) return SP24_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(perm) % 4 != 0) return SP24_ERR_ALIGN;
    size_t na = ((size_t)(M - 1) * lda + K) * es, np = ((size_t)(M - 1) * ldp + K) * es;
    if (ranges_overlap(A, na, P, np) || ranges_overlap(P, np, perm, (size_t)K * 4)) return SP24_ERR_SHAPE;
    return launch_permute_columns(A, perm, P, M, K, lda, ldp, t, static_cast<hipStream_t>(stream));
}

sp24_status sp24_permute_rows(const void* A, const int32_t* perm, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, sp24_dtype t,
                              void* stream)
{
    if (!is_input_type(t)) return SP24_ERR_DTYPE;
    if (M < 0 || M > 0x7FFFFFFF || !k_legal(K, t)) return SP24_ERR_SHAPE;
    int es = esize_of(t);
    sp24_status s = check_matrix(A, M, K, lda, es);
    if (s != SP24_OK) return s;
    s = check_matrix(P, M, K, ldp, es);
    if (s != SP24_OK) return s;
    if (M == 0) return SP24_OK;
    if (!perm) return SP24_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(perm) % 4 != 0) return SP24_ERR_ALIGN;
    size_t na = ((size_t)(M - 1) * lda + K) * es, np = ((size_t)(M - 1) * ldp + K) * es;
    if (ranges_overlap(A, na, P, np) || ranges_overlap(P, np, perm, (size_t)M * 4)) return SP24_ERR_SHAPE;
    return launch_permute_rows(A, perm, P, M, K, lda, ldp, t, static_cast<hipStream_t>(stream));
}

sp24_status sp24_retained_magnitude(const void* A, const int32_t* perm, double* total, int64_t M, int64_t K, int64_t lda,
                                    sp24_dtype t, void* stream)
{
    if (!is_input_type(t)) return SP24_ERR_DTYPE;
    if (M < 0 || !k_legal(K, t) || K > 0x7FFFFFFF) return SP24_ERR_SHAPE;
    int es = esize_of(t);
    sp24_status s = check_matrix(A, M, K, lda, es);
    if (s != SP24_OK) return s;
    if (!total) return SP24_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(total) % 8 != 0 || reinterpret_cast<uintptr_t>(perm) % 4 != 0) return SP24_ERR_ALIGN;
    if (M > 0) {
        size_t na = ((size_t)(M - 1) * lda + K) * es;
        if (ranges_overlap(A, na, total, 8) || (perm && ranges_overlap(perm, (size_t)K * 4, total, 8))) return SP24_ERR_SHAPE;
    }
    return launch_retained_magnitude(A, perm, total, M, K, lda, t, static_cast<hipStream_t>(stream));
}

sp24_status sp24_permute_search(const void* A, int32_t* perm, int64_t M, int64_t K, int64_t lda, sp24_dtype t, int sweeps, void* stream)
{
    if (!is_input_type(t)) return SP24_ERR_DTYPE;
    if (M < 0 || !k_legal(K, t) || K > 0x7FFFFFFF || sweeps < 0 || sweeps > 64) return SP24_ERR_SHAPE;
    int es = esize_of(t);
    sp24_status s = check_matrix(A, M, K, lda, es);
    if (s != SP24_OK) return s;
    if (!perm) return SP24_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(perm) % 4 != 0) return SP24_ERR_ALIGN;
    if (M > 0 && ranges_overlap(A, ((size_t)(M - 1) * lda + K) * es, perm, (size_t)K * 4)) return SP24_ERR_SHAPE;
    return launch_permute_search(A, perm, M, K, lda, t, sweeps, static_cast<hipStream_t>(stream));
}

// Argument checks of every product entry point.  *empty: nothing to compute (M or N is 0).
// x_bytes: extent of the NHWC input when a.conv.on (a.B then points at it), else unused
static sp24_status mm_validate(const MmArgs& a, size_t x_bytes, bool* empty)
{
    *empty = false;
    if (!is_input_type(a.in) || !out_legal(a.in, a.out, a.epi.on != 0)) return SP24_ERR_DTYPE;
    if (a.bo != SP24_B_KMAJOR && a.bo != SP24_B_NMAJOR) return SP24_ERR_LAYOUT;
    if (a.M < 0 || a.N < 0 || !k_legal(a.K, a.in)) return SP24_ERR_SHAPE;
    if (a.sparse) {
        if (!is_layout(a.layout)) return SP24_ERR_LAYOUT;
        if (!layout_fits(a.M, a.K, a.layout)) return SP24_ERR_LAYOUT;
    }
    if (a.M == 0 || a.N == 0) {
        *empty = true;
        return SP24_OK;
    }
    int es = esize_of(a.in), os = esize_of(a.out);
    sp24_status s;
    if (a.epi.on) {
        if (!a.epi.w_scale) return SP24_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(a.epi.w_scale) % 4 != 0 || reinterpret_cast<uintptr_t>(a.epi.bias) % 4 != 0) return SP24_ERR_ALIGN;
    }
    if (a.sparse) {
        if (!a.A || !a.meta) return SP24_ERR_NULL;
        if (!aligned16(a.A) || !aligned16(a.meta)) return SP24_ERR_ALIGN;
    } else {
        s = check_matrix(a.A, a.M, a.K, a.lda, es);
        if (s != SP24_OK) return s;
    }
    if (a.conv.on) {
        if (!a.B) return SP24_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(a.B) % es != 0) return SP24_ERR_ALIGN;
    } else {
        s = (a.bo == SP24_B_KMAJOR) ? check_matrix(a.B, a.N, a.K, a.ldb, es, false) : check_matrix(a.B, a.K, a.N, a.ldb, es, false);
        if (s != SP24_OK) return s;
    }
    s = check_matrix(a.D, a.M, a.N, a.ldd, os, false);
    if (s != SP24_OK) return s;
    size_t nd = ((size_t)(a.M - 1) * a.ldd + a.N) * os;
    size_t nb = a.conv.on ? x_bytes
                          : (a.bo == SP24_B_KMAJOR) ? ((size_t)(a.N - 1) * a.ldb + a.K) * es : ((size_t)(a.K - 1) * a.ldb + a.N) * es;
    size_t nA = a.sparse ? sp24_values_bytes(a.M, a.K, a.in) : ((size_t)(a.M - 1) * a.lda + a.K) * es;
    if (ranges_overlap(a.D, nd, a.B, nb) || ranges_overlap(a.D, nd, a.A, nA)) return SP24_ERR_SHAPE;
    if (a.sparse && ranges_overlap(a.D, nd, a.meta, sp24_meta_bytes(a.M, a.K, a.in, a.layout))) return SP24_ERR_SHAPE;
    if (a.epi.on && (ranges_overlap(a.D, nd, a.epi.w_scale, (size_t)a.M * 4) ||
                     (a.epi.bias && ranges_overlap(a.D, nd, a.epi.bias, (size_t)a.M * 4))))
        return SP24_ERR_SHAPE;
    return SP24_OK;
}

// N <= 32: where the tiled kernels (tiles of 64 or 128 rows, most of their columns unused) overtake the streaming
// kernel, whose workgroups of 32 rows each re-read all of B and run in more than one round past 256 row blocks.
// Measured at K = 4096 and 8192, M = 2048 .. 128256, operands from HBM, in tiles = ceil(M / 128):
//  * N > 16: the dense product always (M = 4096, K = 8192, N = 32: 40.6 -> 32.6 us), the sparse one from 86 tiles on
//    (11008 rows; below that it depends on M, within 15 % either way);
//  * N <= 16, 16-bit: from 86 tiles on, sparse 3 - 10 % faster up to 128 tiles (64-row tiles), level to 191, then
//    ahead for good (32000 x 4096, N = 1: 36.4 -> 31.5 us; 128256 rows: 133 -> 117 us); dense 15 - 30 % faster
//    at 86 - 256 tiles, past that only for N > 8;
//  * N <= 16, 8-bit: the dense product for N > 8 from 86 tiles on; the sparse one stays with the streaming kernel
//    (10 - 20 % ahead at N <= 8 up to 128256 rows, level at N = 16).
static bool tiled_before_streaming(const MmArgs& a)
{
    if (a.N > 32) return true;                             // the streaming kernel does not take it anyway
    const int64_t tiles = (a.M + 127) / 128;
    if (a.N > 16) return !a.sparse || tiles >= 86;
    if (esize_of(a.in) == 2) return tiles >= 86 && (a.sparse || tiles <= 256 || a.N > 8);
    return !a.sparse && a.N > 8 && tiles >= 86;
}

// The kernel for a checked product: streaming (N <= 32), tiled, or general.
static sp24_status mm_dispatch(const MmArgs& a, hipStream_t st)
{
    bool handled = false;
    sp24_status s;
    const bool tiled_first = a.conv.on || tiled_before_streaming(a);
    if (!tiled_first) {
        s = launch_mm_skinny(a, st, &handled);
        if (handled) return s;
    }
    s = launch_mm_tiled(a, st, &handled);
    if (handled) return s;
    if (tiled_first && !a.conv.on) {
        s = launch_mm_skinny(a, st, &handled);
        if (handled) return s;
    }
    return launch_mm_simple(a, st);
}

static sp24_status mm_common(const MmArgs& a, hipStream_t st, size_t x_bytes = 0)
{
    bool empty;
    const sp24_status s = mm_validate(a, x_bytes, &empty);
    if (s != SP24_OK || empty) return s;
    return mm_dispatch(a, st);
}

// K split across workgroups.  The number of slices is a function of the shape and the input type alone: the one
// with the least estimated time among the candidates, where splitting costs 3 us (8 us for the streaming kernel:
// the second kernel and the shorter pipelines) plus the partial images written and read once at 4 TB/s, and must
// win by a tenth.
//  * N > 32 (tiled kernels, 128x128 tiles; rows past M are computed on a valid row and never stored): 1 .. min(8, compute units / tiles, steps / 4) slices of whole
//    128-byte steps; a launch takes 5 us plus 400 ns per step of its workgroups (fitted to measurements of both
//    types at 16 - 128 steps, operands from HBM); the unsplit product it is compared with runs shorter steps when it
//    has at most 128 tiles (tiles of 64 rows).
//  * N <= 32, M >= 32 (streaming kernel, one workgroup per 32 rows): 1 .. min(8, compute units / row blocks,
//    tiles / 32) slices of whole 64-column tiles; a workgroup takes 130 ns (16-bit) or 80 ns (8-bit) per tile of
//    its 32 rows (measured at K = 16384: latency-bound, the same whether 16 or 128 workgroups run).
//  * N <= 32, M < 32: not split (the general kernel).
struct SplitPlan {
    int slices, slice_steps;    // slice_steps in the kernel's own unit: 128-byte steps, or 64-column tiles
    bool streaming;             // the N <= 32 kernel
    int64_t ldw;                // values per row of a partial image
    size_t bytes;               // workspace: slices images of M x ldw accumulator values
};
static SplitPlan split_plan(int64_t M, int64_t N, int64_t K, sp24_dtype in)
{
    SplitPlan p = {1, 0, N <= 32, 0, 0};
    if (N <= 32 && M < 32) return p;
    const int es = esize_of(in);
    const int64_t ldw = (N + 3) / 4 * 4;
    int64_t units, most, unit_ns, base_ns, fixed_ns;         // K in the kernel's units; slices at most; time per unit; per launch; cost of splitting
    if (p.streaming) {
        units = (K + 63) / 64;
        most = 256 / ((M + 31) / 32);
        if (most > units / 32) most = units / 32;
        unit_ns = es == 2 ? 130 : 80;
        base_ns = 0;
        fixed_ns = 8000;
    } else {
        units = K * es / 128;
        most = 256 / (((M + 127) / 128) * ((N + 127) / 128));
        if (most > units / 4) most = units / 4;
        unit_ns = 400;
        base_ns = 5000;
        fixed_ns = 3000;
    }
    if (most > 8) most = 8;
    // the unsplit tiled product on at most 128 tiles runs on tiles of 64 rows, with shorter steps (215 ns when they are
    // 64 columns wide, 325 ns else: fitted to the sparse products of both types at 64 and 128 steps)
    int64_t unsplit_unit_ns = unit_ns;
    if (!p.streaming && ((M + 127) / 128) * ((N + 127) / 128) <= 128) unsplit_unit_ns = N <= 64 ? 215 : 325;
    int64_t best_ns = (base_ns + units * unsplit_unit_ns) * 9 / 10, best = 1, best_per = units;
    for (int64_t want = 2; want <= most; ++want) {
        const int64_t per = (units + want - 1) / want;
        const int64_t slices = (units + per - 1) / per;      // no slice is empty
        const int64_t ns = base_ns + per * unit_ns + fixed_ns + slices * M * ldw / 500;
        if (ns < best_ns) {
            best_ns = ns;
            best = slices;
            best_per = per;
        }
    }
    if (best <= 1) return p;
    p.slices = (int)best;
    p.slice_steps = (int)best_per;
    p.ldw = ldw;
    p.bytes = (size_t)p.slices * (size_t)M * (size_t)ldw * 4;
    return p;
}

// Address of `scratch` on the current device, looked up once per device (with that device current) and kept.
static sp24_status static_scratch(void** out)
{
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> ptr_of_device[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SP24_ERR_LAUNCH;
    void* p = ptr_of_device[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SP24_ERR_LAUNCH;
        ptr_of_device[dev].store(p, std::memory_order_release);   // two first callers store the same address
    }
    *out = p;
    return SP24_OK;
}

// use_static: the partial products go to the library's own scratch array instead of a caller's workspace
static sp24_status mm_splitk(const MmArgs& a, void* workspace, size_t workspace_bytes, hipStream_t st, bool use_static = false)
{
    bool empty;
    sp24_status s = mm_validate(a, 0, &empty);
    if (s != SP24_OK || empty) return s;
    const SplitPlan plan = split_plan(a.M, a.N, a.K, a.in);
    if (plan.slices <= 1) return mm_dispatch(a, st);
    if (use_static) {
        if (plan.bytes > (size_t)SP24_STATIC_SCRATCH_BYTES) return SP24_ERR_WORKSPACE;
        s = static_scratch(&workspace);
        if (s != SP24_OK) return s;
        workspace_bytes = SP24_STATIC_SCRATCH_BYTES;
    }
    if (!workspace) return SP24_ERR_NULL;
    if (!aligned16(workspace)) return SP24_ERR_ALIGN;
    if (workspace_bytes < plan.bytes) return SP24_ERR_SHAPE;
    const int es = esize_of(a.in);
    const size_t nd = ((size_t)(a.M - 1) * a.ldd + a.N) * esize_of(a.out);
    const size_t nb = (a.bo == SP24_B_KMAJOR) ? ((size_t)(a.N - 1) * a.ldb + a.K) * es : ((size_t)(a.K - 1) * a.ldb + a.N) * es;
    const size_t nA = a.sparse ? sp24_values_bytes(a.M, a.K, a.in) : ((size_t)(a.M - 1) * a.lda + a.K) * es;
    if (ranges_overlap(workspace, plan.bytes, a.D, nd) || ranges_overlap(workspace, plan.bytes, a.B, nb) ||
        ranges_overlap(workspace, plan.bytes, a.A, nA))
        return SP24_ERR_SHAPE;
    if (a.sparse && ranges_overlap(workspace, plan.bytes, a.meta, sp24_meta_bytes(a.M, a.K, a.in, a.layout))) return SP24_ERR_SHAPE;
    MmArgs part = a;
    part.D = workspace;
    part.ldd = plan.ldw;
    part.out = (a.in == SP24_I8) ? SP24_I32 : SP24_F32;
    part.k_slices = plan.slices;
    part.slice_steps = plan.slice_steps;
    bool handled = false;
    s = plan.streaming ? launch_mm_skinny(part, st, &handled) : launch_mm_tiled(part, st, &handled);
    if (!handled) return mm_dispatch(a, st);             // operands that kernel does not take: not split
    if (s != SP24_OK) return s;
    return launch_splitk_reduce(workspace, plan.slices, a.M, a.N, plan.ldw, a.D, a.ldd, a.in == SP24_I8, a.out, st);
}

size_t sp24_splitk_workspace_bytes(int64_t M, int64_t N, int64_t K, sp24_dtype in)
{
    if (!is_input_type(in) || M <= 0 || N <= 0 || !k_legal(K, in)) return 0;
    return split_plan(M, N, K, in).bytes;
}

sp24_status sp24_spmm_splitk(const void* V, const void* meta, const void* B, void* D, int64_t M, int64_t N, int64_t K, int64_t ldb,
                             int64_t ldd, sp24_dtype in, sp24_dtype out, sp24_border bo, sp24_layout l, void* workspace,
                             size_t workspace_bytes, void* stream)
{
    MmArgs a{V, meta, B, D, M, N, K, 0, ldb, ldd, in, out, bo, l, true};
    return mm_splitk(a, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

sp24_status sp24_spmm_splitk_static(const void* V, const void* meta, const void* B, void* D, int64_t M, int64_t N, int64_t K,
                                    int64_t ldb, int64_t ldd, sp24_dtype in, sp24_dtype out, sp24_border bo, sp24_layout l,
                                    void* stream)
{
    MmArgs a{V, meta, B, D, M, N, K, 0, ldb, ldd, in, out, bo, l, true};
    return mm_splitk(a, nullptr, 0, static_cast<hipStream_t>(stream), true);
}

sp24_status sp24_gemm_dense_splitk(const void* A, const void* B, void* D, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb,
                                   int64_t ldd, sp24_dtype in, sp24_dtype out, sp24_border bo, void* workspace,
                                   size_t workspace_bytes, void* stream)
{
    MmArgs a{A, nullptr, B, D, M, N, K, lda, ldb, ldd, in, out, bo, SP24_LAYOUT_CANONICAL, false};
    return mm_splitk(a, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

sp24_status sp24_spmm(const void* V, const void* meta, const void* B, void* D, int64_t M, int64_t N, int64_t K, int64_t ldb,
                      int64_t ldd, sp24_dtype in, sp24_dtype out, sp24_border bo, sp24_layout l, void* stream)
{
    MmArgs a{V, meta, B, D, M, N, K, 0, ldb, ldd, in, out, bo, l, true};
    return mm_common(a, static_cast<hipStream_t>(stream));
}

sp24_status sp24_gemm_dense(const void* A, const void* B, void* D, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb,
                            int64_t ldd, sp24_dtype in, sp24_dtype out, sp24_border bo, void* stream)
{
    MmArgs a{A, nullptr, B, D, M, N, K, lda, ldb, ldd, in, out, bo, SP24_LAYOUT_CANONICAL, false};
    return mm_common(a, static_cast<hipStream_t>(stream));
}

sp24_status sp24_spmm_i8_scaled(const void* V, const void* meta, const void* B, void* D, int64_t M, int64_t N, int64_t K,
                                int64_t ldb, int64_t ldd, const float* w_scale, float x_scale, const float* bias, int relu,
                                float inv_y_scale, sp24_dtype out, sp24_border bo, sp24_layout l, void* stream)
{
    MmArgs a{V, meta, B, D, M, N, K, 0, ldb, ldd, SP24_I8, out, bo, l, true};
    a.epi = Epilogue{w_scale, bias, x_scale, inv_y_scale, relu != 0, 1};
    return mm_common(a, static_cast<hipStream_t>(stream));
}

sp24_status sp24_gemm_dense_i8_scaled(const void* A, const void* B, void* D, int64_t M, int64_t N, int64_t K, int64_t lda,
                                      int64_t ldb, int64_t ldd, const float* w_scale, float x_scale, const float* bias, int relu,
                                      float inv_y_scale, sp24_dtype out, sp24_border bo, void* stream)
{
    MmArgs a{A, nullptr, B, D, M, N, K, lda, ldb, ldd, SP24_I8, out, bo, SP24_LAYOUT_CANONICAL, false};
    a.epi = Epilogue{w_scale, bias, x_scale, inv_y_scale, relu != 0, 1};
    return mm_common(a, static_cast<hipStream_t>(stream));
}

// Shared front end of the two convolution entry points: geometry checks, then the product path with B = X.
static sp24_status conv_common(MmArgs& a, int64_t n_img, int64_t H, int64_t W, int64_t C, int R, int S, int pad_h, int pad_w,
                               int stride_h, int stride_w, hipStream_t st)
{
    if (!is_input_type(a.in) || !out_legal(a.in, a.out, a.epi.on != 0)) return SP24_ERR_DTYPE;
    const int64_t lim = (int64_t)1 << 20;
    if (a.M < 0 || n_img < 0 || H < 1 || W < 1 || C < 1 || R < 1 || S < 1 || pad_h < 0 || pad_w < 0 || stride_h < 1 || stride_w < 1 ||
        H > lim || W > lim || C > lim || R > 4096 || S > 4096 || pad_h > 4096 || pad_w > 4096 || stride_h > 4096 || stride_w > 4096 ||
        H + 2 * pad_h < R || W + 2 * pad_w < S)
        return SP24_ERR_SHAPE;
    const int es = esize_of(a.in);
    if ((C * es) % 16 != 0) return SP24_ERR_SHAPE;      // 16 consecutive bytes of K never straddle a filter tap
    const int64_t OH = (H + 2 * pad_h - R) / stride_h + 1, OW = (W + 2 * pad_w - S) / stride_w + 1;
    const int64_t K = (int64_t)R * S * C;
    if (K > ((int64_t)1 << 30) || (n_img > 0 && OH * OW > (((int64_t)1 << 31) - 1) / n_img)) return SP24_ERR_SHAPE;
    if (n_img > 0 && H * W * C > (((int64_t)1 << 46) / n_img)) return SP24_ERR_SHAPE;
    a.N = n_img * OH * OW;
    a.K = K;
    a.bo = SP24_B_KMAJOR;
    a.ldb = K;
    if (R == 1 && S == 1 && pad_h == 0 && pad_w == 0 && stride_h == 1 && stride_w == 1) {
        // a pointwise convolution is the plain product with the NHWC input as the K-major second operand, one row
        // per pixel: it takes the product kernels as they are (the streaming one for few pixels included)
        a.conv = ConvGeom{};
        a.ldb = C;
        return mm_common(a, st);
    }
    a.conv = ConvGeom{1, (int)H, (int)W, (int)C, R, S, pad_h, pad_w, stride_h, stride_w, (int)OH, (int)OW};
    return mm_common(a, st, (size_t)n_img * H * W * C * es);
}

sp24_status sp24_spmm_conv2d(const void* V, const void* meta, const void* X, void* D, int64_t M, int64_t n_img, int64_t H,
                             int64_t W, int64_t C, int R, int S, int pad_h, int pad_w, int stride_h, int stride_w, int64_t ldd,
                             sp24_dtype in, sp24_dtype out, sp24_layout l, void* stream)
{
    MmArgs a{V, meta, X, D, M, 0, 0, 0, 0, ldd, in, out, SP24_B_KMAJOR, l, true};
    return conv_common(a, n_img, H, W, C, R, S, pad_h, pad_w, stride_h, stride_w, static_cast<hipStream_t>(stream));
}

sp24_status sp24_conv2d_dense(const void* A, const void* X, void* D, int64_t M, int64_t n_img, int64_t H, int64_t W, int64_t C,
                              int R, int S, int pad_h, int pad_w, int stride_h, int stride_w, int64_t lda, int64_t ldd,
                              sp24_dtype in, sp24_dtype out, void* stream)
{
    MmArgs a{A, nullptr, X, D, M, 0, 0, lda, 0, ldd, in, out, SP24_B_KMAJOR, SP24_LAYOUT_CANONICAL, false};
    return conv_common(a, n_img, H, W, C, R, S, pad_h, pad_w, stride_h, stride_w, static_cast<hipStream_t>(stream));
}

sp24_status sp24_spmm_conv2d_i8_scaled(const void* V, const void* meta, const void* X, void* D, int64_t M, int64_t n_img,
                                       int64_t H, int64_t W, int64_t C, int R, int S, int pad_h, int pad_w, int stride_h,
                                       int stride_w, int64_t ldd, const float* w_scale, float x_scale, const float* bias,
                                       int relu, float inv_y_scale, sp24_dtype out, sp24_layout l, void* stream)
{
    MmArgs a{V, meta, X, D, M, 0, 0, 0, 0, ldd, SP24_I8, out, SP24_B_KMAJOR, l, true};
    a.epi = Epilogue{w_scale, bias, x_scale, inv_y_scale, relu != 0, 1};
    return conv_common(a, n_img, H, W, C, R, S, pad_h, pad_w, stride_h, stride_w, static_cast<hipStream_t>(stream));
}

sp24_status sp24_conv2d_dense_i8_scaled(const void* A, const void* X, void* D, int64_t M, int64_t n_img, int64_t H, int64_t W,
                                        int64_t C, int R, int S, int pad_h, int pad_w, int stride_h, int stride_w, int64_t lda,
                                        int64_t ldd, const float* w_scale, float x_scale, const float* bias, int relu,
                                        float inv_y_scale, sp24_dtype out, void* stream)
{
    MmArgs a{A, nullptr, X, D, M, 0, 0, lda, 0, ldd, SP24_I8, out, SP24_B_KMAJOR, SP24_LAYOUT_CANONICAL, false};
    a.epi = Epilogue{w_scale, bias, x_scale, inv_y_scale, relu != 0, 1};
    return conv_common(a, n_img, H, W, C, R, S, pad_h, pad_w, stride_h, stride_w, static_cast<hipStream_t>(stream));
}

const char* sp24_status_string(sp24_status s)
{
    switch (s) {
    case SP24_OK: return "ok";
    case SP24_ERR_NULL: return "a required pointer is NULL";
    case SP24_ERR_SHAPE: return "illegal shape, leading dimension or overlapping buffers";
    case SP24_ERR_ALIGN: return "pointer or leading dimension not 16-byte aligned";
    case SP24_ERR_DTYPE: return "unknown or unsupported element type";
    case SP24_ERR_LAYOUT: return "unknown layout or shape not legal for the layout";
    case SP24_ERR_LAUNCH: return "HIP launch failed";
    case SP24_ERR_WORKSPACE: return "the shape needs more scratch memory than the library's static buffer holds";
    }
    return "unknown status";
}

} // extern "C"
