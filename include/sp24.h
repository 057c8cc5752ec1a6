/*
 * sp24 -- 2:4 structured-sparse matrix multiply for AMD MI355X (gfx950, CDNA4).
 *
 * C ABI of libsp24.so.  The operations are those of "Accelerating Sparse Deep
 * Neural Networks" (arXiv 2104.08378):
 *   - the 2:4 pattern: every aligned group of 4 consecutive values along a row
 *     of the first GEMM operand holds at least 2 zeros (Sec. 1, Sec. 3);
 *   - magnitude pruning to that pattern (Sec. 4.1, Step 2);
 *   - the compressed format: a half-width value array plus 2 bits of position
 *     metadata per kept value (Sec. 3.1);
 *   - sparse x dense = dense matrix multiply with the compressed matrix as the
 *     first operand (Sec. 3.2, Fig. 2), and a same-shape dense multiply, the
 *     denominator of the paper's speedups (Sec. 3.2, Fig. 3).
 *
 * Notation: A is M x K (first operand, K contiguous, row stride lda elements);
 * groups run along K from column 0.  P = pruned A.  V = kept values, M x K/2.
 * B is the dense second operand K x N, D the M x N result (row-major, row
 * stride ldd elements).
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates, frees and synchronises nothing and never changes the current
 *     device.  (sp24_*_bytes and sp24_status_string touch no device at all.)
 *   - Every call is asynchronous on the caller's HIP stream, passed as void*
 *     (a hipStream_t; NULL = the default stream).  Results are valid once the
 *     caller has synchronised that stream.
 *   - All validation happens on the host before any launch: a call that
 *     returns anything but SP24_OK has launched nothing and written nothing.
 *   - Leading dimensions are in elements.  A, P, V and meta must be 16-byte
 *     aligned and every row of A and P must start 16-byte aligned
 *     (ld * element_size % 16 == 0); B and D need only the alignment of their
 *     element type and any leading dimension that covers a row.  Otherwise
 *     SP24_ERR_ALIGN.  (The fast product kernels are chosen when B and D rows
 *     are 16-byte aligned too -- for N-major B also N * element size a
 *     multiple of 16; other cases run a general kernel.)
 *   - K must be a multiple of 16 for 16-bit types and of 32 for the 8-bit types
 *     (the dimension rule of Sec. 3.2 / Sec. 4.2, applied to the inner
 *     dimension), else SP24_ERR_SHAPE.  M and N may be any positive value; a
 *     zero M or N is accepted and does nothing.
 *   - Selection rule where the paper is silent: magnitudes are compared
 *     exactly; on equal magnitude the lower column is kept; every NaN counts
 *     as one magnitude above infinity; |-128| = 128; a removed slot holds +0.
 */
#ifndef SP24_H
#define SP24_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SP24_OK = 0,
    SP24_ERR_NULL = 1,   /* a required pointer is NULL                         */
    SP24_ERR_SHAPE = 2,  /* negative size, illegal K, ld too small, or buffers overlap */
    SP24_ERR_ALIGN = 3,  /* pointer or leading dimension not 16-byte aligned    */
    SP24_ERR_DTYPE = 4,  /* unknown type or unsupported in/out combination      */
    SP24_ERR_LAYOUT = 5, /* unknown layout, or shape not legal for that layout  */
    SP24_ERR_LAUNCH = 6, /* the HIP runtime rejected a launch                   */
    SP24_ERR_WORKSPACE = 7 /* sp24_spmm_splitk_static: the shape needs more than SP24_STATIC_SCRATCH_BYTES */
} sp24_status;

typedef enum {
    SP24_F16 = 0,  /* IEEE binary16                                   */
    SP24_BF16 = 1, /* bfloat16                                        */
    SP24_I8 = 2,   /* signed 8-bit integer (as output: sp24_*_i8_scaled only) */
    SP24_F32 = 3,  /* output only                                     */
    SP24_I32 = 4,  /* output only (required for SP24_I8 inputs)       */
    SP24_F8 = 5    /* input only: 8-bit float, 1 sign, 4 exponent (bias 7), 3 fraction bits, no
                      infinities, NaN = 0x7F / 0xFF, largest finite value 448.  Not one of the
                      formats of the paper's Table 1: the further input format this chip's
                      sparse matrix instruction takes; products accumulate in fp32 like the
                      16-bit types and are written as SP24_F32, SP24_F16 or SP24_BF16 */
} sp24_dtype;

/*
 * Layout of the compressed pair (V, meta) -- Sec. 3.1 fixes the content (two
 * kept values per group in column order; 2 bits per kept value giving its
 * position in the group), not the packing.  A group's code is
 * pos0 | pos1 << 2 with pos0 < pos1 (six legal codes: 0x4 0x8 0x9 0xC 0xD 0xE).
 *
 * SP24_LAYOUT_CANONICAL  V row-major [M][K/2]; meta bytes [M][K/8], the even
 *     group of a byte in bits 0..3.  Interchange format.
 *
 *     Every product accepts it; the tiled layout below is 1.2-1.5x faster.
 *
 * SP24_LAYOUT_TILED  the same codes and values permuted so that one wavefront
 *     loads the operands of a 32x32 sparse-MFMA tile with contiguous 16-byte
 *     and 4-byte accesses.  Needs M % 32 == 0 and K % 64 == 0, else
 *     SP24_ERR_LAYOUT.  Tiles of 32 rows x 64 columns of A are stored in
 *     order [M/32][K/64]; with slot = (m % 32) + 32 * h, where h = 0,1 names
 *     the 32-column half of the tile:
 *       meta: one uint32 per slot, 64 per tile: the canonical bytes
 *             8*kb + 4*h .. +3 of row m as a little-endian word;
 *       V, 8-bit : 16 bytes per slot, 64 slots per tile: canonical V columns
 *             32*kb + 16*h .. +15 of row m;
 *       V, 16-bit: two runs of 64 slots x 16 bytes per tile; run s = 0,1
 *             holds canonical V columns 32*kb + 16*h + 8*s .. +7 of row m.
 *     Total sizes equal the canonical ones.
 */
typedef enum { SP24_LAYOUT_CANONICAL = 0, SP24_LAYOUT_TILED = 1 } sp24_layout;

/* Storage order of the dense second operand B (K x N). */
typedef enum {
    SP24_B_KMAJOR = 0, /* element (k,n) at B[n*ldb + k]: one row per token / pixel */
    SP24_B_NMAJOR = 1  /* element (k,n) at B[k*ldb + n]                            */
} sp24_border;

/* Sizes in bytes of V and meta for an M x K matrix (Sec. 3.1: K/2 values and
 * K/8 metadata bytes per row -- 36 bits per group of four 16-bit values).
 * Return 0 for an illegal type, shape or layout. */
size_t sp24_values_bytes(int64_t M, int64_t K, sp24_dtype t);
size_t sp24_meta_bytes(int64_t M, int64_t K, sp24_dtype t, sp24_layout l);

/*
 * Sec. 4.1 Step 2: P = A with the two smallest-magnitude entries of every
 * group of four set to +0; kept entries are copied bit for bit.
 * A, P: device, M x K, row strides lda, ldp (elements).  P may equal A
 * (in place, then ldp must equal lda); partial overlap is not allowed.
 */
sp24_status sp24_prune(const void* A, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp,
                       sp24_dtype t, void* stream);

/*
 * Sec. 3.1: prune (same rule as sp24_prune) and compress in one pass.
 * A: device, M x K, row stride lda.  V: device, sp24_values_bytes(M,K,t)
 * bytes.  meta: device, sp24_meta_bytes(M,K,t,l) bytes.  Neither may overlap A.
 * Compressing an already pruned matrix keeps exactly its non-zeros.
 */
sp24_status sp24_compress(const void* A, void* V, void* meta, int64_t M, int64_t K, int64_t lda,
                          sp24_dtype t, sp24_layout l, void* stream);

/*
 * Inverse of sp24_compress: P (M x K, row stride ldp) receives the kept values
 * at their recorded positions and +0 elsewhere.  Metadata codes other than the
 * six legal ones give unspecified values in that group (never an out-of-range
 * access).
 */
sp24_status sp24_decompress(const void* V, const void* meta, void* P, int64_t M, int64_t K, int64_t ldp,
                            sp24_dtype t, sp24_layout l, void* stream);

/*
 * Sec. 4.1, Step 2 (channel permutations; Fig. 6): the matrix with its columns
 * taken in the order perm, P[m][k] = A[m][perm[k]], bit for bit.  Permuting
 * the columns of the weights before pruning -- and the rows of the second
 * operand alike: for a K-major B those are the columns of the stored array,
 * the same call -- leaves the product unchanged and can raise the magnitude
 * that pruning keeps.  perm: K int32 entries in device memory, a permutation
 * of 0 .. K-1 (an entry outside that range reads column 0; never an
 * out-of-range access).  A and P as for sp24_prune, but they must not overlap.
 * K < 2^31.
 */
sp24_status sp24_permute_columns(const void* A, const int32_t* perm, void* P, int64_t M, int64_t K,
                                 int64_t lda, int64_t ldp, sp24_dtype t, void* stream);

/*
 * The companion of sp24_permute_columns on the layer that produces the
 * activations (Sec. 4.1, Step 2: the rows of that layer's weights are permuted
 * so that its outputs arrive in the order the permuted columns expect):
 * P[m][:] = A[perm[m]][:], bit for bit.  perm: M int32 entries in device
 * memory, a permutation of 0 .. M-1 (an entry outside that range reads row 0).
 * A and P as for sp24_prune, not overlapping.  M < 2^31.
 */
sp24_status sp24_permute_rows(const void* A, const int32_t* perm, void* P, int64_t M, int64_t K,
                              int64_t lda, int64_t ldp, sp24_dtype t, void* stream);

/*
 * Fig. 6's figure of merit for a column order: *total (one double in device
 * memory, 8-byte aligned, overwritten) = the sum of |a| over the elements that
 * sp24_prune would keep if the groups of four were formed from columns
 * perm[4g] .. perm[4g+3] (perm == NULL: the columns as they are).  Magnitudes
 * and selection as in sp24_prune (|-128| = 128; a kept NaN makes the total
 * NaN).  The terms are exact binary64 values added in no fixed order: results
 * of two calls may differ in the last bits.  A as for sp24_prune; with M == 0
 * the total is 0.
 */
sp24_status sp24_retained_magnitude(const void* A, const int32_t* perm, double* total, int64_t M, int64_t K,
                                    int64_t lda, sp24_dtype t, void* stream);

/*
 * Sec. 4.1, Step 2 / Fig. 6: the search for a column order under which
 * pruning keeps more magnitude.  The paper states the aim and defers the
 * method; this one is the library's own -- bounded, the same result on every
 * run, and never worse than the order it starts from:
 *   - perm (device, K int32, in/out) is read as K/4 groups of four columns;
 *     on entry it must hold a permutation of 0 .. K-1 (0, 1, 2, ... for a
 *     fresh search; an entry outside that range reads column 0, never out of
 *     bounds, and the result is then unspecified);
 *   - the score of a group is the sum over the rows of the row's two largest
 *     magnitudes among its four columns (magnitudes as in sp24_prune, NaN
 *     counting as +infinity);
 *   - a step takes two groups g < h, eight columns (positions 0-3 those of
 *     g), and tries the 35 ways of dealing them out as two groups: a way is
 *     the positions a < b < c that share a group with position 0; ways are
 *     visited in lexicographic order of (a, b, c), the first being the present
 *     arrangement, and a later way wins only with a strictly higher sum of its
 *     two scores; the winner goes back with position 0's group in g, the other
 *     in h, both in ascending position;
 *   - round r = 0, 1, .. pairs every group whose bit r is clear with the group
 *     2^r further on, where that exists; a sweep is the rounds r = 0 ..
 *     ceil(log2(K/4)) - 1; `sweeps` (0 .. 64) sweeps run, one launch per round.
 * Sums are binary64 (exact integers for int8): a row contributes the sum of
 * its two largest magnitudes; rows are added in 256 interleaved partial sums
 * (row m into partial m mod 256, in row order), the partials as a balanced
 * binary tree over neighbours, the two scores of a way last.
 * sp24_retained_magnitude of the result is never below that of the input
 * order.  Apply the result with sp24_permute_columns to the weights and to a
 * K-major second operand (or sp24_permute_rows to the producing layer).
 * A as for sp24_prune; perm 4-byte aligned, not overlapping A.  M == 0 leaves
 * perm as it is.
 */
sp24_status sp24_permute_search(const void* A, int32_t* perm, int64_t M, int64_t K, int64_t lda,
                                sp24_dtype t, int sweeps, void* stream);

/*
 * Sec. 6: a pattern that satisfies the 2:4 constraint along rows and along
 * columns, so that the transposed matrix (the backward pass) can use the
 * sparse product too.  The exhaustive search the paper names, per aligned
 * 4 x 4 block: of the 90 patterns with exactly two kept entries in every row
 * and every column the one whose kept magnitudes sum highest stays, the rest
 * of the block becomes +0; kept entries are copied bit for bit.
 * Made unique by: a pattern's sum is ((r0 + r1) + r2) + r3, r_i = the sum of
 * row i's two kept magnitudes (lower column first), in binary64 for the 16-bit
 * types and exactly for int8; NaN counts as +infinity; patterns are visited in
 * lexicographic order of their four column pairs (pairs ordered (0,1) (0,2)
 * (0,3) (1,2) (1,3) (2,3)) and only a strictly higher sum replaces the best.
 * A, P as for sp24_prune; additionally M % 4 == 0, else SP24_ERR_SHAPE.
 */
sp24_status sp24_prune_transposable(const void* A, void* P, int64_t M, int64_t K, int64_t lda,
                                    int64_t ldp, sp24_dtype t, void* stream);

/*
 * Sec. 4.1 Step 3 (retraining keeps the pattern of Step 2; a removed weight
 * stays zero): P = W with every position that `meta` does not record set to
 * +0, recorded positions copied bit for bit.  W holds the dense weights after
 * an optimizer step; `meta` (layout l) comes from sp24_compress of the Step-2
 * weights.  W, P: device, M x K, row strides ldw, ldp; P may equal W (then
 * ldp = ldw).  Codes other than the six legal ones keep unspecified positions
 * of their group.
 */
sp24_status sp24_mask_apply(const void* W, const void* meta, void* P, int64_t M, int64_t K,
                            int64_t ldw, int64_t ldp, sp24_dtype t, sp24_layout l, void* stream);

/*
 * The compressed values of W under the same fixed pattern: V (layout l, same
 * size as from sp24_compress) receives W's values at the positions `meta`
 * records; nothing is selected and `meta` is not written.  (V, meta) then
 * decompresses to sp24_mask_apply(W, meta) and is ready for sp24_spmm.
 */
sp24_status sp24_compress_masked(const void* W, const void* meta, void* V, int64_t M, int64_t K,
                                 int64_t ldw, sp24_dtype t, sp24_layout l, void* stream);

/*
 * Sec. 3.2, Fig. 2: D = decompress(V, meta) x B.  Products of 16-bit inputs
 * are accumulated in fp32 and written as `out` = SP24_F32, SP24_F16 or
 * SP24_BF16 (one rounding, to nearest even); int8 products are accumulated in
 * int32 and `out` must be SP24_I32 (exact for K <= 2^17).
 * The removed half of A takes no part in the sum (Sec. 3.2: the multiplications
 * by zero are skipped): where B holds an infinity or a NaN opposite a removed
 * position, the result is the finite sum of the kept products, whereas the
 * dense product of the pruned matrix has 0 x inf = NaN there.  NaN and
 * infinities in kept positions propagate as IEEE arithmetic gives them.
 * B: device, ldb >= K (K-major) or ldb >= N (N-major).  D: device, M x N,
 * ldd >= N; must not overlap the inputs.
 */
sp24_status sp24_spmm(const void* V, const void* meta, const void* B, void* D, int64_t M, int64_t N,
                      int64_t K, int64_t ldb, int64_t ldd, sp24_dtype in, sp24_dtype out,
                      sp24_border bo, sp24_layout l, void* stream);

/*
 * The same-shape dense product D = A x B on the dense matrix cores, with the
 * same types, accumulation and layouts as sp24_spmm: the denominator of the
 * sparse-vs-dense speedup (Sec. 3.2, Fig. 3).  A: device, M x K, row stride lda.
 */
sp24_status sp24_gemm_dense(const void* A, const void* B, void* D, int64_t M, int64_t N, int64_t K,
                            int64_t lda, int64_t ldb, int64_t ldd, sp24_dtype in, sp24_dtype out,
                            sp24_border bo, void* stream);

/*
 * Sec. 3.2, Fig. 2: the same two products for shapes with too few output
 * tiles to occupy the chip (32 < N <= 128 at large M and K, a small M x N
 * with a long K, or N <= 32 with few rows and a long K): the inner dimension
 * is cut into slices, one workgroup per tile and slice writes a partial
 * product in the accumulator type (fp32 or int32) to `workspace`, and a
 * second kernel adds the slices in slice order and converts to `out`.  int8 results equal sp24_spmm's bit for bit;
 * results of 16-bit inputs differ from it by the order of the fp32 additions
 * only, and are the same from call to call.
 * How many slices -- a function of M, N, K and `in` alone -- follows from
 * sp24_splitk_workspace_bytes(M, N, K, in): the bytes `workspace` must hold
 * (device, 16-byte aligned, not overlapping any operand; contents before the
 * call are ignored, contents after it unspecified), or 0 when the shape would
 * not be split (or is not legal).  With 0 the call is sp24_spmm /
 * sp24_gemm_dense and `workspace` may be NULL; so it is for operands the
 * tiled and streaming kernels do not take (alignment of B; N <= 32 with an
 * N-major B, or with the canonical layout and K % 64 != 0).  Errors as for sp24_spmm, and
 * SP24_ERR_NULL / SP24_ERR_ALIGN for a missing or misaligned workspace,
 * SP24_ERR_SHAPE when workspace_bytes is too small or it overlaps an operand.
 * Calls sharing one workspace must not overlap in time.
 */
size_t sp24_splitk_workspace_bytes(int64_t M, int64_t N, int64_t K, sp24_dtype in);
sp24_status sp24_spmm_splitk(const void* V, const void* meta, const void* B, void* D, int64_t M,
                             int64_t N, int64_t K, int64_t ldb, int64_t ldd, sp24_dtype in,
                             sp24_dtype out, sp24_border bo, sp24_layout l, void* workspace,
                             size_t workspace_bytes, void* stream);
sp24_status sp24_gemm_dense_splitk(const void* A, const void* B, void* D, int64_t M, int64_t N,
                                   int64_t K, int64_t lda, int64_t ldb, int64_t ldd, sp24_dtype in,
                                   sp24_dtype out, sp24_border bo, void* workspace,
                                   size_t workspace_bytes, void* stream);

/*
 * sp24_spmm_splitk for callers that cannot allocate device memory or carry a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments (minus the workspace), same kernels and
 * the same results bit for bit; the partial products go to an array of
 * SP24_STATIC_SCRATCH_BYTES bytes that the library holds in device memory
 * itself (one copy on every GPU it runs on, for the life of the process).
 * The call allocates and frees nothing.  A shape whose split needs more --
 * sp24_splitk_workspace_bytes(M, N, K, in) > SP24_STATIC_SCRATCH_BYTES -- is
 * refused with SP24_ERR_WORKSPACE before anything is launched; a shape that
 * is not split (0 bytes) runs as sp24_spmm and touches no scratch.  All calls
 * on one GPU share the one array: calls that overlap in time on the same GPU
 * (two streams, two threads) race and give unspecified results; calls on one
 * stream are ordered and safe.  Nothing in the array needs clearing between
 * calls (every value read was written by the same call).
 */
#define SP24_STATIC_SCRATCH_BYTES (8u << 20)
sp24_status sp24_spmm_splitk_static(const void* V, const void* meta, const void* B, void* D, int64_t M,
                                    int64_t N, int64_t K, int64_t ldb, int64_t ldd, sp24_dtype in,
                                    sp24_dtype out, sp24_border bo, sp24_layout l, void* stream);

/*
 * Convolution as a GEMM-like operation whose first argument is the sparse
 * tensor (Sec. 3.2; inner dimension C x R x S, Sec. 4.2), computed as an
 * implicit GEMM: the second operand is never formed in memory.
 *   D[m][(img*OH + oy)*OW + ox] = sum over r, s, c of
 *       W[m][(r*S + s)*C + c] * X[img][oy*stride_h - pad_h + r][ox*stride_w - pad_w + s][c]
 * with W = decompress(V, meta), M filters of K = R*S*C columns (input channel
 * innermost, so a group of four is four consecutive channels of one filter
 * tap); taps outside the image contribute zero; OH = (H + 2*pad_h - R) /
 * stride_h + 1, OW likewise; N = n_img*OH*OW.
 * X: device, NHWC [n_img][H][W][C], dense, element-aligned (16-byte aligned
 * for the fast kernels).  D: device, M x N, ldd >= N.  Types, accumulation,
 * rounding and layouts as for sp24_spmm.
 * SP24_ERR_SHAPE unless H, W, C, R, S >= 1, pads >= 0, strides >= 1,
 * H + 2*pad_h >= R, W + 2*pad_w >= S, C * element size is a multiple of 16
 * bytes (16 bytes of K never straddle a filter tap), K is legal, and the
 * sizes stay below 2^20 (H, W, C), 4096 (R, S, pads, strides), 2^31 (N).
 */
sp24_status sp24_spmm_conv2d(const void* V, const void* meta, const void* X, void* D, int64_t M,
                             int64_t n_img, int64_t H, int64_t W, int64_t C, int R, int S,
                             int pad_h, int pad_w, int stride_h, int stride_w, int64_t ldd,
                             sp24_dtype in, sp24_dtype out, sp24_layout l, void* stream);

/*
 * The same convolution with the dense filter matrix A (M x R*S*C, row stride
 * lda) on the dense matrix cores: the denominator of the speedup for
 * convolution layers (Sec. 3.2, Fig. 3).
 */
sp24_status sp24_conv2d_dense(const void* A, const void* X, void* D, int64_t M, int64_t n_img,
                              int64_t H, int64_t W, int64_t C, int R, int S, int pad_h, int pad_w,
                              int stride_h, int stride_w, int64_t lda, int64_t ldd, sp24_dtype in,
                              sp24_dtype out, void* stream);

/*
 * The INT8 deployment path (Sec. 5: activations carry one scaling factor per
 * tensor, weights one per row of the weight matrix, i.e. per output channel):
 * the int8 sparse product with its de-quantisation fused into the store.
 * For accumulator acc (int32, exact) of row m:
 *     s = w_scale[m] * x_scale
 *     y = fma(float(acc), s, bias[m])        bias = NULL means 0
 *     y = max(y, 0)                          when relu != 0
 * `out` = SP24_F32, SP24_F16 or SP24_BF16 stores y (one rounding to nearest
 * even); `out` = SP24_I8 stores clamp(rint(y * inv_y_scale), -128, 127) with
 * rint rounding half to even.  Every step is one binary32 operation, so the
 * int8 result is uniquely defined.  Scales and bias must be finite.
 * V, meta, B, D, shapes, layouts: as for sp24_spmm with int8 inputs.
 * w_scale, bias: device, M floats each, 4-byte aligned, not overlapping D.
 * inv_y_scale is ignored unless out = SP24_I8.
 */
sp24_status sp24_spmm_i8_scaled(const void* V, const void* meta, const void* B, void* D, int64_t M,
                                int64_t N, int64_t K, int64_t ldb, int64_t ldd, const float* w_scale,
                                float x_scale, const float* bias, int relu, float inv_y_scale,
                                sp24_dtype out, sp24_border bo, sp24_layout l, void* stream);

/* The same epilogue on the dense int8 product D = A x B (speedup denominator of the quantised path). */
sp24_status sp24_gemm_dense_i8_scaled(const void* A, const void* B, void* D, int64_t M, int64_t N,
                                      int64_t K, int64_t lda, int64_t ldb, int64_t ldd,
                                      const float* w_scale, float x_scale, const float* bias, int relu,
                                      float inv_y_scale, sp24_dtype out, sp24_border bo, void* stream);

/*
 * The same epilogue on the convolutions: w_scale holds one factor per output
 * channel m (Sec. 5: per-channel scaling factors for convolution weights).
 * Geometry as for sp24_spmm_conv2d / sp24_conv2d_dense with int8 inputs;
 * scales, bias, relu, inv_y_scale and `out` as for sp24_spmm_i8_scaled.
 */
sp24_status sp24_spmm_conv2d_i8_scaled(const void* V, const void* meta, const void* X, void* D, int64_t M,
                                       int64_t n_img, int64_t H, int64_t W, int64_t C, int R, int S,
                                       int pad_h, int pad_w, int stride_h, int stride_w, int64_t ldd,
                                       const float* w_scale, float x_scale, const float* bias, int relu,
                                       float inv_y_scale, sp24_dtype out, sp24_layout l, void* stream);
sp24_status sp24_conv2d_dense_i8_scaled(const void* A, const void* X, void* D, int64_t M, int64_t n_img,
                                        int64_t H, int64_t W, int64_t C, int R, int S, int pad_h, int pad_w,
                                        int stride_h, int stride_w, int64_t lda, int64_t ldd,
                                        const float* w_scale, float x_scale, const float* bias, int relu,
                                        float inv_y_scale, sp24_dtype out, void* stream);

/* Static, NUL-terminated description of a status code. */
const char* sp24_status_string(sp24_status s);

#ifdef __cplusplus
}
#endif
#endif /* SP24_H */
