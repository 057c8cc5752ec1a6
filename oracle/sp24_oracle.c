/*
 * sp24 oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar CPU statement of what the 2:4 structured-sparse
 * matrix-multiply path computes, written from the paper ("Accelerating Sparse
 * Deep Neural Networks", arXiv 2104.08378).  It exists so that tests, the
 * smoke check and the benchmark's cpu_baseline leg have something independent
 * to compare the GPU library with.  It shares no code, headers, tables or
 * helpers with the GPU library and must never be reached from the product path.
 *
 * Notation (Sec. 3, Fig. 2): A is the first GEMM operand, M x K, row-major,
 * K contiguous.  Groups are 4 consecutive elements of a row, aligned to
 * column 0.  V is the M x K/2 array of kept values, meta the 2-bit positions.
 *
 * Element types: 0 = fp16 (IEEE binary16), 1 = bf16, 2 = int8, 3 = fp8 (the
 * 8-bit float with 4 exponent and 3 fraction bits, no infinities; one of the
 * further input formats of Table 1's kind that the target chip multiplies in
 * its sparse form).  The float types are passed as raw bit patterns
 * (uint16_t, uint8_t for fp8).
 *
 * Readings where the paper is silent (all listed again in the design notes):
 *   - ties in magnitude: the lower column index wins (is kept);
 *   - every NaN has the same, largest, magnitude (above infinity);
 *   - |-128| for int8 is 128 (no wrap);
 *   - a removed slot holds +0 (all bits clear);
 *   - a group with more than two zeros still records two positions, chosen by
 *     the same rule (Sec. 3.1, last sentence of the metadata paragraph);
 *   - inside a group positions are recorded in ascending order, groups in
 *     column order (the [[0,3],[1,2]] example of Sec. 3.1);
 *   - canonical metadata packing: one 4-bit code  pos0 | pos1<<2  per group,
 *     two groups per byte, the even group in bits 0..3; bytes laid out
 *     [M][K/8].  The paper does not give a packing; this one is ours.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { T_F16 = 0, T_BF16 = 1, T_I8 = 2, T_F8 = 3 };

/* ---- exact conversion of the 16-bit storage formats to double ---------- */

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
double sp24o_f16_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24); /* subnormal: f * 2^-10 * 2^-14 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -v : v;
}

/* bfloat16: the upper half of an IEEE binary32 (1 sign, 8 exponent, 7 fraction). */
double sp24o_bf16_to_double(uint16_t b)
{
    int sign = (b >> 15) & 1;
    int e = (b >> 7) & 0xff;
    int f = b & 0x7f;
    double v;
    if (e == 0)
        v = ldexp((double)f, -7 - 126);
    else if (e == 255)
        v = f ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)f / 128.0, e - 127);
    return sign ? -v : v;
}

/*
 * 8-bit float, 1 sign, 4 exponent (bias 7), 3 fraction bits, the "finite" variant: no infinities, the one NaN is
 * exponent and fraction all ones, so the largest finite value is 1.75 * 2^8 = 448; exponent 0 holds the
 * subnormals f * 2^-9.
 */
double sp24o_f8_to_double(uint8_t b)
{
    int sign = (b >> 7) & 1;
    int e = (b >> 3) & 0xf;
    int f = b & 0x7;
    double v;
    if (e == 0)
        v = ldexp((double)f, -9);
    else if (e == 15 && f == 7)
        v = NAN;
    else
        v = ldexp(1.0 + (double)f / 8.0, e - 7);
    return sign ? -v : v;
}

static double elem_to_double(const void *p, long i, int t)
{
    if (t == T_F8)
        return sp24o_f8_to_double(((const uint8_t *)p)[i]);
    if (t == T_F16)
        return sp24o_f16_to_double(((const uint16_t *)p)[i]);
    if (t == T_BF16)
        return sp24o_bf16_to_double(((const uint16_t *)p)[i]);
    return (double)((const int8_t *)p)[i];
}

/* ---- the selection rule (Sec. 4.1, Step 2) ----------------------------- */

/* Magnitude as an ordered pair: NaN above everything, else |x|. */
typedef struct { int is_nan; double abs; } mag_t;

static mag_t magnitude(double x)
{
    mag_t m;
    m.is_nan = isnan(x) ? 1 : 0;
    m.abs = m.is_nan ? 0.0 : fabs(x);
    return m;
}

static int mag_greater(mag_t a, mag_t b)
{
    if (a.is_nan != b.is_nan)
        return a.is_nan > b.is_nan;
    return a.abs > b.abs;
}

static int mag_equal(mag_t a, mag_t b)
{
    return a.is_nan == b.is_nan && a.abs == b.abs;
}

/*
 * keep[i] = 1 for the two elements of the group that survive: element i is
 * removed when at least two others come before it in the order
 * (magnitude descending, column ascending): of every group of four the two
 * entries of least magnitude go (Sec. 4.1, Step 2).
 */
static void select_two(const double x[4], int keep[4])
{
    mag_t m[4];
    for (int i = 0; i < 4; ++i)
        m[i] = magnitude(x[i]);
    for (int i = 0; i < 4; ++i) {
        int ahead = 0;
        for (int j = 0; j < 4; ++j) {
            if (j == i)
                continue;
            if (mag_greater(m[j], m[i]) || (mag_equal(m[j], m[i]) && j < i))
                ++ahead;
        }
        keep[i] = ahead < 2;
    }
}

static void group_keep(const void *A, long base, int t, int keep[4])
{
    double x[4];
    for (int i = 0; i < 4; ++i)
        x[i] = elem_to_double(A, base + i, t);
    select_two(x, keep);
}

static long esize(int t) { return (t == T_I8 || t == T_F8) ? 1 : (t == T_F16 || t == T_BF16) ? 2 : 0; }

/* ---- O1: prune (dense -> dense, Sec. 4.1 Step 2; pattern of Sec. 3) ---- */
int sp24o_prune(const void *A, void *P, long M, long K, int t)
{
    if (K % 4 || esize(t) == 0)
        return 1;
    long es = esize(t);
    for (long m = 0; m < M; ++m)
        for (long g = 0; g < K / 4; ++g) {
            long base = m * K + 4 * g;
            int keep[4];
            group_keep(A, base, t, keep);
            for (int i = 0; i < 4; ++i) {
                char *dst = (char *)P + (base + i) * es;
                const char *src = (const char *)A + (base + i) * es;
                if (keep[i])
                    memmove(dst, src, es); /* bit-for-bit */
                else
                    memset(dst, 0, es);    /* +0 */
            }
        }
    return 0;
}

/* ---- O2: compress (Sec. 3.1: value array + 2-bit positions) ------------ */
int sp24o_compress(const void *A, void *V, uint8_t *meta, long M, long K, int t)
{
    if (K % 8 || esize(t) == 0)
        return 1;
    long es = esize(t);
    memset(meta, 0, (size_t)(M * K / 8));
    for (long m = 0; m < M; ++m)
        for (long g = 0; g < K / 4; ++g) {
            long base = m * K + 4 * g;
            int keep[4], pos[2], n = 0;
            group_keep(A, base, t, keep);
            for (int i = 0; i < 4; ++i)
                if (keep[i])
                    pos[n++] = i; /* ascending */
            for (int s = 0; s < 2; ++s)
                memcpy((char *)V + (m * (K / 2) + 2 * g + s) * es,
                       (const char *)A + (base + pos[s]) * es, es);
            unsigned code = (unsigned)pos[0] | ((unsigned)pos[1] << 2);
            meta[m * (K / 8) + g / 2] |= (uint8_t)(code << (4 * (g & 1)));
        }
    return 0;
}

/* ---- O3: decompress (inverse scatter) ---------------------------------- */
int sp24o_decompress(const void *V, const uint8_t *meta, void *P, long M, long K, int t)
{
    if (K % 8 || esize(t) == 0)
        return 1;
    long es = esize(t);
    memset(P, 0, (size_t)(M * K * es));
    for (long m = 0; m < M; ++m)
        for (long g = 0; g < K / 4; ++g) {
            unsigned code = (meta[m * (K / 8) + g / 2] >> (4 * (g & 1))) & 0xf;
            int pos[2] = { (int)(code & 3), (int)(code >> 2) };
            if (pos[0] >= pos[1])
                return 2; /* not one of the six legal codes */
            for (int s = 0; s < 2; ++s)
                memcpy((char *)P + (m * K + 4 * g + pos[s]) * es,
                       (const char *)V + (m * (K / 2) + 2 * g + s) * es, es);
        }
    return 0;
}

/*
 * ---- O4: the product, by definition (Sec. 3.2, Fig. 2) -------------------
 * D[m][n] = sum_k P[m][k] * B[k][n] over the full, decompressed P (zeros are
 * multiplied out, not skipped).  B is K x N row-major, D is M x N row-major.
 * Float inputs (16-bit, fp8) are converted exactly to double and accumulated in double;
 * int8 accumulates in int32.  The k loop runs in ascending order for every
 * output; rows are independent, which is all the OpenMP pragma uses.
 */
int sp24o_gemm_f64(const void *P, const void *B, double *D,
                   long M, long N, long K, int t)
{
    if (t != T_F16 && t != T_BF16 && t != T_F8)
        return 1;
#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m) {
        double *d = D + m * N;
        for (long n = 0; n < N; ++n)
            d[n] = 0.0;
        for (long k = 0; k < K; ++k) {
            double a = elem_to_double(P, m * K + k, t);
            for (long n = 0; n < N; ++n)
                d[n] += a * elem_to_double(B, k * N + n, t);
        }
    }
    return 0;
}

int sp24o_gemm_i32(const int8_t *P, const int8_t *B, int32_t *D,
                   long M, long N, long K)
{
#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m) {
        int32_t *d = D + m * N;
        for (long n = 0; n < N; ++n)
            d[n] = 0;
        for (long k = 0; k < K; ++k) {
            int32_t a = P[m * K + k];
            for (long n = 0; n < N; ++n)
                d[n] += a * (int32_t)B[k * N + n];
        }
    }
    return 0;
}

/*
 * ---- O5: convolution with the pruned filter bank, by definition ----------
 * The paper treats a convolution as a GEMM-like operation whose first
 * argument is the sparse tensor (Sec. 3.2) with inner dimension C x R x S
 * (Sec. 4.2); the group of four runs over consecutive input channels of one
 * filter tap, k = (r*S + s)*C + c.  Written out directly on the NHWC input
 * X[n_img][H][W][C], no matrix is formed:
 *   D[m][(img*OH + oy)*OW + ox] =
 *       sum_{r,s,c} P[m][(r*S + s)*C + c] * X[img][oy*sh - ph + r][ox*sw - pw + s][c]
 * where taps that fall outside the image contribute nothing (zero padding),
 * OH = (H + 2*ph - R)/sh + 1, OW = (W + 2*pw - S)/sw + 1.  D is M x N
 * row-major with N = n_img*OH*OW.  Same arithmetic as O4.
 */
#define CONV_LOOP(ACC_T, LOAD_P, LOAD_X)                                                     \
    long OH = (H + 2 * ph - R) / sh + 1, OW = (W + 2 * pw - S) / sw + 1;                     \
    long N = n_img * OH * OW, K = R * S * C;                                                 \
    if (H + 2 * ph < R || W + 2 * pw < S || sh < 1 || sw < 1)                                \
        return 1;                                                                            \
    _Pragma("omp parallel for schedule(static)")                                            \
    for (long m = 0; m < M; ++m)                                                             \
        for (long img = 0; img < n_img; ++img)                                               \
            for (long oy = 0; oy < OH; ++oy)                                                 \
                for (long ox = 0; ox < OW; ++ox) {                                           \
                    ACC_T acc = 0;                                                           \
                    for (long r = 0; r < R; ++r)                                             \
                        for (long s = 0; s < S; ++s) {                                       \
                            long iy = oy * sh - ph + r, ix = ox * sw - pw + s;               \
                            if (iy < 0 || iy >= H || ix < 0 || ix >= W)                      \
                                continue;                                                    \
                            for (long c = 0; c < C; ++c)                                     \
                                acc += LOAD_P(m * K + (r * S + s) * C + c) *                 \
                                       LOAD_X(((img * H + iy) * W + ix) * C + c);            \
                        }                                                                    \
                    D[m * N + (img * OH + oy) * OW + ox] = acc;                              \
                }                                                                            \
    return 0;

int sp24o_conv2d_f64(const void *P, const void *X, double *D, long M, long n_img,
                     long H, long W, long C, long R, long S, long ph, long pw, long sh, long sw, int t)
{
    if (t != T_F16 && t != T_BF16 && t != T_F8)
        return 1;
#define LP(i) elem_to_double(P, (i), t)
#define LX(i) elem_to_double(X, (i), t)
    CONV_LOOP(double, LP, LX)
#undef LP
#undef LX
}

int sp24o_conv2d_i32(const int8_t *P, const int8_t *X, int32_t *D, long M, long n_img,
                     long H, long W, long C, long R, long S, long ph, long pw, long sh, long sw)
{
#define LP(i) (int32_t) P[(i)]
#define LX(i) (int32_t) X[(i)]
    CONV_LOOP(int32_t, LP, LX)
#undef LP
#undef LX
}

/*
 * ---- O7: keeping the pattern during retraining (Sec. 4.1, Step 3) ---------
 * Retraining keeps the pattern that Step 2 chose: after an optimizer
 * step on the dense weights W, every position that Step 2 removed is set back
 * to +0 (mask_apply), and the compressed values are refreshed from W at the
 * positions the metadata records, without selecting again (compress_masked).
 * meta is canonical (O2).  Kept values are copied bit for bit.
 */
int sp24o_mask_apply(const void *W, const uint8_t *meta, void *P, long M, long K, int t)
{
    int es = esize(t);
    if (es == 0 || K % 8)
        return 1;
    for (long m = 0; m < M; ++m)
        for (long g = 0; g < K / 4; ++g) {
            uint8_t byte = meta[m * (K / 8) + g / 2];
            int code = (g % 2) ? (byte >> 4) : (byte & 15);
            int p0 = code & 3, p1 = (code >> 2) & 3;
            if (p0 >= p1)
                return 2;
            for (int j = 0; j < 4; ++j) {
                char *dst = (char *)P + (m * K + 4 * g + j) * es;
                if (j == p0 || j == p1)
                    memcpy(dst, (const char *)W + (m * K + 4 * g + j) * es, es);
                else
                    memset(dst, 0, es);
            }
        }
    return 0;
}

int sp24o_compress_masked(const void *W, const uint8_t *meta, void *V, long M, long K, int t)
{
    int es = esize(t);
    if (es == 0 || K % 8)
        return 1;
    for (long m = 0; m < M; ++m)
        for (long g = 0; g < K / 4; ++g) {
            uint8_t byte = meta[m * (K / 8) + g / 2];
            int code = (g % 2) ? (byte >> 4) : (byte & 15);
            int pos[2] = {code & 3, (code >> 2) & 3};
            if (pos[0] >= pos[1])
                return 2;
            for (int s = 0; s < 2; ++s)
                memcpy((char *)V + (m * (K / 2) + 2 * g + s) * es,
                       (const char *)W + (m * K + 4 * g + pos[s]) * es, es);
        }
    return 0;
}

/*
 * ---- O8: patterns that also hold for the transposed matrix -----------------
 * To use the sparse product in the backward pass the 2:4 constraint must hold
 * along rows and along columns (Sec. 6).  The paper names an exhaustive search
 * whose aim is the least loss of weight magnitude and gives no listing; this
 * is that search written out: every aligned 4 x 4 block keeps the entries of
 * the one pattern, among those with exactly two kept entries in each row and
 * each column (there are 90), whose kept magnitudes sum highest.
 * Made unique by: magnitudes as in O1 (every NaN counts as +infinity here);
 * the sum of a pattern is ((r0 + r1) + r2) + r3 with r_i = |a[i][c]| + |a[i][c']|
 * (c < c' the kept columns of row i), in double for the 16-bit types (exact
 * conversion) and in integers for int8; patterns are visited in lexicographic
 * order of their four column pairs, pairs ordered (0,1) (0,2) (0,3) (1,2) (1,3)
 * (2,3), and only a strictly higher sum replaces the best so far.
 */
int sp24o_prune_transposable(const void *A, void *P, long M, long K, int t)
{
    static const int pair[6][2] = {{0, 1}, {0, 2}, {0, 3}, {1, 2}, {1, 3}, {2, 3}};
    int es = esize(t);
    if (es == 0 || M % 4 || K % 4)
        return 1;
    for (long bm = 0; bm < M; bm += 4)
        for (long bk = 0; bk < K; bk += 4) {
            double mag[4][4];
            for (int i = 0; i < 4; ++i)
                for (int j = 0; j < 4; ++j) {
                    long idx = (bm + i) * K + bk + j;
                    if (t == T_I8) {
                        mag[i][j] = fabs((double)((const int8_t *)A)[idx]);
                    } else {
                        double v = elem_to_double(A, idx, t);
                        mag[i][j] = (v != v) ? INFINITY : fabs(v);
                    }
                }
            int best[4] = {-1, -1, -1, -1};
            double best_sum = -1.0;
            int p[4];
            for (p[0] = 0; p[0] < 6; ++p[0])
                for (p[1] = 0; p[1] < 6; ++p[1])
                    for (p[2] = 0; p[2] < 6; ++p[2])
                        for (p[3] = 0; p[3] < 6; ++p[3]) {
                            int count[4] = {0, 0, 0, 0};
                            for (int i = 0; i < 4; ++i) {
                                ++count[pair[p[i]][0]];
                                ++count[pair[p[i]][1]];
                            }
                            if (count[0] != 2 || count[1] != 2 || count[2] != 2 || count[3] != 2)
                                continue;
                            double r[4];
                            for (int i = 0; i < 4; ++i)
                                r[i] = mag[i][pair[p[i]][0]] + mag[i][pair[p[i]][1]];
                            double sum = ((r[0] + r[1]) + r[2]) + r[3];
                            if (sum > best_sum) {
                                best_sum = sum;
                                memcpy(best, p, sizeof best);
                            }
                        }
            for (int i = 0; i < 4; ++i)
                for (int j = 0; j < 4; ++j) {
                    long idx = (bm + i) * K + bk + j;
                    char *dst = (char *)P + idx * es;
                    if (j == pair[best[i]][0] || j == pair[best[i]][1])
                        memcpy(dst, (const char *)A + idx * es, es);
                    else
                        memset(dst, 0, es);
                }
        }
    return 0;
}

/*
 * ---- O6: epilogue of the quantised path ----------------------------------
 * The paper's INT8 recipe (Sec. 5, image classification and translation
 * paragraphs) fixes the granularity of the scaling factors: one per tensor
 * for activations, one per row of the weight matrix (= per output channel of
 * a convolution).  It prints no formula; the one used here is the plain
 * de-quantisation of an integer product, optionally followed by bias, ReLU
 * and re-quantisation with a per-tensor output scale:
 *     s_m  = w_scale[m] * x_scale
 *     y_mn = acc_mn * s_m + bias[m]          (bias = 0 when absent)
 *     y_mn = max(y_mn, 0)                    (when relu)
 *     q_mn = clamp(round_half_even(y_mn * inv_y_scale), -128, 127)
 * sp24o_dequant_f64 evaluates y in double (the reference for floating-point
 * outputs).  sp24o_requant_i8 produces q: a rounding decision, so it is taken
 * in the arithmetic the device uses -- binary32, s_m by one multiplication,
 * y by one fused multiply-add of float(acc), max, one multiplication by
 * inv_y_scale, round to nearest even, clamp.
 */
#include <math.h>

int sp24o_dequant_f64(const int32_t *acc, double *Y, long M, long N, const float *w_scale,
                      float x_scale, const float *bias, int relu)
{
    for (long m = 0; m < M; ++m) {
        double s = (double)w_scale[m] * (double)x_scale;
        double b = bias ? (double)bias[m] : 0.0;
        for (long n = 0; n < N; ++n) {
            double y = (double)acc[m * N + n] * s + b;
            if (relu && y < 0.0)
                y = 0.0;
            Y[m * N + n] = y;
        }
    }
    return 0;
}

int sp24o_requant_i8(const int32_t *acc, int8_t *Q, long M, long N, const float *w_scale,
                     float x_scale, const float *bias, int relu, float inv_y_scale)
{
    for (long m = 0; m < M; ++m) {
        volatile float s = w_scale[m] * x_scale;       /* one binary32 product */
        float b = bias ? bias[m] : 0.0f;
        for (long n = 0; n < N; ++n) {
            float y = fmaf((float)acc[m * N + n], s, b);
            if (relu)
                y = fmaxf(y, 0.0f);
            volatile float t = y * inv_y_scale;        /* one binary32 product */
            float r = nearbyintf(t);                   /* default rounding mode: to nearest even */
            r = fminf(fmaxf(r, -128.0f), 127.0f);
            Q[m * N + n] = (int8_t)(int)r;
        }
    }
    return 0;
}

/* ---- channel permutations (Sec. 4.1, Step 2; Fig. 6) -------------------- */

/*
 * The matrix with its columns taken in the order perm: P[m][k] = A[m][perm[k]]
 * (bit for bit).  perm must hold every column 0 .. K-1 once (else 2).
 */
int sp24o_permute_columns(const void *A, const int32_t *perm, void *P, long M, long K, int t)
{
    int es = esize(t);
    if (es == 0)
        return 1;
    char *seen = (char *)calloc((size_t)(K > 0 ? K : 1), 1);
    if (!seen)
        return 3;
    for (long k = 0; k < K; ++k) {
        if (perm[k] < 0 || perm[k] >= K || seen[perm[k]]) {
            free(seen);
            return 2;
        }
        seen[perm[k]] = 1;
    }
    free(seen);
    for (long m = 0; m < M; ++m)
        for (long k = 0; k < K; ++k)
            memcpy((char *)P + (m * K + k) * es, (const char *)A + (m * K + perm[k]) * es, es);
    return 0;
}

/*
 * The companion step (Sec. 4.1, Step 2): the rows of the matrix in the order
 * perm, P[m][:] = A[perm[m]][:] -- what is done to the weights of the layer
 * that produces the activations, so that the product stays the same.
 * perm must hold every row 0 .. M-1 once (else 2).
 */
int sp24o_permute_rows(const void *A, const int32_t *perm, void *P, long M, long K, int t)
{
    int es = esize(t);
    if (es == 0)
        return 1;
    char *seen = (char *)calloc((size_t)(M > 0 ? M : 1), 1);
    if (!seen)
        return 3;
    for (long m = 0; m < M; ++m) {
        if (perm[m] < 0 || perm[m] >= M || seen[perm[m]]) {
            free(seen);
            return 2;
        }
        seen[perm[m]] = 1;
    }
    free(seen);
    for (long m = 0; m < M; ++m)
        memcpy((char *)P + m * K * es, (const char *)A + (long)perm[m] * K * es, (size_t)(K * es));
    return 0;
}

/*
 * The figure of merit of a column order (Fig. 6: the magnitude that is left
 * after pruning, summed over the matrix): the sum of |a| over the elements that the selection rule of
 * Step 2 keeps when the groups of four are formed from columns perm[4g] ..
 * perm[4g+3] (perm == NULL: the columns as they are).  Plain double sum, rows
 * then groups then positions in ascending order; a kept NaN makes it NaN.
 */
int sp24o_retained_magnitude(const void *A, const int32_t *perm, long M, long K, int t, double *out)
{
    if (esize(t) == 0 || K % 4)
        return 1;
    double total = 0.0;
    for (long m = 0; m < M; ++m)
        for (long g = 0; g < K / 4; ++g) {
            double x[4];
            int keep[4];
            for (int i = 0; i < 4; ++i) {
                long col = perm ? perm[4 * g + i] : 4 * g + i;
                if (col < 0 || col >= K)
                    return 2;
                x[i] = elem_to_double(A, m * K + col, t);
            }
            select_two(x, keep);
            for (int i = 0; i < 4; ++i)
                if (keep[i])
                    total += fabs(x[i]);
        }
    *out = total;
    return 0;
}

/*
 * ---- search for a column order (Sec. 4.1, Step 2; Fig. 6) ------------------
 * The paper states the aim -- a column order under which pruning keeps more
 * magnitude -- and defers the method to a separate publication, so the search
 * below is this build's own: bounded, deterministic, and never worse than
 * the order it starts from.
 *
 * The order perm is read as K/4 groups of four columns (group g = perm[4g] ..
 * perm[4g+3]).  The score of a group is the magnitude pruning keeps in it:
 * the sum over the rows of the row's two largest magnitudes among the group's
 * four columns (NaN counts as +infinity).  A step takes two groups g < h, i.e.
 * eight columns in the order perm[4g..4g+3], perm[4h..4h+3], and tries the 35
 * ways of dealing them out as two groups of four; a way is named by the three
 * positions 0 < a < b < c that share a group with position 0, ways are visited
 * in lexicographic order of (a, b, c) -- the first, (1, 2, 3), is the present
 * arrangement -- and a later way replaces the best so far only with a strictly
 * higher sum of the two scores.  The winner's columns are written back with
 * position 0's group in g and the other in h, each in ascending position.
 * A round r = 0, 1, ... pairs every group g whose bit r is clear with
 * h = g + 2^r (where h exists); the pairs of a round are disjoint.  A sweep is
 * the rounds r = 0 .. ceil(log2(K/4)) - 1 in that order; `sweeps` sweeps run.
 *
 * Arithmetic, fixed so that the result is unique: everything in binary64; a
 * row contributes the sum of its two largest magnitudes (one addition); the
 * rows are added in 256 interleaved partial sums (row m into partial m mod
 * 256, in row order) which are then added as a balanced binary tree over
 * neighbours (partial j + partial j+1, then j + j+2, ...); the two scores of a
 * way are added last.
 *
 * perm: in/out, K entries, a permutation of 0 .. K-1 (else 2).
 */
static double search_magnitude(const void *A, long i, int t)
{
    double x = elem_to_double(A, i, t);
    return isnan(x) ? INFINITY : fabs(x);
}

static double search_group_score(const void *A, long M, long K, int t, const int32_t col[4])
{
    double partial[256];
    for (int j = 0; j < 256; ++j)
        partial[j] = 0.0;
    for (long m = 0; m < M; ++m) {
        double first = 0.0, second = 0.0; /* the two largest of the four magnitudes */
        for (int i = 0; i < 4; ++i) {
            double x = search_magnitude(A, m * K + col[i], t);
            if (x > first) {
                second = first;
                first = x;
            } else if (x > second) {
                second = x;
            }
        }
        partial[m % 256] += first + second;
    }
    for (int w = 1; w < 256; w *= 2)
        for (int j = 0; j < 256; j += 2 * w)
            partial[j] += partial[j + w];
    return partial[0];
}

int sp24o_permute_search(const void *A, int32_t *perm, long M, long K, int t, int sweeps)
{
    if (esize(t) == 0 || K % 4 || sweeps < 0)
        return 1;
    char *seen = (char *)calloc((size_t)(K > 0 ? K : 1), 1);
    if (!seen)
        return 3;
    for (long k = 0; k < K; ++k) {
        if (perm[k] < 0 || perm[k] >= K || seen[perm[k]]) {
            free(seen);
            return 2;
        }
        seen[perm[k]] = 1;
    }
    free(seen);
    const long G = K / 4;
    int rounds = 0;
    while (((long)1 << rounds) < G)
        ++rounds;
    for (int sweep = 0; sweep < sweeps; ++sweep)
        for (int r = 0; r < rounds; ++r) {
            const long step = (long)1 << r;
#pragma omp parallel for schedule(dynamic)
            for (long g = 0; g < G; ++g) {
                const long h = g + step;
                if ((g & step) || h >= G)
                    continue;
                int32_t col[8];
                for (int i = 0; i < 4; ++i) {
                    col[i] = perm[4 * g + i];
                    col[4 + i] = perm[4 * h + i];
                }
                int best[8] = {0, 1, 2, 3, 4, 5, 6, 7}; /* positions: first four -> g, last four -> h */
                double best_sum = 0.0;
                int have = 0;
                for (int a = 1; a < 8; ++a)
                    for (int b = a + 1; b < 8; ++b)
                        for (int c = b + 1; c < 8; ++c) {
                            int way[8], n0 = 0, n1 = 4;
                            for (int p = 0; p < 8; ++p) {
                                if (p == 0 || p == a || p == b || p == c)
                                    way[n0++] = p;
                                else
                                    way[n1++] = p;
                            }
                            int32_t c0[4], c1[4];
                            for (int i = 0; i < 4; ++i) {
                                c0[i] = col[way[i]];
                                c1[i] = col[way[4 + i]];
                            }
                            double sum = search_group_score(A, M, K, t, c0) + search_group_score(A, M, K, t, c1);
                            if (!have || sum > best_sum) {
                                have = 1;
                                best_sum = sum;
                                memcpy(best, way, sizeof way);
                            }
                        }
                for (int i = 0; i < 4; ++i) {
                    perm[4 * g + i] = col[best[i]];
                    perm[4 * h + i] = col[best[4 + i]];
                }
            }
        }
    return 0;
}

/* number of OpenMP threads the row loops use from now on (n >= 1); returns the previous maximum */
int sp24o_set_threads(int n)
{
#ifdef _OPENMP
    int before = omp_get_max_threads();
    if (n >= 1)
        omp_set_num_threads(n);
    return before;
#else
    (void)n;
    return 1;
#endif
}

int sp24o_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
