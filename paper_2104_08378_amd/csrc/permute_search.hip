// Search for a column order under which 2:4 pruning keeps more magnitude (Sec. 4.1, Step 2; Fig. 6).
//
// The paper states the aim and leaves the method to a later publication; the method here is this library's own,
// chosen so that every step is independent work for a whole chip and the result is unique:
//
//   * the order is read as K/4 groups of four columns; the score of a group is the magnitude pruning keeps in it,
//     the sum over the rows of the row's two largest magnitudes among its four columns (NaN counts as +infinity);
//   * a step takes two groups g < h -- eight columns, positions 0..3 those of g -- and tries the 35 ways of dealing
//     them out as two groups of four: a way is the three positions a < b < c that share a group with position 0,
//     ways are visited in lexicographic order of (a, b, c), the first being the present arrangement, and a later
//     way wins only with a strictly higher sum of its two scores.  The winner is written back with position 0's
//     group in g and the other in h, each in ascending position;
//   * round r pairs every group whose bit r is clear with the group 2^r further on (where that exists): the pairs
//     of a round are disjoint, one workgroup takes one pair, and a round is one launch.  A sweep is the rounds
//     r = 0 .. ceil(log2(K/4)) - 1.
//
// Arithmetic (fixed, so that the order found does not depend on the machine): binary64 throughout; a row
// contributes the sum of its two largest magnitudes; the 256 lanes of the workgroup add the rows m = lane, lane +
// 256, ... in row order, and the 256 partial sums are added as a balanced binary tree over neighbours -- the
// butterfly below inside a wavefront (both partners form the same sum: addition commutes), then wavefronts 0 + 1,
// 2 + 3, and those two.  The two scores of a way are added last.  For int8 every sum is an exact integer.
//
// A row's two largest magnitudes among four columns are the largest of the six pair sums of those columns (the
// rounding of a sum is monotone, so the largest rounded pair sum is the rounded sum of the two largest): the
// kernel forms the 28 pair sums of the eight columns once per row and takes 70 maxima of six, one per group of
// four that can be formed.
#include "common.hpp"
#include "launch.hpp"

namespace sp24 {

namespace {

// the 70 sets of four out of eight positions in lexicographic order; the 35 that hold position 0 come first
struct FourOfEight {
    uint8_t pos[70][4];
    uint8_t complement[70];   // index of the set of the other four positions
};
constexpr FourOfEight make_four_of_eight()
{
    FourOfEight t{};
    int n = 0;
    for (int a = 0; a < 8; ++a)
        for (int b = a + 1; b < 8; ++b)
            for (int c = b + 1; c < 8; ++c)
                for (int d = c + 1; d < 8; ++d) {
                    t.pos[n][0] = (uint8_t)a;
                    t.pos[n][1] = (uint8_t)b;
                    t.pos[n][2] = (uint8_t)c;
                    t.pos[n][3] = (uint8_t)d;
                    ++n;
                }
    for (int i = 0; i < 70; ++i) {
        const unsigned mine = (1u << t.pos[i][0]) | (1u << t.pos[i][1]) | (1u << t.pos[i][2]) | (1u << t.pos[i][3]);
        for (int j = 0; j < 70; ++j) {
            const unsigned other = (1u << t.pos[j][0]) | (1u << t.pos[j][1]) | (1u << t.pos[j][2]) | (1u << t.pos[j][3]);
            if ((mine ^ other) == 0xFFu) t.complement[i] = (uint8_t)j;
        }
    }
    return t;
}

// magnitude of element `bits` as the type the row sums are formed in
template <int DT>
__device__ __forceinline__ auto search_magnitude(uint32_t bits)
{
    if constexpr (DT == SP24_I8) {
        const int v = (int)(int8_t)bits;
        return v < 0 ? -v : v;
    } else if constexpr (DT == SP24_F8) {
        return (double)magnitude_f8(bits);
    } else {
        float f;
        if constexpr (DT == SP24_F16) f = (float)__builtin_bit_cast(_Float16, (uint16_t)(bits & 0x7FFFu));
        else f = __uint_as_float((bits & 0x7FFFu) << 16);
        return (f != f) ? (double)__builtin_inff() : (double)f;
    }
}

template <typename T>
__device__ __forceinline__ T larger(T a, T b) { return a > b ? a : b; }

} // namespace

template <int DT>
__global__ __launch_bounds__(256) void k_permute_search_round(const uint8_t* __restrict__ A, int32_t* perm, int64_t M, int64_t K,
                                                              int64_t lda_bytes, int bit, int64_t G)
{
    constexpr int ES = is8<DT> ? 1 : 2;
    using sum_t = typename std::conditional<DT == SP24_I8, int, double>::type;
    constexpr FourOfEight sets = make_four_of_eight();
    __shared__ double part[4][70];
    __shared__ int winner;

    // pair number -> g (bit `bit` clear) and h = g + 2^bit
    const int64_t p = blockIdx.x, step = (int64_t)1 << bit;
    const int64_t g = ((p >> bit) << (bit + 1)) | (p & (step - 1)), h = g | step;
    if (h >= G) return;
    int64_t off[8];                                            // byte offsets of the eight columns in a row
    int32_t col[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t c = (uint32_t)perm[4 * (i < 4 ? g : h) + (i & 3)];
        col[i] = c < (uint64_t)K ? (int32_t)c : 0;            // an entry outside 0 .. K-1 reads column 0, never out of bounds
        off[i] = (int64_t)col[i] * ES;
    }

    sum_t acc[70];
#pragma unroll
    for (int s = 0; s < 70; ++s) acc[s] = 0;
    for (int64_t m = threadIdx.x; m < M; m += 256) {
        const uint8_t* row = A + m * lda_bytes;
        sum_t x[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t bits;
            if constexpr (ES == 1) bits = row[off[i]];
            else bits = *reinterpret_cast<const uint16_t*>(row + off[i]);
            x[i] = search_magnitude<DT>(bits);
        }
        sum_t pair[8][8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = i + 1; j < 8; ++j) pair[i][j] = x[i] + x[j];
#pragma unroll
        for (int s = 0; s < 70; ++s) {
            const int a = sets.pos[s][0], b = sets.pos[s][1], c = sets.pos[s][2], d = sets.pos[s][3];
            acc[s] += larger(larger(larger(pair[a][b], pair[c][d]), larger(pair[a][c], pair[b][d])), larger(pair[a][d], pair[b][c]));
        }
    }

    // the 256 partial sums as a binary tree over neighbours
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int s = 0; s < 70; ++s) {
        double v = (double)acc[s];
#pragma unroll
        for (int w = 1; w < 64; w *= 2) v = v + __shfl_xor(v, w, 64);
        if (lane == 0) part[wave][s] = v;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double best = 0.0;
        int arg = 0;
        for (int k = 0; k < 35; ++k) {
            const int o = sets.complement[k];
            const double mine = (part[0][k] + part[1][k]) + (part[2][k] + part[3][k]);
            const double other = (part[0][o] + part[1][o]) + (part[2][o] + part[3][o]);
            const double sum = mine + other;
            if (k == 0 || sum > best) {
                best = sum;
                arg = k;
            }
        }
        winner = arg;
    }
    __syncthreads();
    const int arg = winner;
    if (arg != 0 && threadIdx.x < 8) {
        // position threadIdx.x of the new arrangement: the winner's four positions, then the other four, ascending
        const int i = threadIdx.x;
        const int src = i < 4 ? sets.pos[arg][i] : sets.pos[sets.complement[arg]][i - 4];
        int32_t c = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) c = (src == j) ? col[j] : c;
        perm[4 * (i < 4 ? g : h) + (i & 3)] = c;
    }
}

sp24_status launch_permute_search(const void* A, int32_t* perm, int64_t M, int64_t K, int64_t lda, sp24_dtype t, int sweeps, hipStream_t st)
{
    const int64_t G = K / 4;
    int rounds = 0;
    while (((int64_t)1 << rounds) < G) ++rounds;
    if (M == 0 || rounds == 0) return SP24_OK;
    const int es = esize_of(t);
    const dim3 grid((unsigned)(((int64_t)1 << rounds) / 2)), block(256);
    const uint8_t* a = static_cast<const uint8_t*>(A);
    for (int sweep = 0; sweep < sweeps; ++sweep)
        for (int r = 0; r < rounds; ++r) {
            if (t == SP24_F16) k_permute_search_round<SP24_F16><<<grid, block, 0, st>>>(a, perm, M, K, lda * es, r, G);
            else if (t == SP24_BF16) k_permute_search_round<SP24_BF16><<<grid, block, 0, st>>>(a, perm, M, K, lda * es, r, G);
            else if (t == SP24_F8) k_permute_search_round<SP24_F8><<<grid, block, 0, st>>>(a, perm, M, K, lda * es, r, G);
            else k_permute_search_round<SP24_I8><<<grid, block, 0, st>>>(a, perm, M, K, lda * es, r, G);
            if (hipGetLastError() != hipSuccess) return SP24_ERR_LAUNCH;
        }
    return SP24_OK;
}

} // namespace sp24
