// Prune / compress / decompress kernels: one streaming pass each, HBM-bound.
//
// Sec. 3.1 notes that the fixed 2-of-4 structure needs no indirection: the
// position of every kept value in memory follows from the compression rate
// alone.  That is what lets each lane below work on a fixed 16..64 byte piece
// of a row with full-width loads and stores and no inter-lane traffic.
#include "common.hpp"
#include "launch.hpp"

#include <type_traits>

namespace sp24 {

// ---- per-group arithmetic ------------------------------------------------

// 16-bit: a group is two dwords (x0 | x1<<16, x2 | x3<<16).
template <int DT>
__device__ __forceinline__ uint32_t mask16(uint32_t w0, uint32_t w1)
{
    return keep_mask(mag_key16<DT>(w0), mag_key16<DT>(w0 >> 16), mag_key16<DT>(w1), mag_key16<DT>(w1 >> 16));
}

// int8: a group is one dword.
__device__ __forceinline__ uint32_t mask8(uint32_t w)
{
    return keep_mask(mag_key8(w & 0xFFu), mag_key8((w >> 8) & 0xFFu), mag_key8((w >> 16) & 0xFFu), mag_key8(w >> 24));
}

// keep mask of a recorded code pos0 | pos1 << 2 (any 4-bit value gives a mask inside the group)
__device__ __forceinline__ uint32_t mask_of_code(uint32_t code)
{
    return (1u << (code & 3u)) | (1u << ((code >> 2) & 3u));
}

__device__ __forceinline__ void prune16(uint32_t& w0, uint32_t& w1, uint32_t m)
{
    w0 &= ((m & 1u) ? 0xFFFFu : 0u) | ((m & 2u) ? 0xFFFF0000u : 0u);
    w1 &= ((m & 4u) ? 0xFFFFu : 0u) | ((m & 8u) ? 0xFFFF0000u : 0u);
}

__device__ __forceinline__ uint32_t prune8(uint32_t w, uint32_t m)
{
    return w & (((m & 1u) ? 0xFFu : 0u) | ((m & 2u) ? 0xFF00u : 0u) | ((m & 4u) ? 0xFF0000u : 0u) | ((m & 8u) ? 0xFF000000u : 0u));
}

// the two survivors in column order, packed low/high
__device__ __forceinline__ uint32_t pack16(uint32_t w0, uint32_t w1, uint32_t m)
{
    uint32_t x0 = w0 & 0xFFFFu, x1 = w0 >> 16, x2 = w1 & 0xFFFFu, x3 = w1 >> 16;
    uint32_t first = (m & 1u) ? x0 : (m & 2u) ? x1 : x2;
    uint32_t second = (m & 8u) ? x3 : (m & 4u) ? x2 : x1;
    return first | (second << 16);
}

__device__ __forceinline__ uint32_t pack8(uint32_t w, uint32_t m)
{
    uint32_t x0 = w & 0xFFu, x1 = (w >> 8) & 0xFFu, x2 = (w >> 16) & 0xFFu, x3 = w >> 24;
    uint32_t first = (m & 1u) ? x0 : (m & 2u) ? x1 : x2;
    uint32_t second = (m & 8u) ? x3 : (m & 4u) ? x2 : x1;
    return first | (second << 8);
}

// scatter two values back by a 4-bit code (pos0 | pos1 << 2)
__device__ __forceinline__ void unpack16(uint32_t pair, uint32_t code, uint32_t& w0, uint32_t& w1)
{
    uint32_t p0 = code & 3u, p1 = (code >> 2) & 3u;
    uint32_t v0 = pair & 0xFFFFu, v1 = pair >> 16;
    uint32_t x0 = (p0 == 0u) ? v0 : 0u;
    uint32_t x1 = (p0 == 1u) ? v0 : (p1 == 1u) ? v1 : 0u;
    uint32_t x2 = (p0 == 2u) ? v0 : (p1 == 2u) ? v1 : 0u;
    uint32_t x3 = (p1 == 3u) ? v1 : 0u;
    w0 = x0 | (x1 << 16);
    w1 = x2 | (x3 << 16);
}

__device__ __forceinline__ uint32_t unpack8(uint32_t pair, uint32_t code)
{
    uint32_t p0 = code & 3u, p1 = (code >> 2) & 3u;
    uint32_t v0 = pair & 0xFFu, v1 = (pair >> 8) & 0xFFu;
    uint32_t x0 = (p0 == 0u) ? v0 : 0u;
    uint32_t x1 = (p0 == 1u) ? v0 : (p1 == 1u) ? v1 : 0u;
    uint32_t x2 = (p0 == 2u) ? v0 : (p1 == 2u) ? v1 : 0u;
    uint32_t x3 = (p1 == 3u) ? v1 : 0u;
    return x0 | (x1 << 8) | (x2 << 16) | (x3 << 24);
}

// The codes of the 16-byte piece c of row m (4 groups for int8, 2 for 16-bit types) from stored metadata, in the
// low bits of the result, group 0 first.  K8 = K/8 (canonical row length in bytes), KB = K/64 (tiles per row block).
template <int DT, int LAYOUT>
__device__ __forceinline__ uint32_t stored_codes(const uint8_t* meta, int64_t m, int64_t c, int64_t K8, int64_t KB)
{
    constexpr int ES = (DT == SP24_I8) ? 1 : 2;
    constexpr int GROUPS = 4 / ES;                       // groups per 16-byte piece
    if constexpr (LAYOUT == SP24_LAYOUT_CANONICAL) {
        if constexpr (DT == SP24_I8) return *reinterpret_cast<const uint16_t*>(meta + m * K8 + c * 2);
        else return meta[m * K8 + c];
    } else {
        const int64_t e0 = c * (16 / ES);                // first column of the piece
        const int64_t kb = e0 >> 6;
        const uint32_t h = (uint32_t)(e0 >> 5) & 1u, g0 = (uint32_t)(e0 & 31) >> 2;
        const uint32_t word = reinterpret_cast<const uint32_t*>(meta)[((m >> 5) * KB + kb) * 64 + (m & 31) + 32 * h];
        return (word >> (4 * g0)) & ((1u << (4 * GROUPS)) - 1u);
    }
}

// ---- prune: dense -> dense ----------------------------------------------
// One lane per 16-byte piece of a row.  FIXED: the keep pattern comes from stored metadata instead of the
// magnitudes (Sec. 4.1 Step 3: removed weights stay zero while the network is retrained).
template <int DT, bool FIXED, int LAYOUT>
__global__ __launch_bounds__(256) void k_prune(const uint8_t* __restrict__ A, uint8_t* __restrict__ P, int64_t M,
                                               int64_t chunks_per_row, int64_t lda_bytes, int64_t ldp_bytes,
                                               const uint8_t* __restrict__ meta, int64_t K8, int64_t KB)
{
    int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= M * chunks_per_row) return;
    int64_t m = id / chunks_per_row, c = id - m * chunks_per_row;
    uint4v w = *reinterpret_cast<const uint4v*>(A + m * lda_bytes + c * 16);
    uint32_t codes = 0;
    if constexpr (FIXED) codes = stored_codes<DT, LAYOUT>(meta, m, c, K8, KB);
    if constexpr (DT == SP24_I8) {
        for (int g = 0; g < 4; ++g) w[g] = prune8(w[g], FIXED ? mask_of_code((codes >> (4 * g)) & 0xFu) : mask8(w[g]));
    } else {
        for (int g = 0; g < 2; ++g) {
            uint32_t w0 = w[2 * g], w1 = w[2 * g + 1];
            prune16(w0, w1, FIXED ? mask_of_code((codes >> (4 * g)) & 0xFu) : mask16<DT>(w0, w1));
            w[2 * g] = w0;
            w[2 * g + 1] = w1;
        }
    }
    *reinterpret_cast<uint4v*>(P + m * ldp_bytes + c * 16) = w;
}

// ---- patterns that also hold for the transposed matrix (Sec. 6) -----------
// Exhaustive search per aligned 4x4 block over the 90 patterns with two kept entries in every row and column;
// the one with the highest sum of kept magnitudes stays.  One lane per block.  To be reproducible bit for bit the
// sum of a pattern is ((r0 + r1) + r2) + r3, r_i the sum of row i's two kept magnitudes (lower column first), in
// double for the 16-bit types and in integers for int8; NaN counts as +infinity; patterns are visited in
// lexicographic order of their row pairs, pairs ordered (0,1) (0,2) (0,3) (1,2) (1,3) (2,3); a later pattern
// replaces the best only with a strictly higher sum.
struct PatternTable {
    uint8_t pair[90][4];
};
constexpr PatternTable make_pattern_table()
{
    constexpr int c0[6] = {0, 0, 0, 1, 1, 2}, c1[6] = {1, 2, 3, 2, 3, 3};
    PatternTable t{};
    int n = 0;
    for (int p0 = 0; p0 < 6; ++p0)
        for (int p1 = 0; p1 < 6; ++p1)
            for (int p2 = 0; p2 < 6; ++p2)
                for (int p3 = 0; p3 < 6; ++p3) {
                    int count[4] = {0, 0, 0, 0};
                    const int p[4] = {p0, p1, p2, p3};
                    for (int i = 0; i < 4; ++i) { ++count[c0[p[i]]]; ++count[c1[p[i]]]; }
                    if (count[0] == 2 && count[1] == 2 && count[2] == 2 && count[3] == 2) {
                        for (int i = 0; i < 4; ++i) t.pair[n][i] = (uint8_t)p[i];
                        ++n;
                    }
                }
    return t;
}

template <int DT>
__global__ __launch_bounds__(256) void k_prune_transposable(const uint8_t* __restrict__ A, uint8_t* __restrict__ P, int64_t M4,
                                                            int64_t K4, int64_t lda_bytes, int64_t ldp_bytes)
{
    constexpr int ES = (DT == SP24_I8) ? 1 : 2;
    using sum_t = typename std::conditional<DT == SP24_I8, int, double>::type;
    constexpr PatternTable table = make_pattern_table();
    constexpr int c0[6] = {0, 0, 0, 1, 1, 2}, c1[6] = {1, 2, 3, 2, 3, 3};
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= M4 * K4) return;
    const int64_t bm = id / K4, bk = id - bm * K4;
    uint32_t raw[4][2];                                   // a row of the block: 4 or 8 bytes
    sum_t r[4][6];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint8_t* src = A + (bm * 4 + i) * lda_bytes + bk * (4 * ES);
        sum_t mag[4];
        if constexpr (DT == SP24_I8) {
            raw[i][0] = *reinterpret_cast<const uint32_t*>(src);
            raw[i][1] = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) mag[j] = (int)mag_key8((raw[i][0] >> (8 * j)) & 0xFFu);
        } else {
            const uint2v w = *reinterpret_cast<const uint2v*>(src);
            raw[i][0] = w[0];
            raw[i][1] = w[1];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t bits = (raw[i][j >> 1] >> (16 * (j & 1))) & 0x7FFFu;      // sign cleared
                float f;
                if constexpr (DT == SP24_F16) f = (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
                else f = __uint_as_float(bits << 16);
                mag[j] = (f != f) ? (double)__builtin_inff() : (double)f;
            }
        }
#pragma unroll
        for (int p = 0; p < 6; ++p) r[i][p] = mag[c0[p]] + mag[c1[p]];
    }
    // pair indices of the winner, 3 bits per row
    uint32_t win = 0;
    if constexpr (DT == SP24_I8) {
        // Integer sums (at most 8 * 128) do not depend on the order of addition, so the rows are added in two halves
        // shared between patterns, and sum and pattern travel in one word: the sum above 12 bits that hold 4095 minus
        // the pattern's row pairs in visiting order (row 0's pair in the top three bits).  The largest word is the
        // largest sum and, among equal sums, the pattern visited first.
        int top[6][6], bottom[6][6];
#pragma unroll
        for (int p = 0; p < 6; ++p)
#pragma unroll
            for (int t = 0; t < 6; ++t) {
                top[p][t] = (r[0][p] + r[1][t]) << 12;
                bottom[p][t] = (r[2][p] + r[3][t]) << 12;
            }
        uint32_t best_word = 0;
#pragma unroll
        for (int e = 0; e < 90; ++e) {
            const uint32_t visit = (table.pair[e][0] << 9) | (table.pair[e][1] << 6) | (table.pair[e][2] << 3) | table.pair[e][3];
            const uint32_t word = (uint32_t)(top[table.pair[e][0]][table.pair[e][1]] + bottom[table.pair[e][2]][table.pair[e][3]]) + (4095u - visit);
            best_word = max(best_word, word);
        }
        const uint32_t visit = 4095u - (best_word & 4095u);
        win = (visit >> 9) | (((visit >> 6) & 7u) << 3) | (((visit >> 3) & 7u) << 6) | ((visit & 7u) << 9);
    } else {
        // sums in the stated order; r0 + r1 is shared by the patterns that agree in their first two rows, and the
        // winner's row pairs (constants of the unrolled loop) are carried along instead of its number
        sum_t top[6][6];
#pragma unroll
        for (int p = 0; p < 6; ++p)
#pragma unroll
            for (int t = 0; t < 6; ++t) top[p][t] = r[0][p] + r[1][t];
        sum_t best_sum = (sum_t)-1;
#pragma unroll
        for (int e = 0; e < 90; ++e) {
            const sum_t sum = (top[table.pair[e][0]][table.pair[e][1]] + r[2][table.pair[e][2]]) + r[3][table.pair[e][3]];
            const uint32_t packed = table.pair[e][0] | (table.pair[e][1] << 3) | (table.pair[e][2] << 6) | (table.pair[e][3] << 9);
            const bool better = sum > best_sum;
            best_sum = better ? sum : best_sum;
            win = better ? packed : win;
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t p = (win >> (3 * i)) & 7u;
        // columns of pair p: c0 = {0,0,0,1,1,2}, c1 = {1,2,3,2,3,3} as 2-bit fields of two constants
        const uint32_t k0 = (0x940u >> (2 * p)) & 3u, k1 = (0xFB9u >> (2 * p)) & 3u;
        const uint32_t keep = (1u << k0) | (1u << k1);
        uint8_t* dst = P + (bm * 4 + i) * ldp_bytes + bk * (4 * ES);
        if constexpr (DT == SP24_I8) {
            *reinterpret_cast<uint32_t*>(dst) = prune8(raw[i][0], keep);
        } else {
            uint32_t w0 = raw[i][0], w1 = raw[i][1];
            prune16(w0, w1, keep);
            uint2v w;
            w[0] = w0;
            w[1] = w1;
            *reinterpret_cast<uint2v*>(dst) = w;
        }
    }
}

// ---- compress, canonical layout -------------------------------------------
// One lane per 16 input bytes: 8 bytes of V and 1 (16-bit) or 2 (int8) bytes
// of metadata; consecutive lanes write consecutive addresses in both arrays.
// FIXED: the metadata is an input; the values at its recorded positions are gathered, nothing is selected.
template <int DT, bool FIXED>
__global__ __launch_bounds__(256) void k_compress_canon(const uint8_t* __restrict__ A, uint8_t* __restrict__ V,
                                                        uint8_t* __restrict__ meta, int64_t M, int64_t chunks_per_row,
                                                        int64_t lda_bytes)
{
    int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= M * chunks_per_row) return;
    int64_t m = id / chunks_per_row, c = id - m * chunks_per_row;
    uint4v w = *reinterpret_cast<const uint4v*>(A + m * lda_bytes + c * 16);
    uint2v v;
    if constexpr (DT == SP24_I8) {
        uint32_t m0, m1, m2, m3;
        if constexpr (FIXED) {
            const uint32_t codes = *reinterpret_cast<const uint16_t*>(meta + id * 2);
            m0 = mask_of_code(codes & 0xFu), m1 = mask_of_code((codes >> 4) & 0xFu);
            m2 = mask_of_code((codes >> 8) & 0xFu), m3 = mask_of_code(codes >> 12);
        } else {
            m0 = mask8(w[0]), m1 = mask8(w[1]), m2 = mask8(w[2]), m3 = mask8(w[3]);
            uint32_t codes = code_of_mask(m0) | (code_of_mask(m1) << 4) | (code_of_mask(m2) << 8) | (code_of_mask(m3) << 12);
            *reinterpret_cast<uint16_t*>(meta + id * 2) = (uint16_t)codes; // rows are K/8 = 2*chunks bytes: id*2 is exact
        }
        v[0] = pack8(w[0], m0) | (pack8(w[1], m1) << 16);
        v[1] = pack8(w[2], m2) | (pack8(w[3], m3) << 16);
    } else {
        uint32_t m0, m1;
        if constexpr (FIXED) {
            const uint32_t codes = meta[id];
            m0 = mask_of_code(codes & 0xFu), m1 = mask_of_code(codes >> 4);
        } else {
            m0 = mask16<DT>(w[0], w[1]), m1 = mask16<DT>(w[2], w[3]);
            meta[id] = (uint8_t)(code_of_mask(m0) | (code_of_mask(m1) << 4)); // rows are K/8 = chunks bytes
        }
        v[0] = pack16(w[0], w[1], m0);
        v[1] = pack16(w[2], w[3], m1);
    }
    *reinterpret_cast<uint2v*>(V + id * 8) = v; // V rows are 8 * chunks bytes in both cases
}

// ---- compress, tiled layout -----------------------------------------------
// One lane per slot: 32 consecutive elements of one row (half of a 32x64
// tile).  A wavefront covers one whole tile, so its V and metadata stores are
// contiguous runs of 1 KiB and 256 bytes.
template <int DT, bool FIXED>
__global__ __launch_bounds__(256) void k_compress_tiled(const uint8_t* __restrict__ A, uint8_t* __restrict__ V,
                                                        uint32_t* __restrict__ meta, int64_t tiles, int64_t KB,
                                                        int64_t lda_bytes)
{
    int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t tile = id >> 6;
    if (tile >= tiles) return;
    uint32_t slot = (uint32_t)id & 63u, r = slot & 31u, h = slot >> 5;
    int64_t rb = tile / KB, kb = tile - rb * KB;
    int64_t m = rb * 32 + r;
    uint32_t codes = 0;
    uint32_t given = 0;
    if constexpr (FIXED) given = meta[tile * 64 + slot];
    if constexpr (DT == SP24_I8) {
        const uint4v* src = reinterpret_cast<const uint4v*>(A + m * lda_bytes + kb * 64 + h * 32);
        uint4v v;
        for (int q = 0; q < 2; ++q) {
            uint4v w = src[q];
            uint32_t pk[4];
            for (int g = 0; g < 4; ++g) {
                uint32_t mk = FIXED ? mask_of_code((given >> (4 * (4 * q + g))) & 0xFu) : mask8(w[g]);
                pk[g] = pack8(w[g], mk);
                if constexpr (!FIXED) codes |= code_of_mask(mk) << (4 * (4 * q + g));
            }
            v[2 * q] = pk[0] | (pk[1] << 16);
            v[2 * q + 1] = pk[2] | (pk[3] << 16);
        }
        *reinterpret_cast<uint4v*>(V + (tile * 64 + slot) * 16) = v;
    } else {
        const uint4v* src = reinterpret_cast<const uint4v*>(A + m * lda_bytes + kb * 128 + h * 64);
        for (int s = 0; s < 2; ++s) {
            uint4v v;
            for (int q = 0; q < 2; ++q) {
                uint4v w = src[2 * s + q];
                const uint32_t gc = (given >> (8 * (2 * s + q))) & 0xFFu;
                uint32_t m0 = FIXED ? mask_of_code(gc & 0xFu) : mask16<DT>(w[0], w[1]);
                uint32_t m1 = FIXED ? mask_of_code(gc >> 4) : mask16<DT>(w[2], w[3]);
                v[2 * q] = pack16(w[0], w[1], m0);
                v[2 * q + 1] = pack16(w[2], w[3], m1);
                if constexpr (!FIXED) codes |= (code_of_mask(m0) | (code_of_mask(m1) << 4)) << (8 * (2 * s + q));
            }
            *reinterpret_cast<uint4v*>(V + ((tile * 2 + s) * 64 + slot) * 16) = v;
        }
    }
    if constexpr (!FIXED) meta[tile * 64 + slot] = codes;
}

// ---- decompress -----------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(256) void k_decompress_canon(const uint8_t* __restrict__ V, const uint8_t* __restrict__ meta,
                                                          uint8_t* __restrict__ P, int64_t M, int64_t chunks_per_row,
                                                          int64_t ldp_bytes)
{
    int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= M * chunks_per_row) return;
    int64_t m = id / chunks_per_row, c = id - m * chunks_per_row;
    uint2v v = *reinterpret_cast<const uint2v*>(V + id * 8);
    uint4v w;
    if constexpr (DT == SP24_I8) {
        uint32_t codes = *reinterpret_cast<const uint16_t*>(meta + id * 2);
        w[0] = unpack8(v[0] & 0xFFFFu, codes & 0xFu);
        w[1] = unpack8(v[0] >> 16, (codes >> 4) & 0xFu);
        w[2] = unpack8(v[1] & 0xFFFFu, (codes >> 8) & 0xFu);
        w[3] = unpack8(v[1] >> 16, codes >> 12);
    } else {
        uint32_t codes = meta[id];
        uint32_t a, b;
        unpack16(v[0], codes & 0xFu, a, b);
        w[0] = a; w[1] = b;
        unpack16(v[1], codes >> 4, a, b);
        w[2] = a; w[3] = b;
    }
    *reinterpret_cast<uint4v*>(P + m * ldp_bytes + c * 16) = w;
}

template <int DT>
__global__ __launch_bounds__(256) void k_decompress_tiled(const uint8_t* __restrict__ V, const uint32_t* __restrict__ meta,
                                                          uint8_t* __restrict__ P, int64_t tiles, int64_t KB,
                                                          int64_t ldp_bytes)
{
    int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t tile = id >> 6;
    if (tile >= tiles) return;
    uint32_t slot = (uint32_t)id & 63u, r = slot & 31u, h = slot >> 5;
    int64_t rb = tile / KB, kb = tile - rb * KB;
    int64_t m = rb * 32 + r;
    uint32_t codes = meta[tile * 64 + slot];
    if constexpr (DT == SP24_I8) {
        uint4v v = *reinterpret_cast<const uint4v*>(V + (tile * 64 + slot) * 16);
        uint4v* dst = reinterpret_cast<uint4v*>(P + m * ldp_bytes + kb * 64 + h * 32);
        for (int q = 0; q < 2; ++q) {
            uint4v w;
            w[0] = unpack8(v[2 * q] & 0xFFFFu, (codes >> (16 * q)) & 0xFu);
            w[1] = unpack8(v[2 * q] >> 16, (codes >> (16 * q + 4)) & 0xFu);
            w[2] = unpack8(v[2 * q + 1] & 0xFFFFu, (codes >> (16 * q + 8)) & 0xFu);
            w[3] = unpack8(v[2 * q + 1] >> 16, (codes >> (16 * q + 12)) & 0xFu);
            dst[q] = w;
        }
    } else {
        uint4v* dst = reinterpret_cast<uint4v*>(P + m * ldp_bytes + kb * 128 + h * 64);
        for (int s = 0; s < 2; ++s) {
            uint4v v = *reinterpret_cast<const uint4v*>(V + ((tile * 2 + s) * 64 + slot) * 16);
            for (int q = 0; q < 2; ++q) {
                uint32_t cc = (codes >> (8 * (2 * s + q))) & 0xFFu;
                uint4v w;
                uint32_t a, b;
                unpack16(v[2 * q], cc & 0xFu, a, b);
                w[0] = a; w[1] = b;
                unpack16(v[2 * q + 1], cc >> 4, a, b);
                w[2] = a; w[3] = b;
                dst[2 * s + q] = w;
            }
        }
    }
}

// ---- launchers ------------------------------------------------------------
static inline unsigned blocks_for(int64_t items) { return (unsigned)((items + 255) / 256); }

// meta == nullptr: select by magnitude; else keep the pattern that `meta` (in layout l) records
template <int DT>
static void run_prune(const void* A, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, const void* meta, sp24_layout l,
                      hipStream_t st)
{
    constexpr int64_t es = (DT == SP24_I8) ? 1 : 2;
    const int64_t cpr = K * es / 16;
    const dim3 grid(blocks_for(M * cpr));
    const uint8_t *a = (const uint8_t*)A, *mt = (const uint8_t*)meta;
    uint8_t* p = (uint8_t*)P;
    if (!meta) k_prune<DT, false, SP24_LAYOUT_CANONICAL><<<grid, 256, 0, st>>>(a, p, M, cpr, lda * es, ldp * es, nullptr, 0, 0);
    else if (l == SP24_LAYOUT_CANONICAL)
        k_prune<DT, true, SP24_LAYOUT_CANONICAL><<<grid, 256, 0, st>>>(a, p, M, cpr, lda * es, ldp * es, mt, K / 8, K / 64);
    else k_prune<DT, true, SP24_LAYOUT_TILED><<<grid, 256, 0, st>>>(a, p, M, cpr, lda * es, ldp * es, mt, K / 8, K / 64);
}

// fixed: `meta` is an input and only V is written
template <int DT, bool FIXED>
static void run_compress(const void* A, void* V, void* meta, int64_t M, int64_t K, int64_t lda, sp24_layout l, hipStream_t st)
{
    constexpr int64_t es = (DT == SP24_I8) ? 1 : 2;
    if (l == SP24_LAYOUT_CANONICAL) {
        int64_t cpr = K * es / 16;
        k_compress_canon<DT, FIXED><<<blocks_for(M * cpr), 256, 0, st>>>((const uint8_t*)A, (uint8_t*)V, (uint8_t*)meta, M, cpr, lda * es);
    } else {
        int64_t KB = K / 64, tiles = (M / 32) * KB;
        k_compress_tiled<DT, FIXED><<<blocks_for(tiles * 64), 256, 0, st>>>((const uint8_t*)A, (uint8_t*)V, (uint32_t*)meta, tiles, KB, lda * es);
    }
}

template <int DT>
static void run_decompress(const void* V, const void* meta, void* P, int64_t M, int64_t K, int64_t ldp, sp24_layout l, hipStream_t st)
{
    constexpr int64_t es = (DT == SP24_I8) ? 1 : 2;
    if (l == SP24_LAYOUT_CANONICAL) {
        int64_t cpr = K * es / 16;
        k_decompress_canon<DT><<<blocks_for(M * cpr), 256, 0, st>>>((const uint8_t*)V, (const uint8_t*)meta, (uint8_t*)P, M, cpr, ldp * es);
    } else {
        int64_t KB = K / 64, tiles = (M / 32) * KB;
        k_decompress_tiled<DT><<<blocks_for(tiles * 64), 256, 0, st>>>((const uint8_t*)V, (const uint32_t*)meta, (uint8_t*)P, tiles, KB, ldp * es);
    }
}

static sp24_status launch_result() { return hipGetLastError() == hipSuccess ? SP24_OK : SP24_ERR_LAUNCH; }

sp24_status launch_prune(const void* A, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, sp24_dtype t, hipStream_t st)
{
    if (M * K == 0) return SP24_OK;
    if (t == SP24_F16) run_prune<SP24_F16>(A, P, M, K, lda, ldp, nullptr, SP24_LAYOUT_CANONICAL, st);
    else if (t == SP24_BF16) run_prune<SP24_BF16>(A, P, M, K, lda, ldp, nullptr, SP24_LAYOUT_CANONICAL, st);
    else run_prune<SP24_I8>(A, P, M, K, lda, ldp, nullptr, SP24_LAYOUT_CANONICAL, st);
    return launch_result();
}

sp24_status launch_prune_transposable(const void* A, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, sp24_dtype t, hipStream_t st)
{
    if (M * K == 0) return SP24_OK;
    const int64_t M4 = M / 4, K4 = K / 4;
    const dim3 grid(blocks_for(M4 * K4));
    const uint8_t* a = (const uint8_t*)A;
    uint8_t* p = (uint8_t*)P;
    if (t == SP24_F16) k_prune_transposable<SP24_F16><<<grid, 256, 0, st>>>(a, p, M4, K4, lda * 2, ldp * 2);
    else if (t == SP24_BF16) k_prune_transposable<SP24_BF16><<<grid, 256, 0, st>>>(a, p, M4, K4, lda * 2, ldp * 2);
    else k_prune_transposable<SP24_I8><<<grid, 256, 0, st>>>(a, p, M4, K4, lda, ldp);
    return launch_result();
}

sp24_status launch_mask_apply(const void* W, const void* meta, void* P, int64_t M, int64_t K, int64_t ldw, int64_t ldp, sp24_dtype t,
                              sp24_layout l, hipStream_t st)
{
    if (M * K == 0) return SP24_OK;
    if (t == SP24_F16) run_prune<SP24_F16>(W, P, M, K, ldw, ldp, meta, l, st);
    else if (t == SP24_BF16) run_prune<SP24_BF16>(W, P, M, K, ldw, ldp, meta, l, st);
    else run_prune<SP24_I8>(W, P, M, K, ldw, ldp, meta, l, st);
    return launch_result();
}

sp24_status launch_compress_masked(const void* W, const void* meta, void* V, int64_t M, int64_t K, int64_t ldw, sp24_dtype t,
                                   sp24_layout l, hipStream_t st)
{
    if (M * K == 0) return SP24_OK;
    void* mt = const_cast<void*>(meta);   // read only in the fixed-mask kernels
    if (t == SP24_F16) run_compress<SP24_F16, true>(W, V, mt, M, K, ldw, l, st);
    else if (t == SP24_BF16) run_compress<SP24_BF16, true>(W, V, mt, M, K, ldw, l, st);
    else run_compress<SP24_I8, true>(W, V, mt, M, K, ldw, l, st);
    return launch_result();
}

sp24_status launch_compress(const void* A, void* V, void* meta, int64_t M, int64_t K, int64_t lda, sp24_dtype t, sp24_layout l, hipStream_t st)
{
    if (M * K == 0) return SP24_OK;
    if (t == SP24_F16) run_compress<SP24_F16, false>(A, V, meta, M, K, lda, l, st);
    else if (t == SP24_BF16) run_compress<SP24_BF16, false>(A, V, meta, M, K, lda, l, st);
    else run_compress<SP24_I8, false>(A, V, meta, M, K, lda, l, st);
    return launch_result();
}

sp24_status launch_decompress(const void* V, const void* meta, void* P, int64_t M, int64_t K, int64_t ldp, sp24_dtype t, sp24_layout l, hipStream_t st)
{
    if (M * K == 0) return SP24_OK;
    if (t == SP24_F16) run_decompress<SP24_F16>(V, meta, P, M, K, ldp, l, st);
    else if (t == SP24_BF16) run_decompress<SP24_BF16>(V, meta, P, M, K, ldp, l, st);
    else run_decompress<SP24_I8>(V, meta, P, M, K, ldp, l, st);
    return launch_result();
}

} // namespace sp24
