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
// The kernels below are bound by their instruction count as much as by memory, so the selection is written on
// packed 16-bit halves (two elements of a group per instruction) and its result is turned into masks, positions
// and byte selectors by arithmetic rather than by compares and selects.
typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ s16x2 as_s16x2(uint32_t v) { return __builtin_bit_cast(s16x2, v); }
__device__ __forceinline__ u16x2 as_u16x2(uint32_t v) { return __builtin_bit_cast(u16x2, v); }
__device__ __forceinline__ uint32_t as_u32(s16x2 v) { return __builtin_bit_cast(uint32_t, v); }
__device__ __forceinline__ uint32_t as_u32(u16x2 v) { return __builtin_bit_cast(uint32_t, v); }
__device__ __forceinline__ uint32_t swap_halves(uint32_t v) { return __builtin_amdgcn_alignbit(v, v, 16); }
// The value as it is, but its origin hidden from the optimiser: a sign bit taken from a packed difference would
// otherwise be turned back into one 16-bit compare and select per element, several times the instructions.
__device__ __forceinline__ uint32_t opaque(uint32_t v)
{
    asm("" : "+v"(v));
    return v;
}
// (a & m) | (b & ~m): one v_bfi_b32
__device__ __forceinline__ uint32_t bit_select(uint32_t m, uint32_t a, uint32_t b) { return (a & m) | (b & ~m); }

// One-byte types: a group is one dword; two groups a and b are taken together, column i of both in the halves of one
// register (a in the low half), so that every step of the selection is one packed instruction for both groups
// and none moves data between halves.  Keys |x| * 4 + (3 - column) are distinct and order a group by (magnitude
// descending, column ascending); the two largest stay, i.e. those not below the second largest key t.
// Returned: key - t per column, negative (bit 15 of the half set) where the element is removed.
struct Sel8x2 {
    uint32_t s[4];
};
template <int DT>
__device__ __forceinline__ Sel8x2 select8x2(uint32_t wa, uint32_t wb)
{
    s16x2 k[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s16x2 x;
        if constexpr (DT == SP24_F8) {
            // 8-bit float: the bit pattern without its sign orders the magnitudes, the NaN pattern on top; byte i
            // of a and of b into the low bytes of the halves
            x = as_s16x2(__builtin_amdgcn_perm(wb, wa, 0x0C040C00u + 0x00010001u * i) & 0x007F007Fu);
        } else {
            // int8: byte i of a and of b into the high bytes of the halves (the low bytes cleared), then sign-extended
            x = as_s16x2(__builtin_amdgcn_perm(wb, wa, 0x040C000Cu + 0x01000100u * i)) >> 8;
            x = __builtin_elementwise_max(x, -x);             // |-128| = 128 fits the half
        }
        k[i] = (x << 2) + s16x2{(short)(3 - i), (short)(3 - i)};
    }
    // second largest of four = max(min of the pair maxima, max of the pair minima)
    const s16x2 m = __builtin_elementwise_min(__builtin_elementwise_max(k[0], k[1]), __builtin_elementwise_max(k[2], k[3]));
    const s16x2 l = __builtin_elementwise_max(__builtin_elementwise_min(k[0], k[1]), __builtin_elementwise_min(k[2], k[3]));
    const s16x2 t = __builtin_elementwise_max(m, l);
    Sel8x2 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r.s[i] = opaque(as_u32(k[i] - t));
    return r;
}

__device__ __forceinline__ void prune8x2(uint32_t& wa, uint32_t& wb, const Sel8x2& sel)
{
    uint32_t gone[4];                                          // 0xFFFF per removed element
#pragma unroll
    for (int i = 0; i < 4; ++i) gone[i] = as_u32(as_s16x2(sel.s[i]) >> 15);
    const uint32_t t01 = bit_select(0x00FF00FFu, gone[0], gone[1]), t23 = bit_select(0x00FF00FFu, gone[2], gone[3]);
    wa &= ~__builtin_amdgcn_perm(t23, t01, 0x05040100u);
    wb &= ~__builtin_amdgcn_perm(t23, t01, 0x07060302u);
}

// Two int8 groups: their survivors in column order (bytes 0-1 those of a, bytes 2-3 those of b) and their codes
// (bits 0-3 a, bits 4-7 b).  With d_i the removed flags (exactly two are set per group) the survivors sit at
// pos0 = d0 * (1 + d1) and pos1 = 3 - d3 * (1 + d2).
template <int DT>
__device__ __forceinline__ void compress8x2(uint32_t wa, uint32_t wb, uint32_t& values, uint32_t& codes)
{
    const Sel8x2 sel = select8x2<DT>(wa, wb);
    u16x2 d[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) d[i] = as_u16x2(sel.s[i]) >> 15;
    const u16x2 p0 = d[0] * d[1] + d[0];
    const u16x2 p1 = as_u16x2(as_u32(d[3] * d[2] + d[3]) ^ 0x00030003u);
    const uint32_t c = as_u32(p0 + (p1 << 2));                // (code of a, code of b)
    codes = (c | (c >> 12)) & 0xFFu;
    const uint32_t byte_sel = as_u32(p0 + (p1 << 8));          // v_perm selectors pos0, pos1 of a (low half) and b
    values = __builtin_amdgcn_perm(__builtin_amdgcn_perm(0u, wb, byte_sel >> 16), __builtin_amdgcn_perm(0u, wa, byte_sel), 0x05040100u);
}

// metadata code pos0 | pos1 << 2 (Sec. 3.1: 2 bits per kept value, ascending) from pos0 | pos1 << 16; bits above 3 are junk
__device__ __forceinline__ uint32_t code_bits(uint32_t z) { return z | (z >> 14); }
// the inverse for a stored code (any 4-bit value stays inside the group)
__device__ __forceinline__ uint32_t positions_of_code(uint32_t code) { return (code & 3u) | ((code & 0xCu) << 14); }

// the two survivors of an int8 group in column order in bytes 0 and 1 (bytes 2 and 3 are junk)
__device__ __forceinline__ uint32_t pack8(uint32_t w, uint32_t z) { return __builtin_amdgcn_perm(0u, w, z | (z >> 8)); }
// bytes 0-1 of a and of b side by side
__device__ __forceinline__ uint32_t low_halves(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }

// keep mask of a recorded code pos0 | pos1 << 2 (any 4-bit value gives a mask inside the group)
__device__ __forceinline__ uint32_t mask_of_code(uint32_t code)
{
    return (1u << (code & 3u)) | (1u << ((code >> 2) & 3u));
}
// a 4-bit keep mask as byte / halfword masks
__device__ __forceinline__ uint32_t prune8_by_mask(uint32_t w, uint32_t m)
{
    return w & (((m & 1u) ? 0xFFu : 0u) | ((m & 2u) ? 0xFF00u : 0u) | ((m & 4u) ? 0xFF0000u : 0u) | ((m & 8u) ? 0xFF000000u : 0u));
}
__device__ __forceinline__ void prune16_by_mask(uint32_t& w0, uint32_t& w1, uint32_t m)
{
    w0 &= ((m & 1u) ? 0xFFFFu : 0u) | ((m & 2u) ? 0xFFFF0000u : 0u);
    w1 &= ((m & 4u) ? 0xFFFFu : 0u) | ((m & 8u) ? 0xFFFF0000u : 0u);
}

// 16-bit types: a group is two dwords, (x0, x1) and (x2, x3).  Magnitude keys: the bit pattern without its sign,
// every NaN clamped to one key above infinity.  The 15-bit keys leave one spare bit per half, which orders equal
// magnitudes: 2k + 1 for x0 and x1, 2k for x2 and x3.  With the pairs A = {x0, x2} (low halves) and B = {x1, x3}
// (high halves) that bit makes the order inside a pair strict, and "an element of A outranks an element of B
// exactly when its key is >=" agrees with (magnitude descending, column ascending) for all four mixed pairs.
// With each pair sorted (hiA >= loA, hiB >= loB) the survivors are both of A when loA outranks hiB (p), both of B
// when loB outranks hiA (q), else hiA and hiB.  Returned: halfword masks, 0xFFFF where the element stays.
struct Keep16 {
    uint32_t k0, k1;
};
template <int DT>
__device__ __forceinline__ Keep16 select16(uint32_t w0, uint32_t w1)
{
    constexpr uint32_t cap = (((DT == SP24_F16) ? 0x7C00u : 0x7F80u) + 1u) * 0x00010001u;
    const u16x2 a = __builtin_elementwise_min(as_u16x2(w0 & 0x7FFF7FFFu), as_u16x2(cap));
    const u16x2 b = __builtin_elementwise_min(as_u16x2(w1 & 0x7FFF7FFFu), as_u16x2(cap));
    const u16x2 r0 = (a << 1) + u16x2{1, 1}, r1 = b << 1;
    const uint32_t hi = as_u32(__builtin_elementwise_max(r0, r1)), lo = as_u32(__builtin_elementwise_min(r0, r1));
    const u16x2 one = {1, 1}, zero = {0, 0};
    // c: 0xFFFF in a half where the element of (x0, x1) is the larger of its pair
    const uint32_t c = as_u32(zero - __builtin_elementwise_min(__builtin_elementwise_sub_sat(r0, r1), one));
    // (hiB - loA, loB - hiA), saturating at 0: p <=> the low half is 0, q <=> the high half is not
    const uint32_t x = __builtin_amdgcn_perm(lo, hi, 0x07060302u), y = __builtin_amdgcn_perm(lo, hi, 0x01000504u);
    const u16x2 f = __builtin_elementwise_min(__builtin_elementwise_sub_sat(as_u16x2(x), as_u16x2(y)), one);   // (!p, q) as 0 / 1
    const uint32_t w = as_u32(zero - f);                      // (~P, Q) as halfword masks
    const uint32_t m_lo = w ^ 0x0000FFFFu;                    // masks of (loA, loB): (P, Q)
    const uint32_t m_hi = swap_halves(w) ^ 0x0000FFFFu;       // masks of (hiA, hiB): (~Q, ~P)
    return {bit_select(c, m_hi, m_lo), bit_select(c, m_lo, m_hi)};
}

// positions (pos0 | pos1 << 16) of a 16-bit group's survivors: with d_i the removed flags (exactly two are set),
// pos0 = d0 * (1 + d1) and pos1 = 3 - d3 * (1 + d2)
__device__ __forceinline__ uint32_t positions16(const Keep16& k)
{
    const uint32_t d01 = ~k.k0 & 0x00010001u, d23 = ~k.k1 & 0x00010001u;     // (d0, d1), (d2, d3)
    const u16x2 a = as_u16x2(bit_select(0xFFFFu, d01, d23)), b = as_u16x2(__builtin_amdgcn_alignbit(d23, d01, 16));   // (d0, d3), (d1, d2)
    return as_u32(a * b + a) ^ 0x00030000u;                  // (pos0, 3 - pos1) -> pos0 | pos1 << 16
}

// the two survivors of a 16-bit group in column order: halfword p of (w1 : w0) is bytes 2p, 2p + 1
__device__ __forceinline__ uint32_t pack16(uint32_t w0, uint32_t w1, uint32_t z)
{
    return __builtin_amdgcn_perm(w1, w0, z * 0x0202u + 0x01000100u);
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

// Four int8 groups (16 bytes of a row): the survivors (8 bytes) and the four codes (16 bits, group 0 lowest).
// FIXED: the positions come from `given` (four stored codes) instead of the magnitudes.
template <int DT, bool FIXED>
__device__ __forceinline__ void compress8x4(const uint4v& w, uint32_t given, uint32_t& v0, uint32_t& v1, uint32_t& codes)
{
    if constexpr (FIXED) {
        uint32_t pk[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) pk[g] = pack8(w[g], positions_of_code(given >> (4 * g)));
        v0 = low_halves(pk[0], pk[1]);
        v1 = low_halves(pk[2], pk[3]);
        codes = 0;
    } else {
        uint32_t c01, c23;
        compress8x2<DT>(w[0], w[1], v0, c01);
        compress8x2<DT>(w[2], w[3], v1, c23);
        codes = c01 | (c23 << 8);
    }
}

// Two 16-bit groups (16 bytes of a row): the survivors (8 bytes) and the two codes (8 bits).
template <int DT, bool FIXED>
__device__ __forceinline__ void compress16x2(const uint4v& w, uint32_t given, uint32_t& v0, uint32_t& v1, uint32_t& codes)
{
    uint32_t z0, z1;
    if constexpr (FIXED) {
        z0 = positions_of_code(given);
        z1 = positions_of_code(given >> 4);
        codes = 0;
    } else {
        z0 = positions16(select16<DT>(w[0], w[1]));
        z1 = positions16(select16<DT>(w[2], w[3]));
        codes = (code_bits(z0) & 0xFu) | ((code_bits(z1) & 0xFu) << 4);
    }
    v0 = pack16(w[0], w[1], z0);
    v1 = pack16(w[2], w[3], z1);
}

// The codes of the 16-byte piece c of row m (4 groups for int8, 2 for 16-bit types) from stored metadata, in the
// low bits of the result, group 0 first.  K8 = K/8 (canonical row length in bytes), KB = K/64 (tiles per row block).
template <int DT, int LAYOUT>
__device__ __forceinline__ uint32_t stored_codes(const uint8_t* meta, int64_t m, int64_t c, int64_t K8, int64_t KB)
{
    constexpr int ES = is8<DT> ? 1 : 2;
    constexpr int GROUPS = 4 / ES;                       // groups per 16-byte piece
    if constexpr (LAYOUT == SP24_LAYOUT_CANONICAL) {
        if constexpr (is8<DT>) return *reinterpret_cast<const uint16_t*>(meta + m * K8 + c * 2);
        else return meta[m * K8 + c];
    } else {
        const int64_t e0 = c * (16 / ES);                // first column of the piece
        const int64_t kb = e0 >> 6;
        const uint32_t h = (uint32_t)(e0 >> 5) & 1u, g0 = (uint32_t)(e0 & 31) >> 2;
        const uint32_t word = reinterpret_cast<const uint32_t*>(meta)[((m >> 5) * KB + kb) * 64 + (m & 31) + 32 * h];
        return (word >> (4 * g0)) & ((1u << (4 * GROUPS)) - 1u);
    }
}

// Work assignment of the row-major kernels: a workgroup of 256 lanes covers 256 >> lg_cb rows x (1 << lg_cb)
// 16-byte pieces, so that short rows still fill it and a lane finds its row and piece with shifts;
// blockIdx.x walks along the row, blockIdx.y (with a stride loop for very tall matrices) down the rows.
struct RowTile {
    int lg_cb;
    __device__ __forceinline__ int64_t piece() const { return (int64_t)blockIdx.x * (1 << lg_cb) + (threadIdx.x & ((1u << lg_cb) - 1u)); }
    __device__ __forceinline__ int64_t first_row() const { return (int64_t)blockIdx.y * (256 >> lg_cb) + (threadIdx.x >> lg_cb); }
    __device__ __forceinline__ int64_t row_stride() const { return (int64_t)gridDim.y * (256 >> lg_cb); }
};

// ---- prune: dense -> dense ----------------------------------------------
// One lane per 16-byte piece of a row.  FIXED: the keep pattern comes from stored metadata instead of the
// magnitudes (Sec. 4.1 Step 3: removed weights stay zero while the network is retrained).
template <int DT, bool FIXED, int LAYOUT>
__global__ __launch_bounds__(256) void k_prune(const uint8_t* __restrict__ A, uint8_t* __restrict__ P, int64_t M,
                                               int64_t chunks_per_row, int64_t lda_bytes, int64_t ldp_bytes,
                                               const uint8_t* __restrict__ meta, int64_t K8, int64_t KB, RowTile rt)
{
    const int64_t c = rt.piece();
    if (c >= chunks_per_row) return;
    for (int64_t m = rt.first_row(); m < M; m += rt.row_stride()) {
        uint4v w = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(A + m * lda_bytes + c * 16));
        uint32_t codes = 0;
        if constexpr (FIXED) codes = stored_codes<DT, LAYOUT>(meta, m, c, K8, KB);
        if constexpr (is8<DT>) {
            if constexpr (FIXED) {
#pragma unroll
                for (int g = 0; g < 4; ++g) w[g] = prune8_by_mask(w[g], mask_of_code((codes >> (4 * g)) & 0xFu));
            } else {
#pragma unroll
                for (int g = 0; g < 4; g += 2) {
                    uint32_t wa = w[g], wb = w[g + 1];
                    prune8x2(wa, wb, select8x2<DT>(wa, wb));
                    w[g] = wa;
                    w[g + 1] = wb;
                }
            }
        } else {
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                uint32_t w0 = w[2 * g], w1 = w[2 * g + 1];
                if constexpr (FIXED) prune16_by_mask(w0, w1, mask_of_code((codes >> (4 * g)) & 0xFu));
                else {
                    const Keep16 k = select16<DT>(w0, w1);
                    w0 &= k.k0;
                    w1 &= k.k1;
                }
                w[2 * g] = w0;
                w[2 * g + 1] = w1;
            }
        }
        __builtin_nontemporal_store(w, reinterpret_cast<uint4v*>(P + m * ldp_bytes + c * 16));
    }
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
    constexpr int ES = is8<DT> ? 1 : 2;
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
        if constexpr (is8<DT>) {
            raw[i][0] = *reinterpret_cast<const uint32_t*>(src);
            raw[i][1] = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (DT == SP24_I8) mag[j] = (int)mag_key8((raw[i][0] >> (8 * j)) & 0xFFu);
                else mag[j] = (double)magnitude_f8(raw[i][0] >> (8 * j));
            }
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
        if constexpr (is8<DT>) {
            *reinterpret_cast<uint32_t*>(dst) = prune8_by_mask(raw[i][0], keep);
        } else {
            uint32_t w0 = raw[i][0], w1 = raw[i][1];
            prune16_by_mask(w0, w1, keep);
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
                                                        int64_t lda_bytes, RowTile rt)
{
    const int64_t c = rt.piece();
    if (c >= chunks_per_row) return;
    for (int64_t m = rt.first_row(); m < M; m += rt.row_stride()) {
        const int64_t id = m * chunks_per_row + c;      // V rows are 8 * chunks bytes, metadata rows chunks (16-bit) or 2 * chunks (int8) bytes
        const uint4v w = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(A + m * lda_bytes + c * 16));
        uint2v v;
        uint32_t v0, v1, codes;
        if constexpr (is8<DT>) {
            uint32_t given = 0;
            if constexpr (FIXED) given = *reinterpret_cast<const uint16_t*>(meta + id * 2);
            compress8x4<DT, FIXED>(w, given, v0, v1, codes);
            if constexpr (!FIXED) *reinterpret_cast<uint16_t*>(meta + id * 2) = (uint16_t)codes;
        } else {
            uint32_t given = 0;
            if constexpr (FIXED) given = meta[id];
            compress16x2<DT, FIXED>(w, given, v0, v1, codes);
            if constexpr (!FIXED) meta[id] = (uint8_t)codes;
        }
        v[0] = v0;
        v[1] = v1;
        *reinterpret_cast<uint2v*>(V + id * 8) = v;
    }
}

// ---- compress, tiled layout -----------------------------------------------
// A wavefront takes 32 rows x 128 bytes of A -- one 32x64 tile of a 16-bit type, two neighbouring tiles of int8 --
// and every lane compresses 64 consecutive bytes of one row: for the 16-bit types one slot (half of the tile's
// row), for int8 both slots of its row in one tile.  V and metadata leave as contiguous runs of 512 bytes or more.
// int8 reads its rows whole (8 rows x 128 contiguous bytes per load instruction) into a row-major image in LDS
// (rows padded by one 16-byte piece) and each lane takes its 64 bytes from there; for the 16-bit types, whose lanes
// already cover whole 128-byte lines in pairs, the lanes load their bytes themselves (measured: the image costs
// them 7 %, and gains int8 9 %).  blockIdx.y (with a stride loop) is the 32-row block, blockIdx.x walks along K.
template <int DT, bool FIXED>
__global__ __launch_bounds__(256) void k_compress_tiled(const uint8_t* __restrict__ A, uint8_t* __restrict__ V,
                                                        uint32_t* __restrict__ meta, int64_t RBs, int64_t KB,
                                                        int64_t lda_bytes, int64_t row_bytes)
{
    constexpr int kPitch = 9;                                                // 8 pieces of a row and one of padding
    __shared__ uint4v image[is8<DT> ? 4 : 1][is8<DT> ? 32 * kPitch : 1];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6, r = lane & 31u, h = lane >> 5;
    const int64_t col0 = ((int64_t)blockIdx.x * 4 + wave) * 128;            // first byte of the wavefront's columns
    if (col0 >= row_bytes) return;
    const bool whole = col0 + 128 <= row_bytes;                             // int8 with an odd number of tiles: the last wavefront has one
    for (int64_t rb = blockIdx.y; rb < RBs; rb += gridDim.y) {
        uint4v w[4];
        if constexpr (is8<DT>) {
            uint4v* img = image[wave];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint32_t row = (lane >> 3) + 8 * t, pc = lane & 7u;
                if (whole || pc < 4) img[row * kPitch + pc] = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(A + (rb * 32 + row) * lda_bytes + col0 + pc * 16));
            }
            // the image is this wavefront's own and the LDS serves a wavefront's operations in order: no barrier,
            // only the compiler must not move the reads above the writes
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int q = 0; q < 4; ++q) w[q] = img[r * kPitch + 4 * h + q];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();                                // the next block's writes stay behind these reads
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        } else {
            const uint4v* src = reinterpret_cast<const uint4v*>(A + (rb * 32 + r) * lda_bytes + col0 + h * 64);
#pragma unroll
            for (int q = 0; q < 4; ++q) w[q] = src[q];
        }
        if constexpr (is8<DT>) {
            const int64_t kb = col0 / 64 + h;                               // this lane's tile
            if (kb < KB) {
                const int64_t tile = rb * KB + kb;
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {                            // slot r + 32 * hh: columns 32 * hh .. + 31 of the tile
                    const int64_t slot = tile * 64 + r + 32 * hh;
                    uint32_t given = 0, c0, c1;
                    if constexpr (FIXED) given = meta[slot];
                    uint4v v;
                    uint32_t a, b;
                    compress8x4<DT, FIXED>(w[2 * hh], given, a, b, c0);
                    v[0] = a; v[1] = b;
                    compress8x4<DT, FIXED>(w[2 * hh + 1], given >> 16, a, b, c1);
                    v[2] = a; v[3] = b;
                    __builtin_nontemporal_store(v, reinterpret_cast<uint4v*>(V + slot * 16));
                    if constexpr (!FIXED) __builtin_nontemporal_store(c0 | (c1 << 16), &meta[slot]);
                }
            }
        } else {
            const int64_t tile = rb * KB + col0 / 128;
            uint32_t given = 0, codes = 0;
            if constexpr (FIXED) given = meta[tile * 64 + lane];
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                uint4v v;
                uint32_t a, b, c;
                compress16x2<DT, FIXED>(w[2 * s], given >> (16 * s), a, b, c);
                v[0] = a; v[1] = b;
                codes |= c << (16 * s);
                compress16x2<DT, FIXED>(w[2 * s + 1], given >> (16 * s + 8), a, b, c);
                v[2] = a; v[3] = b;
                codes |= c << (16 * s + 8);
                __builtin_nontemporal_store(v, reinterpret_cast<uint4v*>(V + ((tile * 2 + s) * 64 + lane) * 16));
            }
            if constexpr (!FIXED) __builtin_nontemporal_store(codes, &meta[tile * 64 + lane]);
        }
    }
}

// ---- decompress -----------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(256) void k_decompress_canon(const uint8_t* __restrict__ V, const uint8_t* __restrict__ meta,
                                                          uint8_t* __restrict__ P, int64_t M, int64_t chunks_per_row,
                                                          int64_t ldp_bytes, RowTile rt)
{
    const int64_t c = rt.piece();
    if (c >= chunks_per_row) return;
    for (int64_t m = rt.first_row(); m < M; m += rt.row_stride()) {
        const int64_t id = m * chunks_per_row + c;
        uint2v v = *reinterpret_cast<const uint2v*>(V + id * 8);
        uint4v w;
        if constexpr (is8<DT>) {
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
        __builtin_nontemporal_store(w, reinterpret_cast<uint4v*>(P + m * ldp_bytes + c * 16));
    }
}

// One lane per slot reads its values and codes (contiguous runs per wavefront) and forms the 32 (int8) or 64
// (16-bit) bytes of its row.  Written straight from there a store instruction would touch 64 separate 16-byte
// pieces, two per row; instead the wavefront's tile goes through a row-major image in LDS (rows padded by one
// piece) and leaves as whole rows: 64 (int8) or 128 (16-bit) contiguous bytes per row and instruction.
template <int DT>
__global__ __launch_bounds__(256) void k_decompress_tiled(const uint8_t* __restrict__ V, const uint32_t* __restrict__ meta,
                                                          uint8_t* __restrict__ P, int64_t RBs, int64_t KB,
                                                          int64_t ldp_bytes)
{
    constexpr int kPieces = is8<DT> ? 4 : 8;          // 16-byte pieces per tile row
    constexpr int kPitch = kPieces + 1;
    __shared__ uint4v image[4][32 * kPitch];
    const uint32_t slot = threadIdx.x & 63u, wave = threadIdx.x >> 6, r = slot & 31u, h = slot >> 5;
    const int64_t kb = (int64_t)blockIdx.x * 4 + wave;
    if (kb >= KB) return;
    uint4v* img = image[wave];
    for (int64_t rb = blockIdx.y; rb < RBs; rb += gridDim.y) {
        const int64_t tile = rb * KB + kb;
        uint32_t codes = meta[tile * 64 + slot];
        if constexpr (is8<DT>) {
            uint4v v = *reinterpret_cast<const uint4v*>(V + (tile * 64 + slot) * 16);
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                uint4v w;
                w[0] = unpack8(v[2 * q] & 0xFFFFu, (codes >> (16 * q)) & 0xFu);
                w[1] = unpack8(v[2 * q] >> 16, (codes >> (16 * q + 4)) & 0xFu);
                w[2] = unpack8(v[2 * q + 1] & 0xFFFFu, (codes >> (16 * q + 8)) & 0xFu);
                w[3] = unpack8(v[2 * q + 1] >> 16, (codes >> (16 * q + 12)) & 0xFu);
                img[r * kPitch + 2 * h + q] = w;
            }
        } else {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                uint4v v = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(V + ((tile * 2 + s) * 64 + slot) * 16));
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    uint32_t cc = (codes >> (8 * (2 * s + q))) & 0xFFu;
                    uint4v w;
                    uint32_t a, b;
                    unpack16(v[2 * q], cc & 0xFu, a, b);
                    w[0] = a; w[1] = b;
                    unpack16(v[2 * q + 1], cc >> 4, a, b);
                    w[2] = a; w[3] = b;
                    img[r * kPitch + 4 * h + 2 * s + q] = w;
                }
            }
        }
        // the image is this wavefront's own and the LDS serves a wavefront's operations in order: no barrier, only
        // the compiler must not move the reads above the writes
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        constexpr int kRowsPerStore = 64 / kPieces;
#pragma unroll
        for (int t = 0; t < 32 / kRowsPerStore; ++t) {
            const uint32_t row = slot / kPieces + t * kRowsPerStore, pc = slot % kPieces;
            const uint4v w = img[row * kPitch + pc];
            __builtin_nontemporal_store(w, reinterpret_cast<uint4v*>(P + (rb * 32 + row) * ldp_bytes + kb * (16 * kPieces) + pc * 16));
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();                      // the next tile's writes stay behind these reads
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// ---- launchers ------------------------------------------------------------
static inline unsigned blocks_for(int64_t items) { return (unsigned)((items + 255) / 256); }

// blockIdx.y extent for `row_blocks` blocks of rows: one workgroup each, up to the grid limit (beyond it the
// kernels walk down the rows with a stride loop).  Fewer, resident workgroups that loop were measured and are not
// used: equal on most kernels, 10 % slower on the fixed-mask pruning.
static inline int64_t grid_rows(int64_t row_blocks, int64_t) { return row_blocks < 65535 ? row_blocks : 65535; }
// grid and lane assignment of a row-major kernel over M rows of cpr 16-byte pieces
static inline RowTile row_tile(int64_t M, int64_t cpr, dim3& grid)
{
    int lg = 0;
    while (lg < 8 && (1 << lg) < cpr) ++lg;
    const int64_t rows_per_block = 256 >> lg, row_blocks = (M + rows_per_block - 1) / rows_per_block;
    const int64_t gx = (cpr + (1 << lg) - 1) >> lg;
    grid = dim3((unsigned)gx, (unsigned)grid_rows(row_blocks, gx));
    return RowTile{lg};
}
// grid of a tiled-layout kernel: blockIdx.x over groups of tiles along K, blockIdx.y over 32-row blocks
static inline dim3 tile_grid(int64_t RBs, int64_t KB, int tiles_per_block)
{
    const int64_t gx = (KB + tiles_per_block - 1) / tiles_per_block;
    return dim3((unsigned)gx, (unsigned)grid_rows(RBs, gx));
}

// meta == nullptr: select by magnitude; else keep the pattern that `meta` (in layout l) records
template <int DT>
static void run_prune(const void* A, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, const void* meta, sp24_layout l,
                      hipStream_t st)
{
    constexpr int64_t es = is8<DT> ? 1 : 2;
    const int64_t cpr = K * es / 16;
    dim3 grid;
    const RowTile rt = row_tile(M, cpr, grid);
    const uint8_t *a = (const uint8_t*)A, *mt = (const uint8_t*)meta;
    uint8_t* p = (uint8_t*)P;
    if (!meta) k_prune<DT, false, SP24_LAYOUT_CANONICAL><<<grid, 256, 0, st>>>(a, p, M, cpr, lda * es, ldp * es, nullptr, 0, 0, rt);
    else if (l == SP24_LAYOUT_CANONICAL)
        k_prune<DT, true, SP24_LAYOUT_CANONICAL><<<grid, 256, 0, st>>>(a, p, M, cpr, lda * es, ldp * es, mt, K / 8, K / 64, rt);
    else k_prune<DT, true, SP24_LAYOUT_TILED><<<grid, 256, 0, st>>>(a, p, M, cpr, lda * es, ldp * es, mt, K / 8, K / 64, rt);
}

// fixed: `meta` is an input and only V is written
template <int DT, bool FIXED>
static void run_compress(const void* A, void* V, void* meta, int64_t M, int64_t K, int64_t lda, sp24_layout l, hipStream_t st)
{
    constexpr int64_t es = is8<DT> ? 1 : 2;
    if (l == SP24_LAYOUT_CANONICAL) {
        int64_t cpr = K * es / 16;
        dim3 grid;
        const RowTile rt = row_tile(M, cpr, grid);
        k_compress_canon<DT, FIXED><<<grid, 256, 0, st>>>((const uint8_t*)A, (uint8_t*)V, (uint8_t*)meta, M, cpr, lda * es, rt);
    } else {
        int64_t KB = K / 64, RBs = M / 32;
        k_compress_tiled<DT, FIXED><<<tile_grid(RBs, KB, is8<DT> ? 8 : 4), 256, 0, st>>>((const uint8_t*)A, (uint8_t*)V, (uint32_t*)meta, RBs, KB, lda * es, K * es);
    }
}

template <int DT>
static void run_decompress(const void* V, const void* meta, void* P, int64_t M, int64_t K, int64_t ldp, sp24_layout l, hipStream_t st)
{
    constexpr int64_t es = is8<DT> ? 1 : 2;
    if (l == SP24_LAYOUT_CANONICAL) {
        int64_t cpr = K * es / 16;
        dim3 grid;
        const RowTile rt = row_tile(M, cpr, grid);
        k_decompress_canon<DT><<<grid, 256, 0, st>>>((const uint8_t*)V, (const uint8_t*)meta, (uint8_t*)P, M, cpr, ldp * es, rt);
    } else {
        int64_t KB = K / 64, RBs = M / 32;
        k_decompress_tiled<DT><<<tile_grid(RBs, KB, 4), 256, 0, st>>>((const uint8_t*)V, (const uint32_t*)meta, (uint8_t*)P, RBs, KB, ldp * es);
    }
}

static sp24_status launch_result() { return hipGetLastError() == hipSuccess ? SP24_OK : SP24_ERR_LAUNCH; }

sp24_status launch_prune(const void* A, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, sp24_dtype t, hipStream_t st)
{
    if (M * K == 0) return SP24_OK;
    if (t == SP24_F16) run_prune<SP24_F16>(A, P, M, K, lda, ldp, nullptr, SP24_LAYOUT_CANONICAL, st);
    else if (t == SP24_BF16) run_prune<SP24_BF16>(A, P, M, K, lda, ldp, nullptr, SP24_LAYOUT_CANONICAL, st);
    else if (t == SP24_F8) run_prune<SP24_F8>(A, P, M, K, lda, ldp, nullptr, SP24_LAYOUT_CANONICAL, st);
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
    else if (t == SP24_F8) k_prune_transposable<SP24_F8><<<grid, 256, 0, st>>>(a, p, M4, K4, lda, ldp);
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
    else if (t == SP24_F8) run_compress<SP24_F8, false>(A, V, meta, M, K, lda, l, st);
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
