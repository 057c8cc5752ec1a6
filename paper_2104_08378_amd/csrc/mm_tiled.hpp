// Tiled, software-pipelined matrix-multiply kernels for large shapes.
//
// Sparse product (Sec. 3.2, Fig. 2) on the 32x32 sparse matrix-core
// instructions, and the same-shape dense product on the dense ones.  A
// workgroup of WM x WN wavefronts computes a (32*TM*WM) x (32*TN*WN) tile of D;
// each wavefront owns TM x TN accumulator tiles of 32x32.  The large
// configuration is 4 x 2 wavefronts of 64 x 128 each: a 256 x 256 tile, half of
// the compute unit's register file in accumulators, two wavefronts per SIMD.
//
//   - a step consumes 128 bytes of every B row (128 int8 / 64 16-bit values of K);
//   - every operand travels global -> LDS without passing through registers
//     (global_load_lds) into a ring of stages, ahead of its use.  For the
//     sparse kernel that is B plus the compressed A in its tiled layout, whose
//     32-row tiles are contiguous 1 KiB runs of values and 256-byte runs of
//     metadata words already in lane order (Sec. 3.1: no indirection,
//     full-width reads), so a wavefront reads its A operands back with one
//     conflict-free 16-byte and one 4-byte LDS read per lane;
//   - one s_barrier per step and no fence: a wavefront awaits its own
//     transfers with s_waitcnt vmcnt, the barrier then makes everybody's visible;
//   - memory instructions are dealt out between the matrix-core instructions
//     (sched_group_barrier) so that their issue time overlaps the arithmetic;
//   - B rows in LDS are 128 bytes, unpadded (a transfer instruction fills
//     1 KiB = 8 rows contiguously); the 16-byte piece c of row n sits at slot
//     c ^ ((n >> 1) & 7), so that the fragment reads of 16 neighbouring rows
//     hit 16 different 16-byte columns of the 256-byte-wide bank array;
//   - workgroup ids are remapped so that the workgroups resident on one XCD
//     (ids congruent mod 8) cover a compact 8 x n block of tiles and share
//     their A and B panels in that XCD's L2.
#pragma once
#include "common.hpp"
#include "launch.hpp"
#include "mfma.hpp"

namespace sp24 {

constexpr int kRowBytes = 128;   // bytes of one operand row consumed per step

typedef __attribute__((address_space(3))) void* lds_ptr;

// s_waitcnt immediate (gfx9 encoding) that waits for vmcnt <= n and leaves expcnt / lgkmcnt alone
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// sched_group_barrier masks
constexpr int kSgMfma = 0x008, kSgVmem = 0x010, kSgDsRead = 0x100;

// Workgroup id -> tile coordinates.  The hardware deals consecutive ids round-robin over the 8 XCDs; each XCD
// is given a contiguous range of tiles, swept in groups of 8 tile rows.
__device__ __forceinline__ void tile_of_workgroup(int tiles_m, int tiles_n, int& tm, int& tn)
{
    const int nwg = tiles_m * tiles_n;
    int wg = blockIdx.x;
    const int per = (nwg + 7) / 8;
    const int xcd = wg & 7, idx = wg >> 3;
    const int full = nwg - (per - 1) * 8;   // XCDs that own `per` ids (the rest own per - 1)
    wg = (xcd < full) ? xcd * per + idx : full * per + (xcd - full) * (per - 1) + idx;
    constexpr int GM = 8;
    const int group = wg / (GM * tiles_n);
    const int first_m = group * GM;
    const int gsz = min(tiles_m - first_m, GM);
    const int in_group = wg - group * GM * tiles_n;
    tm = first_m + in_group % gsz;
    tn = in_group / gsz;
}

// The part of the inner dimension that a workgroup covers.  Normally all of it.  With K split across gridDim.y
// workgroups per tile, slice blockIdx.y takes the whole steps first .. first + nsteps - 1 (the last slice also the
// partial step) and writes its partial product to image blockIdx.y of D: M rows of ldd accumulator-typed values.
struct KRange {
    int first, nsteps, tail;
};
__device__ __forceinline__ KRange k_range_of_workgroup(MmArgs& a, int total_steps, int tail)
{
    if (a.k_slices <= 1) return {0, total_steps, tail};
    const int slice = blockIdx.y;
    const int first = min(slice * a.slice_steps, total_steps);
    a.D = reinterpret_cast<uint8_t*>(a.D) + (int64_t)slice * a.M * a.ldd * 4;
    return {first, min(a.slice_steps, total_steps - first), slice == a.k_slices - 1 ? tail : 0};
}

// Transfer ROWS rows x 128 bytes (row r of the stage = global row min(row0 + r, limit - 1)) into a stage.
// Offsets of the ROWS/8/NW transfer instructions (8 rows each) of one of NW wavefronts, relative to the first row.
template <int ROWS, int NW>
__device__ __forceinline__ void dma_offsets(int64_t row0, int64_t limit, int64_t ld_bytes, int wave, int lane, uint32_t (&off)[ROWS / 8 / NW])
{
#pragma unroll
    for (int j = 0; j < ROWS / 8 / NW; ++j) {
        const int row = (wave * (ROWS / 8 / NW) + j) * 8 + (lane >> 3);
        int64_t g = row0 + row;
        if (g >= limit) g = limit - 1;                       // ragged edge: fetch a valid row, never stored
        const int piece = (lane & 7) ^ ((row >> 1) & 7);
        off[j] = (uint32_t)((g - row0) * ld_bytes + piece * 16);
    }
}

// One global -> LDS transfer instruction: lane l moves 16 (or 4) bytes from base + off to lds + 16*l (4*l).
// `base` and `lds` must be wavefront-uniform.  Written as inline assembly on purpose: with the compiler's own
// builtin in a loop, its wait-count pass treats the LDS counter as out of order and turns every wait for an
// LDS read into lgkmcnt(0), which serialises the operand reads with the arithmetic.  The price is that the
// compiler does not count these transfers in vmcnt: every wait for them below is written by hand.
// a pointer the compiler can keep in scalar registers (the value must be the same in every lane)
__device__ __forceinline__ const uint8_t* wave_uniform(const uint8_t* p)
{
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const uint8_t*>(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ void lds_dma16(const uint8_t* base, uint32_t off, const uint8_t* lds)
{
    const uint32_t l = (uint32_t)(uintptr_t)(lds_ptr)lds;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(wave_uniform(base)), "s"(l) : "m0", "memory");
}
__device__ __forceinline__ void lds_dma4(const uint8_t* base, uint32_t off, const uint8_t* lds)
{
    const uint32_t l = (uint32_t)(uintptr_t)(lds_ptr)lds;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(off), "s"(wave_uniform(base)), "s"(l) : "m0", "memory");
}

// The same transfer with a full 64-bit address per lane (for gathers that a base + 32-bit offset cannot express).
__device__ __forceinline__ void lds_dma16_addr(const uint8_t* addr, const uint8_t* lds)
{
    const uint32_t l = (uint32_t)(uintptr_t)(lds_ptr)lds;
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(addr), "s"(l) : "m0", "memory");
}

__device__ __forceinline__ void lds_dma4_addr(const uint8_t* addr, const uint8_t* lds)
{
    const uint32_t l = (uint32_t)(uintptr_t)(lds_ptr)lds;
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(addr), "s"(l) : "m0", "memory");
}

// 128 zero bytes: the source of B rows that fall into a convolution's padding or past the last output pixel, and
// of every operand piece that lies past K in the last step when K is not a whole number of steps.
__device__ __attribute__((aligned(128))) const uint8_t k_zero_row[128] = {};

// One transfer of the last, partial step: lanes whose piece lies past K fetch zeros instead (branch-free).
template <bool DWORD>
__device__ __forceinline__ void lds_dma_tail(const uint8_t* base, uint32_t off, bool past_k, const uint8_t* lds)
{
    const uint64_t mask = (uint64_t)0 - (uint64_t)past_k;
    const uint64_t src = ((reinterpret_cast<uint64_t>(base) + off) & ~mask) | (reinterpret_cast<uint64_t>(k_zero_row) & mask);
    if constexpr (DWORD) lds_dma4_addr(reinterpret_cast<const uint8_t*>(src), lds);
    else lds_dma16_addr(reinterpret_cast<const uint8_t*>(src), lds);
}

// Does transfer j of a K-major operand block (dma_offsets) / of an N-major B block (dma_offsets_nmajor) lie past
// the first `tail` bytes of K in the step, for this lane?
template <int ROWS, int NW>
__device__ __forceinline__ bool past_k_kmajor(int j, int wave, int lane, int tail)
{
    const int row = (wave * (ROWS / 8 / NW) + j) * 8 + (lane >> 3);
    return (((lane & 7) ^ ((row >> 1) & 7)) << 4) >= tail;
}
template <int BN, int NW, int ES>
__device__ __forceinline__ bool past_k_nmajor(int j, int wave, int lane, int tail)
{
    const int p = (wave * (BN / 8 / NW) + j) * 1024 + lane * 16;
    return (p / (BN * ES)) * ES >= tail;
}

// Position of a K step inside a convolution's inner dimension k = (r*S + s)*C + c: a step (128 bytes of K) lies
// inside one filter tap when C * element size is a multiple of 128 bytes.
struct ConvTap {
    int r, s, c0;
    __device__ __forceinline__ void next(const ConvGeom& g, int bk)
    {
        c0 += bk;
        if (c0 == g.C) {
            c0 = 0;
            if (++s == g.S) { s = 0; ++r; }
        }
    }
};

// B rows of a convolution read as an implicit GEMM (Sec. 3.2; inner dimension C x R x S, Sec. 4.2): row n of the
// operand is output pixel n, and its 128 bytes of a step are 128 contiguous bytes of the NHWC input at the
// pixel that filter tap (r, s) meets -- or zeros when that pixel is padding.  Per lane and transfer: the input
// coordinates of tap (0, 0) and the byte offset of that (possibly virtual) pixel, swizzle piece included.
template <int ROWS, int NW, int ES>
struct conv_rows {
    static constexpr int NJ = ROWS / 8 / NW;
    int iy0[NJ], ix0[NJ];
    int32_t off[NJ];
    __device__ __forceinline__ void init(const ConvGeom& g, int64_t n0, int64_t N, int wave, int lane)
    {
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int row = (wave * NJ + j) * 8 + (lane >> 3);
            const int piece = (lane & 7) ^ ((row >> 1) & 7);
            const int64_t n = n0 + row;
            if (n < N) {
                const int t = (int)(n / g.OW), ox = (int)(n - (int64_t)t * g.OW);
                const int img = t / g.OH, oy = t - img * g.OH;
                iy0[j] = oy * g.stride_h - g.pad_h;
                ix0[j] = ox * g.stride_w - g.pad_w;
                off[j] = (((img * g.H + iy0[j]) * g.W + ix0[j]) * g.C) * ES + piece * 16;
            } else {                                       // past the last pixel: always zeros, never stored
                iy0[j] = -(1 << 24);
                ix0[j] = 0;
                off[j] = 0;
            }
        }
    }
    // transfer j of this wavefront for the step at tap t
    __device__ __forceinline__ void issue(int j, const uint8_t* X, const ConvGeom& g, const ConvTap& t, uint8_t* stage, int wave) const
    {
        const int tap_off = ((t.r * g.W + t.s) * g.C + t.c0) * ES;
        // branch-free select between the pixel and the zero row (a divergent branch per transfer costs far more)
        const uint64_t inside = (uint64_t)((unsigned)(iy0[j] + t.r) < (unsigned)g.H) & (uint64_t)((unsigned)(ix0[j] + t.s) < (unsigned)g.W);
        const uint64_t mask = (uint64_t)0 - inside;
        const uint64_t pixel = reinterpret_cast<uint64_t>(X) + (uint32_t)(off[j] + tap_off);
        const uint64_t src = (pixel & mask) | (reinterpret_cast<uint64_t>(k_zero_row) & ~mask);
        lds_dma16_addr(reinterpret_cast<const uint8_t*>(src), stage + (wave * NJ + j) * 1024);
    }
};

// ---------------------------------------------------------------------------
// B stored N-major (element (k, n) at B[k*ldb + n]).  A stage then holds the step's K rows, each the tile's BN
// columns (BN * element size bytes, 16-byte chunks swizzled by row), and a wavefront reads its fragments with
// the transposing LDS reads of gfx950: in every group of 16 lanes, lane l receives from the 8-byte pieces the
// 16 lanes address
//     ds_read_b64_tr_b8 :  byte j (0..7)    = byte l % 8 of the piece of lane 2*j + l / 8
//     ds_read_b64_tr_b16:  element j (0..3) = element l % 4 of the piece of lane 4*j + l / 4
// (measured).  With lane s of a group addressing row k0 + s/2 (s/4), columns 8*(s%2).. (4*(s%4)..), lane l gets
// column l of the group's 16 columns, rows k0 .. k0+7 (k0+3): K-contiguous values, as the matrix cores want them.
// ---------------------------------------------------------------------------
typedef short short4v __attribute__((ext_vector_type(4)));
typedef int int2v __attribute__((ext_vector_type(2)));

// swizzle of the 16-byte chunks of row k: rows that one transposing read touches land in different banks
template <int ES>
__device__ __forceinline__ int nmajor_swizzle(int k, int chunks)
{
    return (ES == 1) ? ((2 * (k & 7)) & (chunks - 1)) : ((4 * (k & 3)) & (chunks - 1));
}

// Offsets (from the tile's first column of the step's first row) of the B transfers of one of NW wavefronts:
// LDS position p of the B region <- row p / row_bytes, chunk (p % row_bytes) / 16 ^ swizzle(row); chunks past the
// last column of the matrix are replaced by the last valid one (never stored).
template <int BN, int NW, int ES>
__device__ __forceinline__ void dma_offsets_nmajor(int64_t col0, int64_t N, int64_t ld_bytes, int wave, int lane, uint32_t (&off)[BN / 8 / NW])
{
    constexpr int kRowB = BN * ES, kChunks = kRowB / 16;
    const int64_t left = (N - col0) * ES / 16;
    const int valid = left < kChunks ? (int)left : kChunks;
#pragma unroll
    for (int j = 0; j < BN / 8 / NW; ++j) {
        const int p = (wave * (BN / 8 / NW) + j) * 1024 + lane * 16;
        const int row = p / kRowB;
        int c = ((p % kRowB) >> 4) ^ nmajor_swizzle<ES>(row, kChunks);
        if (c >= valid) c = valid - 1;
        off[j] = (uint32_t)(row * ld_bytes + c * 16);
    }
}

// Per-lane addressing of the transposing fragment reads: piece c2 (16 K-bytes at K-byte offset 16*(2*c2 + q) of
// the step) of column (wavefront's first column + 32*nj + lane % 32).
template <int BN, int TN, int ES>
struct nmajor_frags {
    static constexpr int kRowB = BN * ES, kChunks = kRowB / 16;
    static constexpr int kRowsPerC2 = 32 / ES;        // K rows per unit of c2 (two pieces: q = 0, 1)
    static constexpr int kRowsPerRead = 8 / ES;       // K rows one transposing read covers
    int row_off;                                      // bytes: this lane's source row
    int col_off[TN];                                  // bytes within the row, swizzled, per 32-column block
    __device__ __forceinline__ void init(int wn, int lane)
    {
        const int g = lane >> 4, s = lane & 15, q = g >> 1;
        const int sub = (ES == 1) ? (s >> 1) : (s >> 2);                       // row inside one read
        const int col_in_group = (ES == 1) ? 8 * (s & 1) : 8 * (s & 3);        // bytes
        row_off = ((kRowsPerC2 / 2) * q + sub) * kRowB;
        const int swz = nmajor_swizzle<ES>(sub, kChunks);
#pragma unroll
        for (int nj = 0; nj < TN; ++nj) {
            const int bytes = (wn * 32 * TN + nj * 32 + 16 * (g & 1)) * ES + col_in_group;
            col_off[nj] = (((bytes >> 4) ^ swz) << 4) + (bytes & 15);
        }
    }
    // the 16 bytes of piece 2*c2 + q for this lane's column of block nj; `b` = start of the B region of a stage
    __device__ __forceinline__ uint4v piece(const uint8_t* b, int c2, int nj) const
    {
        const uint8_t* p0 = b + row_off + col_off[nj] + c2 * kRowsPerC2 * kRowB;
        const uint8_t* p1 = p0 + kRowsPerRead * kRowB;
        uint4v v;
        if constexpr (ES == 1) {
            const int2v x = __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) int2v*)p0);
            const int2v y = __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) int2v*)p1);
            v[0] = (uint32_t)x[0]; v[1] = (uint32_t)x[1]; v[2] = (uint32_t)y[0]; v[3] = (uint32_t)y[1];
        } else {
            const int2v x = __builtin_bit_cast(int2v, __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)p0));
            const int2v y = __builtin_bit_cast(int2v, __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)p1));
            v[0] = (uint32_t)x[0]; v[1] = (uint32_t)x[1]; v[2] = (uint32_t)y[0]; v[3] = (uint32_t)y[1];
        }
        return v;
    }
};

template <int ROWS, int NW>
__device__ __forceinline__ void dma_rows(const uint8_t* base, const uint32_t (&off)[ROWS / 8 / NW], uint8_t* stage, int wave)
{
#pragma unroll
    for (int j = 0; j < ROWS / 8 / NW; ++j) lds_dma16(base, off[j], stage + (wave * (ROWS / 8 / NW) + j) * 1024);
}

// Epilogue of the tiled kernels.  A wavefront's accumulators hold, per 32x32 tile, 32 consecutive columns of
// one row per register -- 64- or 128-byte pieces when stored directly.  Instead each 32-row block of the
// wavefront's tile is written to LDS as a row-major image in the output type and read back 16 bytes per lane,
// so that a store instruction covers whole rows of the wavefront's tile (256 or 512 contiguous bytes each).
// `scratch` is this wavefront's own 32 x kPitch bytes; the direct path serves outputs that are not 16-byte tileable.
template <int OUT, int TN>
struct epilogue_geometry {
    static constexpr int kOsz = out_size<OUT>();
    static constexpr int kRowBytesOut = 32 * TN * kOsz;
    // 4- and 1-byte outputs: a padded pitch (4 rows apart = half a bank row apart).  2-byte outputs: rows packed,
    // and 16-byte chunk c of a row kept at chunk_in_image(row, c): the 64-byte blocks (one per 32x32 tile) permuted by
    // row bits 0-2, the chunks inside a block by row bits 3-4.  An image write -- 64 lanes, rows 4q + (lane & 1), four
    // bytes each, usually two such rows per instruction -- then hits every bank once, and a lane's own two values
    // never share a bank, whichever rows the compiler pairs (measured: bank-conflict cycles of the kernel 786 k ->
    // 262 k per launch on the 4096 x 8192 bf16 output, 0.5 % of its LDS cycles).
    static constexpr int kPitch = kRowBytesOut + (kOsz == 4 ? 32 : kOsz == 2 ? 0 : 16);
    __device__ static int block_swizzle(int row)
    {
        const int hi = ((row >> 2) ^ (row >> 1)) & 1;
        return TN == 4 ? (row & 1) + 2 * hi : TN == 2 ? hi : 0;
    }
    __device__ static int chunk_in_image(int row, int c) { return (((c >> 2) ^ block_swizzle(row)) << 2) + ((c & 3) ^ ((row >> 3) & 3)); }
    static constexpr int kWaveBytes = 32 * kPitch;
};

template <int DT, int OUT, int TM, int TN>
__device__ __forceinline__ void store_wave_tile(const MmArgs& a, typename acc_of<DT>::type (&acc)[TM][TN], uint8_t* scratch,
                                                int64_t row_base, int64_t col_base, int lane)
{
    using G = epilogue_geometry<OUT, TN>;
    constexpr int kOsz = G::kOsz, kPitch = G::kPitch;
    const bool vec_ok = (reinterpret_cast<uintptr_t>(a.D) & 15u) == 0 && (a.ldd * kOsz) % 16 == 0 && a.N % (16 / kOsz) == 0;
    if (!vec_ok) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                store_tile<DT, OUT>(a.D, a.ldd, row_base + i * 32, col_base + j * 32, a.M, a.N, acc[i][j], lane, a.epi);
        return;
    }
    const int r = lane & 31, q = lane >> 5;
    constexpr int kChunksPerRow = G::kRowBytesOut / 16;
    uint8_t* Dp = reinterpret_cast<uint8_t*>(a.D);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        // quantised path: scale and bias of this lane's 16 rows of the block (rows past M are never stored)
        float es[16], eb[16];
        if constexpr (DT == SP24_I8 && OUT != SP24_I32) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                int64_t m = row_base + i * 32 + 8 * (e / 4) + 4 * q + (e % 4);
                epilogue_row(a.epi, m < a.M ? m : a.M - 1, es[e], eb[e]);
            }
        }
        if constexpr (kOsz == 2) {
            // A lane holds rows e, e + 1 of one column; converted as a pair they fill a register.  Neighbouring
            // lanes (columns r, r ^ 1) then trade halves: the even lane ends up with row e of both columns, the odd
            // one with row e + 1, so that the image is written 4 bytes per lane.
            const uint32_t sel = (lane & 1) ? 0x03020706u : 0x05040100u;   // v_perm_b32: bytes 0-3 own, 4-7 neighbour
            // this lane's 4 bytes of row 8*(e/4) + 4*q + e%4 + (lane & 1), block j: chunk 4*j + r/8 of the row, bytes (r/2 % 4) * 4
            uint8_t* img = scratch + (4 * q + (lane & 1)) * kPitch + ((r >> 1) & 3) * 4;
            const int row0 = 4 * q + (lane & 1);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; e += 2) {
                    float y0, y1;
                    if constexpr (DT == SP24_I8) {
                        y0 = dequant_value(acc[i][j][e], es[e], eb[e], a.epi.relu);
                        y1 = dequant_value(acc[i][j][e + 1], es[e + 1], eb[e + 1], a.epi.relu);
                    } else {
                        y0 = acc[i][j][e];
                        y1 = acc[i][j][e + 1];
                    }
                    const uint32_t own = pack_out16<OUT>(y0, y1);
                    const uint32_t nb = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)own, 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, true);
                    const int row = row0 + 8 * (e / 4) + (e % 4);
                    *reinterpret_cast<uint32_t*>(img + (8 * (e / 4) + (e % 4)) * kPitch + G::chunk_in_image(row, 4 * j + (r >> 3)) * 16) = __builtin_amdgcn_perm(nb, own, sel);
                }
        } else {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    uint8_t* p = scratch + (8 * (e / 4) + 4 * q + (e % 4)) * kPitch + (j * 32 + r) * kOsz;
                    auto v = acc[i][j][e];
                    float s = 0.0f, b = 0.0f;
                    if constexpr (DT == SP24_I8 && OUT != SP24_I32) { s = es[e]; b = eb[e]; }
                    store_bits<OUT>(p, 0, output_bits<OUT>(v, s, b, a.epi));
                }
        }
#pragma unroll
        for (int it = 0; it < 32 * kChunksPerRow / 64; ++it) {
            const int idx = it * 64 + lane;
            const int row = idx / kChunksPerRow, c = idx % kChunksPerRow;
            const int cs = (kOsz == 2) ? G::chunk_in_image(row, c) : c;           // where chunk c of the row lies in the image
            const uint4v v = *reinterpret_cast<const uint4v*>(scratch + row * kPitch + cs * 16);
            const int64_t grow = row_base + i * 32 + row, gcol = col_base + c * (16 / kOsz);
            // D is written once and not read again here: stores that bypass L2 allocation leave the L2 to the A and
            // B panels that neighbouring tiles share
            if (grow < a.M && gcol < a.N) __builtin_nontemporal_store(v, reinterpret_cast<uint4v*>(Dp + (grow * a.ldd + gcol) * kOsz));
        }
    }
}

// ---------------------------------------------------------------------------
// Sparse kernel.  Stage layout: [B: BN rows x 128 B, swizzled][V: 2 KiB per
// 32-row block, in the tiled layout's own order][meta: 256 B per 32x64 tile].
// NS stages; the transfers for step s+NS-1 are issued during step s, and the
// first operands of step s+1 are read from LDS during the tail of step s.
// ---------------------------------------------------------------------------
// BSRC: where B comes from -- 0 a K-major matrix, 1 NHWC activations (implicit GEMM), 2 an N-major matrix
template <int DT, int OUT, int WM, int WN, int TM, int TN, int NS, int BSRC>
__global__ __launch_bounds__(64 * WM * WN, 1) void k_spmm_pipe(MmArgs a, int tiles_m, int tiles_n)
{
    constexpr bool CONV = BSRC == 1, NMAJ = BSRC == 2;
    constexpr int ES = is8<DT> ? 1 : 2;
    constexpr int BK = kRowBytes / ES;        // K elements per step
    constexpr int T64 = BK / 64;              // 32x64 A tiles per step and row block (2 for int8, 1 for 16-bit)
    constexpr int NW = WM * WN;
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    constexpr int RB = BM / 32;               // row blocks per workgroup tile
    constexpr int NJB = BN / 8 / NW;          // B transfers per wavefront and step (1 KiB each)
    constexpr int NJV = RB * 2 / NW;          // V transfers (1 KiB each)
    constexpr int NJM = RB * T64 / NW;        // metadata transfers (256 B each)
    static_assert(RB * T64 % NW == 0 && BN % (8 * NW) == 0, "transfers must divide evenly over the wavefronts");
    constexpr int NV = NJB + NJV + NJM;
    constexpr int kVOff = BN * kRowBytes, kMOff = kVOff + RB * 2048;
    constexpr int kStageBytes = kMOff + RB * T64 * 256;
    using acc_t = typename acc_of<DT>::type;
    constexpr int kEpiBytes = NW * epilogue_geometry<OUT, TN>::kWaveBytes;
    static_assert(NS >= 3 && (NS - 2) * NV <= 63, "at least three stages; vmcnt is a 6-bit counter");
    constexpr int kLdsBytes = NS * kStageBytes > kEpiBytes ? NS * kStageBytes : kEpiBytes;
    __shared__ __attribute__((aligned(1024))) uint8_t lds_all[kLdsBytes];

    int tm, tn;
    tile_of_workgroup(tiles_m, tiles_n, tm, tn);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int r = lane & 31, q = lane >> 5;
    const int64_t KB64 = a.K / 64;
    // whole steps, and the bytes of K in a further, partial step (0: none), of this workgroup's share of K
    const KRange share = k_range_of_workgroup(a, (int)(a.K / BK), (int)((a.K * ES) % kRowBytes));
    const int nsteps = share.nsteps, tail = share.tail;
    const int64_t rb_total = a.M / 32;

    // ---- transfers of this wavefront ----
    const int64_t ldb_bytes = a.ldb * ES;
    // K-major: the tile's first row of B, a step is 128 bytes further; N-major: its first column, a step BK rows further
    const int64_t b_step = NMAJ ? (int64_t)BK * ldb_bytes : (int64_t)kRowBytes;
    const uint8_t* b_blk = reinterpret_cast<const uint8_t*>(a.B) + (NMAJ ? (int64_t)tn * BN * ES : (int64_t)tn * BN * ldb_bytes) +
                           share.first * b_step;
    uint32_t b_off[NJB];
    conv_rows<BN, NW, ES> b_conv;
    if constexpr (CONV) b_conv.init(a.conv, (int64_t)tn * BN, a.N, wave, lane);
    else if constexpr (NMAJ) dma_offsets_nmajor<BN, NW, ES>((int64_t)tn * BN, a.N, ldb_bytes, wave, lane, b_off);
    else dma_offsets<BN, NW>((int64_t)tn * BN, a.N, ldb_bytes, wave, lane, b_off);
    // V: transfer x of this wavefront is 1 KiB number (wave*NJV + x) of the RB*2 of a step: row block /2, half %2.
    // metadata: transfer x is 256-byte tile number (wave*NJM + x) of the RB*T64 of a step.
    // Either way the stage receives the tiled layout's slot order (slot = lane).  From the tiled layout a transfer
    // is one contiguous run; from the canonical one lane (m % 32, h) fetches its 16 bytes of values and 4 bytes
    // of codes from row m of the row-major arrays (Sec. 3.1: their position follows from the row and column alone).
    const bool canonical = a.layout == SP24_LAYOUT_CANONICAL;
    const uint8_t* v_base[NJV];                            // wavefront-uniform
    const uint8_t* m_base[NJM];
    uint32_t v_off[NJV], m_off[NJM];                       // per lane
    const int64_t v_step = canonical ? 64 : 2048, m_step = canonical ? 8 * T64 : T64 * 256;   // bytes per step
    if (canonical) {
        const int64_t vrow = a.K / 2 * ES, mrow = a.K / 8, row0 = (int64_t)tm * BM;
        const int h = lane >> 5;
#pragma unroll
        for (int x = 0; x < NJV; ++x) {
            const int id = wave * NJV + x;
            int64_t row = row0 + (id >> 1) * 32 + (lane & 31);
            if (row >= a.M) row = a.M - 1;                 // ragged M: a valid row, never stored
            v_base[x] = wave_uniform(reinterpret_cast<const uint8_t*>(a.A) + row0 * vrow);
            v_off[x] = (uint32_t)((row - row0) * vrow + ((ES == 1) ? 32 * (id & 1) + 16 * h : 32 * h + 16 * (id & 1)));
        }
#pragma unroll
        for (int x = 0; x < NJM; ++x) {
            const int id = wave * NJM + x;
            int64_t row = row0 + (id / T64) * 32 + (lane & 31);
            if (row >= a.M) row = a.M - 1;
            m_base[x] = wave_uniform(reinterpret_cast<const uint8_t*>(a.meta) + row0 * mrow);
            m_off[x] = (uint32_t)((row - row0) * mrow + 8 * (id % T64) + 4 * h);
        }
    } else {
#pragma unroll
        for (int x = 0; x < NJV; ++x) {
            const int id = wave * NJV + x;
            int64_t rb = (int64_t)tm * RB + (id >> 1);
            if (rb >= rb_total) rb = rb_total - 1;         // ragged M: compute on a valid row block, never stored
            v_base[x] = wave_uniform(reinterpret_cast<const uint8_t*>(a.A) + rb * KB64 * (1024 * ES) + (id & 1) * 1024);
            v_off[x] = lane * 16;
        }
#pragma unroll
        for (int x = 0; x < NJM; ++x) {
            const int id = wave * NJM + x;
            int64_t rb = (int64_t)tm * RB + id / T64;
            if (rb >= rb_total) rb = rb_total - 1;
            m_base[x] = wave_uniform(reinterpret_cast<const uint8_t*>(a.meta) + (rb * KB64 + id % T64) * 256);
            m_off[x] = lane * 4;
        }
    }
#pragma unroll
    for (int x = 0; x < NJV; ++x) v_base[x] += share.first * v_step;
#pragma unroll
    for (int x = 0; x < NJM; ++x) m_base[x] += share.first * m_step;

    // last, partial step (K not a whole number of steps; never with a convolution): which of this lane's transfers
    // lie past K.  A step holds tail bytes of every B row, tail/2 bytes of values and tail/(8*ES) bytes of codes
    // per A row; in the tiled layout a whole 64-column tile is present or absent.
    uint32_t past_k = 0;                                   // bit x: transfer x of this wavefront
    if (tail) {
#pragma unroll
        for (int x = 0; x < NJB; ++x) {
            const bool p = NMAJ ? past_k_nmajor<BN, NW, ES>(x, wave, lane, tail) : past_k_kmajor<BN, NW>(x, wave, lane, tail);
            past_k |= (uint32_t)p << x;
        }
        const int h = lane >> 5;
#pragma unroll
        for (int x = 0; x < NJV; ++x) {
            const int id = wave * NJV + x;
            const int col = (ES == 1) ? 32 * (id & 1) + 16 * h : 32 * h + 16 * (id & 1);     // byte of the 64 value bytes of a row and step
            const bool p = canonical ? col >= tail / 2 : ((ES == 1) ? 64 * (id & 1) >= tail : false);
            past_k |= (uint32_t)p << (NJB + x);
        }
#pragma unroll
        for (int x = 0; x < NJM; ++x) {
            const int id = wave * NJM + x;
            const bool p = canonical ? (8 * (id % T64) + 4 * h) * 8 * ES >= tail : 64 * ES * (id % T64) >= tail;
            past_k |= (uint32_t)p << (NJB + NJV + x);
        }
    }

    auto stage_ptr = [&](int u) -> uint8_t* { return lds_all + u * kStageBytes; };
    // transfer number x (0 .. NV-1) of this wavefront for a step: B rows, then values, then codes
    // (convolution: `tap` is the position of `step` in the inner dimension)
    // `partial_tag` (compile time): the step is the partial one past the last whole step; pieces past K are zeros.
    // The main loop only ever fetches whole steps, so that a step stays one basic block.
    auto dma_one = [&](int step, const ConvTap& tap, int u, int x, auto partial_tag) {
        uint8_t* stg = stage_ptr(u);
        constexpr bool partial = decltype(partial_tag)::value && !CONV;
        const bool pk = (past_k >> x) & 1u;
        if (x < NJB) {
            uint8_t* dst = stg + (wave * NJB + x) * 1024;
            if constexpr (CONV) b_conv.issue(x, reinterpret_cast<const uint8_t*>(a.B), a.conv, tap, stg, wave);
            else if (partial) lds_dma_tail<false>(b_blk + (int64_t)step * b_step, b_off[x], pk, dst);
            else lds_dma16(b_blk + (int64_t)step * b_step, b_off[x], dst);
        } else if (x < NJB + NJV) {
            uint8_t* dst = stg + kVOff + (wave * NJV + x - NJB) * 1024;
            if (partial) lds_dma_tail<false>(v_base[x - NJB] + (int64_t)step * v_step, v_off[x - NJB], pk, dst);
            else lds_dma16(v_base[x - NJB] + (int64_t)step * v_step, v_off[x - NJB], dst);
        } else {
            uint8_t* dst = stg + kMOff + (wave * NJM + x - NJB - NJV) * 256;
            if (partial) lds_dma_tail<true>(m_base[x - NJB - NJV] + (int64_t)step * m_step, m_off[x - NJB - NJV], pk, dst);
            else lds_dma4(m_base[x - NJB - NJV] + (int64_t)step * m_step, m_off[x - NJB - NJV], dst);
        }
    };
    auto dma = [&](int step, const ConvTap& tap, int u) {
#pragma unroll
        for (int x = 0; x < NV; ++x) dma_one(step, tap, u, x, std::false_type{});
    };
    // the step whose transfers are issued next, kept NS - 1 ahead of the arithmetic.  It stops at the last step:
    // past the end that step is fetched again into a stage nobody reads, which keeps the counts uniform.
    int f_step = 0;
    ConvTap f_tap = {0, 0, 0};
    auto advance_fetch = [&]() {
        if (f_step + 1 < nsteps) {
            ++f_step;
            if constexpr (CONV) f_tap.next(a.conv, BK);
        }
    };

    acc_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = acc_t{};

    // B fragment read offsets: row (wn*32*TN + nj*32 + r), piece c = 2*c2 + q at slot c ^ ((r >> 1) & 7)
    int frag_off[4];
#pragma unroll
    for (int c2 = 0; c2 < 4; ++c2) frag_off[c2] = (wn * 32 * TN + r) * kRowBytes + ((((2 * c2) | q) ^ ((r >> 1) & 7)) << 4);
    nmajor_frags<BN, TN, ES> b_nm;
    if constexpr (NMAJ) b_nm.init(wn, lane);
    const int va_off = kVOff + wm * TM * 2048 + lane * 16;
    const int ma_off = kMOff + wm * TM * T64 * 256 + lane * 4;

    // Operand reads from a stage.  A operands of matrix-core instruction j of the step: values (row block i,
    // half j), codes (int8: tile j; 16-bit: the one tile, the instruction picks its half through abid).
    auto read_a = [&](const uint8_t* base, int j, int4v (&xa)[TM], int (&xm)[TM], bool with_codes) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            xa[i] = *reinterpret_cast<const int4v*>(base + va_off + (i * 2 + j) * 1024);
            if (with_codes) xm[i] = *reinterpret_cast<const int*>(base + ma_off + (i * T64 + (is8<DT> ? j : 0)) * 256);
        }
    };
    auto read_frag = [&](const uint8_t* base, int t, int8v& bv) {
        const int j = t / TN, nj = t % TN;
        // K-byte offset of the two pieces of instruction j: (int8) 64j + 32h + 16q, (16-bit) 64h + 32j + 16q
        const int c2lo = is8<DT> ? 2 * j : j, c2hi = is8<DT> ? 2 * j + 1 : 2 + j;
        uint4v lo, hi;
        if constexpr (NMAJ) {
            lo = b_nm.piece(base, c2lo, nj);
            hi = b_nm.piece(base, c2hi, nj);
        } else {
            lo = *reinterpret_cast<const uint4v*>(base + frag_off[c2lo] + nj * 32 * kRowBytes);
            hi = *reinterpret_cast<const uint4v*>(base + frag_off[c2hi] + nj * 32 * kRowBytes);
        }
        bv[0] = lo[0]; bv[1] = lo[1]; bv[2] = lo[2]; bv[3] = lo[3];
        bv[4] = hi[0]; bv[5] = hi[1]; bv[6] = hi[2]; bv[7] = hi[3];
    };

    // Operands carried from the tail of one step into the next: A operands of instruction 0, fragments 0 and 1.
    int4v a_first[TM];
    int m_first[TM];
    int8v f_first[2];

    // One step s (stage u holds its operands; fragments t = 0 .. NF-1, TM instructions each).  LDS reads run two
    // fragments ahead of the arithmetic, so by t = T1 every read of stage u has been issued.  One barrier per step,
    // before t = T1.  A wavefront arrives there when
    //   * its own transfers for step s+1 have landed (vmcnt counts in order: only those of the NS - 2 later steps,
    //     all issued by now, may still be in flight), and
    //   * its reads of stage u have returned (lgkmcnt 0).
    // Past the barrier, therefore, stage u+1 is complete and visible -- the first operands of step s+1 are read
    // while the last instructions of step s run, so that no wavefront starts a step waiting for LDS -- and stage u
    // is free: the transfers for step s+NS go there, dealt out between the matrix instructions from here to the
    // next barrier (the first 2 of NF fragments' worth in this step, the rest at t < T1 of step s+1).
    constexpr int NF = 2 * TN, T1 = NF - 2;
    constexpr int kWait = waitcnt_vm((NS - 2) * NV);
    constexpr int kWaitAndReads = kWait & ~(15 << 8);      // the same, and lgkmcnt 0
    // transfer numbers dealt to slot m of the NF * TM matrix instructions between two barriers
    auto dma_slot = [&](int m, int u) {
#pragma unroll
        for (int x = m * NV / (NF * TM); x < (m + 1) * NV / (NF * TM); ++x) dma_one(f_step, f_tap, u, x, std::false_type{});
    };
    auto do_step = [&](int u) {
        const uint8_t* cur = stage_ptr(u);
        const uint8_t* nxt = stage_ptr((u + 1) % NS);
        int4v av[2][TM];
        int mv[2][TM];
        int8v f[3];
#pragma unroll
        for (int i = 0; i < TM; ++i) { av[0][i] = a_first[i]; mv[0][i] = m_first[i]; }
        f[0] = f_first[0];
        f[1] = f_first[1];
#pragma unroll
        for (int t = 0; t < NF; ++t) {
            const int j = t / TN, nj = t % TN;
            if (t == T1) {
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_waitcnt(kWaitAndReads);
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                advance_fetch();                         // from here on: the transfers of step s+NS, into stage u
            }
            if (t + 2 < NF) read_frag(cur, t + 2, f[(t + 2) % 3]);
            else read_frag(nxt, t + 2 - NF, f_first[t + 2 - NF]);
            if (t == 0) read_a(cur, 1, av[1], mv[1], is8<DT>);
            if (t == T1) read_a(nxt, 0, a_first, m_first, true);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if constexpr (is8<DT>) acc[i][nj] = smfmac32<DT, 0>(av[j][i], f[t % 3], acc[i][nj], mv[j][i]);
                else if (j == 0) acc[i][nj] = smfmac32<DT, 0>(av[0][i], f[t % 3], acc[i][nj], mv[0][i]);
                else acc[i][nj] = smfmac32<DT, 1>(av[1][i], f[t % 3], acc[i][nj], mv[0][i]);
                if (t < T1) dma_slot(2 * TM + t * TM + i, (u + NS - 1) % NS);
                else dma_slot((t - T1) * TM + i, u);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    if (nsteps > 0) {
        // prologue: the first NS - 1 stages on their way, and of the next step what a step issues after its barrier;
        // first operands of step 0 once stage 0 has landed (the wait leaves room for the NS - 2 later stages only,
        // a few transfers more than it must)
#pragma unroll
        for (int u = 0; u < NS - 1; ++u) {
            dma(f_step, f_tap, u);
            advance_fetch();
        }
#pragma unroll
        for (int m = 0; m < 2 * TM; ++m) dma_slot(m, NS - 1);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(kWait);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        read_a(lds_all, 0, a_first, m_first, true);
        read_frag(lds_all, 0, f_first[0]);
        read_frag(lds_all, 1, f_first[1]);
        __builtin_amdgcn_sched_barrier(0);
        // NS steps per iteration, so that stage indices are compile-time constants; the remainder runs after the loop
        int step = 0;
        for (; step + NS <= nsteps; step += NS) {
#pragma unroll
            for (int u = 0; u < NS; ++u) do_step(u);
        }
#pragma unroll
        for (int u = 0; u < NS - 1; ++u)
            if (step + u < nsteps) do_step(u);
    }
    // the surplus transfers have landed and every wavefront is done with the stages
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (!CONV && tail != 0) {
        // K is not a whole number of steps: one more, partial step on its own -- fetched into stage 0 with every
        // piece past K replaced by zeros, then computed without overlap (it happens once per tile)
#pragma unroll
        for (int x = 0; x < NV; ++x) dma_one(nsteps, f_tap, 0, x, std::true_type{});
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        int4v av[2][TM];
        int mv[2][TM];
        read_a(lds_all, 0, av[0], mv[0], true);
        read_a(lds_all, 1, av[1], mv[1], is8<DT>);
#pragma unroll
        for (int t = 0; t < NF; ++t) {
            const int j = t / TN, nj = t % TN;
            int8v fb;
            read_frag(lds_all, t, fb);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if constexpr (is8<DT>) acc[i][nj] = smfmac32<DT, 0>(av[j][i], fb, acc[i][nj], mv[j][i]);
                else if (j == 0) acc[i][nj] = smfmac32<DT, 0>(av[0][i], fb, acc[i][nj], mv[0][i]);
                else acc[i][nj] = smfmac32<DT, 1>(av[1][i], fb, acc[i][nj], mv[0][i]);
            }
        }
        __builtin_amdgcn_s_barrier();                // every wavefront has read stage 0 before it becomes store scratch
        __builtin_amdgcn_sched_barrier(0);
    }
    // LDS becomes store scratch
    store_wave_tile<DT, OUT, TM, TN>(a, acc, lds_all + wave * epilogue_geometry<OUT, TN>::kWaveBytes,
                                     (int64_t)tm * BM + wm * TM * 32, (int64_t)tn * BN + wn * TN * 32, lane);
}

// ---------------------------------------------------------------------------
// Dense kernel: the speedup denominator (Sec. 3.2, Fig. 3).  A and B both go
// through LDS (A is plain row-major, so its fragments are not contiguous in
// memory); NS stages, transfers NS - 1 steps ahead.
// ---------------------------------------------------------------------------
template <int DT, int OUT, int WM, int WN, int TM, int TN, int NS, int BSRC>
__global__ __launch_bounds__(64 * WM * WN, 1) void k_gemm_pipe(MmArgs a, int tiles_m, int tiles_n)
{
    constexpr bool CONV = BSRC == 1, NMAJ = BSRC == 2;
    constexpr int ES = is8<DT> ? 1 : 2;
    constexpr int BK = kRowBytes / ES;
    constexpr int NW = WM * WN;
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    constexpr int NJA = BM / 8 / NW, NJB = BN / 8 / NW;
    constexpr int kStageBytes = (BM + BN) * kRowBytes;
    using acc_t = typename acc_of<DT>::type;
    constexpr int kEpiBytes = NW * epilogue_geometry<OUT, TN>::kWaveBytes;
    static_assert(NS >= 2 && (NS - 2) * (NJA + NJB) <= 63, "at least two stages; vmcnt is a 6-bit counter");
    constexpr int kLdsBytes = NS * kStageBytes > kEpiBytes ? NS * kStageBytes : kEpiBytes;
    __shared__ __attribute__((aligned(1024))) uint8_t lds_all[kLdsBytes];

    int tm, tn;
    tile_of_workgroup(tiles_m, tiles_n, tm, tn);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int r = lane & 31, q = lane >> 5;
    // whole steps, and the bytes of K in a further, partial step (0: none), of this workgroup's share of K
    const KRange share = k_range_of_workgroup(a, (int)(a.K / BK), (int)((a.K * ES) % kRowBytes));
    const int nsteps = share.nsteps, tail = share.tail;

    const int64_t lda_bytes = a.lda * ES, ldb_bytes = a.ldb * ES;
    const int64_t b_step = NMAJ ? (int64_t)BK * ldb_bytes : (int64_t)kRowBytes;
    const uint8_t* a_blk = reinterpret_cast<const uint8_t*>(a.A) + (int64_t)tm * BM * lda_bytes + (int64_t)share.first * kRowBytes;
    const uint8_t* b_blk = reinterpret_cast<const uint8_t*>(a.B) + (NMAJ ? (int64_t)tn * BN * ES : (int64_t)tn * BN * ldb_bytes) +
                           share.first * b_step;
    uint32_t a_off[NJA], b_off[NJB];
    dma_offsets<BM, NW>((int64_t)tm * BM, a.M, lda_bytes, wave, lane, a_off);
    conv_rows<BN, NW, ES> b_conv;
    if constexpr (CONV) b_conv.init(a.conv, (int64_t)tn * BN, a.N, wave, lane);
    else if constexpr (NMAJ) dma_offsets_nmajor<BN, NW, ES>((int64_t)tn * BN, a.N, ldb_bytes, wave, lane, b_off);
    else dma_offsets<BN, NW>((int64_t)tn * BN, a.N, ldb_bytes, wave, lane, b_off);
    nmajor_frags<BN, TN, ES> b_nm;
    if constexpr (NMAJ) b_nm.init(wn, lane);

    acc_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = acc_t{};

    auto stage_ptr = [&](int u) -> uint8_t* { return lds_all + u * kStageBytes; };
    // (convolution: `tap` is the position of `step` in the inner dimension)
    // the partial step past the last whole one: pieces past K come from the zero row
    auto dma_partial = [&](int step, int u) {
        if constexpr (!CONV) {
#pragma unroll
            for (int j = 0; j < NJA; ++j)
                lds_dma_tail<false>(a_blk + (int64_t)step * kRowBytes, a_off[j], past_k_kmajor<BM, NW>(j, wave, lane, tail),
                                    stage_ptr(u) + (wave * NJA + j) * 1024);
#pragma unroll
            for (int j = 0; j < NJB; ++j)
                lds_dma_tail<false>(b_blk + (int64_t)step * b_step, b_off[j],
                                    NMAJ ? past_k_nmajor<BN, NW, ES>(j, wave, lane, tail) : past_k_kmajor<BN, NW>(j, wave, lane, tail),
                                    stage_ptr(u) + BM * kRowBytes + (wave * NJB + j) * 1024);
        }
    };
    auto dma = [&](int step, const ConvTap& tap, int u) {
        dma_rows<BM, NW>(a_blk + (int64_t)step * kRowBytes, a_off, stage_ptr(u), wave);
        if constexpr (CONV) {
#pragma unroll
            for (int j = 0; j < NJB; ++j)
                b_conv.issue(j, reinterpret_cast<const uint8_t*>(a.B), a.conv, tap, stage_ptr(u) + BM * kRowBytes, wave);
        } else dma_rows<BN, NW>(b_blk + (int64_t)step * b_step, b_off, stage_ptr(u) + BM * kRowBytes, wave);
    };
    // the step whose transfers are issued next, NS - 1 ahead of the arithmetic; it stops at the last step, which
    // is then fetched again into stages nobody reads
    int f_step = 0;
    ConvTap f_tap = {0, 0, 0};
    auto advance_fetch = [&]() {
        if (f_step + 1 < nsteps) {
            ++f_step;
            if constexpr (CONV) f_tap.next(a.conv, BK);
        }
    };

    // fragment of instruction jj (k-bytes 32*jj .. +31 of the step): lane reads piece 2*jj + q of its row
    int fa_off[4], fb_off[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        const int slot = (((2 * jj) | q) ^ ((r >> 1) & 7)) << 4;
        fa_off[jj] = (wm * 32 * TM + r) * kRowBytes + slot;
        fb_off[jj] = (BM + wn * 32 * TN + r) * kRowBytes + slot;
    }

    // the fragments of sub-step jj (32 bytes of K) of a stage
    auto read_frags = [&](const uint8_t* base, int jj, int4v (&xa)[TM], int4v (&xb)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i) xa[i] = *reinterpret_cast<const int4v*>(base + fa_off[jj] + i * 32 * kRowBytes);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if constexpr (NMAJ) xb[j] = __builtin_bit_cast(int4v, b_nm.piece(base + BM * kRowBytes, jj, j));
            else xb[j] = *reinterpret_cast<const int4v*>(base + fb_off[jj] + j * 32 * kRowBytes);
        }
    };
    // a whole stage on its own (the partial last step)
    auto compute = [&](int u) {
        const uint8_t* base = stage_ptr(u);
        int4v fa[2][TM], fb[2][TN];
        read_frags(base, 0, fa[0], fb[0]);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            if (jj + 1 < 4) read_frags(base, jj + 1, fa[(jj + 1) & 1], fb[(jj + 1) & 1]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i) acc[i][j] = mfma32<DT>(fa[jj & 1][i], fb[jj & 1][j], acc[i][j]);
        }
    };

    // One step s (stage u), four sub-steps of TM * TN matrix instructions; fragments are read one sub-step ahead, so
    // when sub-step 3 begins every read of stage u has been issued.  One barrier per step, before sub-step 3, as in
    // the sparse kernel: a wavefront arrives when its transfers for step s+1 have landed and its reads of stage u
    // have returned; past it stage u+1 is visible (its first fragments are read under the last sub-step) and stage u
    // is free for the transfers of step s+NS.  With two stages those are all issued right behind the barrier -- the
    // stage is needed again one step later -- else they are spread over the matrix instructions up to the next one.
    constexpr int NV = NJA + NJB;
    constexpr int kSlots = (NS == 2) ? TM * TN : 4 * TM * TN;   // matrix instructions the NV transfers are dealt over
    constexpr int kBehindBarrier = TM * TN * NV / kSlots;       // transfers issued in sub-step 3
    constexpr int kWaitAndReads = waitcnt_vm((NS - 2) * NV) & ~(15 << 8);
    auto dma_one = [&](int step, const ConvTap& tap, int u, int x) {
        if (x < NJA) lds_dma16(a_blk + (int64_t)step * kRowBytes, a_off[x], stage_ptr(u) + (wave * NJA + x) * 1024);
        else if constexpr (CONV) b_conv.issue(x - NJA, reinterpret_cast<const uint8_t*>(a.B), a.conv, tap, stage_ptr(u) + BM * kRowBytes, wave);
        else lds_dma16(b_blk + (int64_t)step * b_step, b_off[x - NJA], stage_ptr(u) + BM * kRowBytes + (wave * NJB + x - NJA) * 1024);
    };
    auto dma_slot = [&](int m, int u) {
        if (m < kSlots) {
#pragma unroll
            for (int x = m * NV / kSlots; x < (m + 1) * NV / kSlots; ++x) dma_one(f_step, f_tap, u, x);
        }
    };
    int4v fa_first[TM], fb_first[TN];                        // sub-step 0 of the next step
    auto do_step = [&](int u) {
        const uint8_t* cur = stage_ptr(u);
        const uint8_t* nxt = stage_ptr((u + 1) % NS);
        int4v fa[2][TM], fb[2][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[0][i] = fa_first[i];
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[0][j] = fb_first[j];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            if (jj == 3) {
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_waitcnt(kWaitAndReads);
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                advance_fetch();                             // from here on: the transfers of step s+NS, into stage u
            }
            if (jj < 3) read_frags(cur, jj + 1, fa[(jj + 1) & 1], fb[(jj + 1) & 1]);
            else read_frags(nxt, 0, fa_first, fb_first);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    acc[i][j] = mfma32<DT>(fa[jj & 1][i], fb[jj & 1][j], acc[i][j]);
                    if (jj == 3) dma_slot(j * TM + i, u);
                    else dma_slot((jj + 1) * TM * TN + j * TM + i, (u + NS - 1) % NS);
                }
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    if (nsteps > 0) {
        // the first NS - 1 stages on their way, and of the next step what a step issues behind its barrier; the
        // first fragments once stage 0 has landed
#pragma unroll
        for (int u = 0; u < NS - 1; ++u) {
            dma(f_step, f_tap, u);
            advance_fetch();
        }
#pragma unroll
        for (int m = 0; m < TM * TN; ++m) dma_slot(m, NS - 1);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(waitcnt_vm((NS - 2) * NV + kBehindBarrier));
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(lds_all, 0, fa_first, fb_first);
        __builtin_amdgcn_sched_barrier(0);
        int step = 0;
        for (; step + NS <= nsteps; step += NS) {
#pragma unroll
            for (int u = 0; u < NS; ++u) do_step(u);
        }
#pragma unroll
        for (int u = 0; u < NS - 1; ++u)
            if (step + u < nsteps) do_step(u);
    }
    // the surplus transfers have landed and every wavefront is done with the stages
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (!CONV && tail != 0) {
        // K is not a whole number of steps: one more, partial step on its own (pieces past K are zeros)
        dma_partial(nsteps, 0);
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        compute(0);
        __builtin_amdgcn_s_barrier();                // every wavefront has read stage 0 before it becomes store scratch
        __builtin_amdgcn_sched_barrier(0);
    }
    // LDS becomes store scratch
    store_wave_tile<DT, OUT, TM, TN>(a, acc, lds_all + wave * epilogue_geometry<OUT, TN>::kWaveBytes,
                                     (int64_t)tm * BM + wm * TM * 32, (int64_t)tn * BN + wn * TN * 32, lane);
}

// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------
// NSS / NSD: pipeline stages of the sparse / dense kernel; CONVS: whether the tile shape serves convolutions too
// (a shape that never does is not compiled for them)
template <int DT, int OUT, int WM, int WN, int TM, int TN, int NSS, int NSD, bool CONVS = true>
static sp24_status run_pipe(const MmArgs& a, hipStream_t st)
{
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    const dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)(a.k_slices > 1 ? a.k_slices : 1)), block(64 * WM * WN);
    if constexpr (!CONVS) {
        if (a.conv.on) return SP24_ERR_LAUNCH;
        if (a.sparse) {
            if (a.bo == SP24_B_NMAJOR) k_spmm_pipe<DT, OUT, WM, WN, TM, TN, NSS, 2><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
            else k_spmm_pipe<DT, OUT, WM, WN, TM, TN, NSS, 0><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
        } else {
            if (a.bo == SP24_B_NMAJOR) k_gemm_pipe<DT, OUT, WM, WN, TM, TN, NSD, 2><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
            else k_gemm_pipe<DT, OUT, WM, WN, TM, TN, NSD, 0><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
        }
        return hipGetLastError() == hipSuccess ? SP24_OK : SP24_ERR_LAUNCH;
    }
    if (a.sparse) {
        if (a.conv.on) k_spmm_pipe<DT, OUT, WM, WN, TM, TN, NSS, 1><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
        else if (a.bo == SP24_B_NMAJOR) k_spmm_pipe<DT, OUT, WM, WN, TM, TN, NSS, 2><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
        else k_spmm_pipe<DT, OUT, WM, WN, TM, TN, NSS, 0><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
    } else {
        if (a.conv.on) k_gemm_pipe<DT, OUT, WM, WN, TM, TN, NSD, 1><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
        else if (a.bo == SP24_B_NMAJOR) k_gemm_pipe<DT, OUT, WM, WN, TM, TN, NSD, 2><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
        else k_gemm_pipe<DT, OUT, WM, WN, TM, TN, NSD, 0><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
    }
    return hipGetLastError() == hipSuccess ? SP24_OK : SP24_ERR_LAUNCH;
}

template <int DT, int OUT>
static sp24_status pick_tile_general(const MmArgs& a, hipStream_t st)
{
    // 256x256 tiles when there are enough of them for half the chip, else 128x128
    const int64_t big = ((a.M + 255) / 256) * ((a.N + 255) / 256);
    // one workgroup of eight wavefronts of 64x128 each per compute unit (its wavefronts sit two to a SIMD, so that
    // one computes while the other waits).  The large tile moves half the operand bytes per product through the
    // L2 and LDS, and that outweighs idle compute units well below a full chip.  Measured on 100 - 192 large tiles,
    // K from 512 to 8192, operands from HBM: up to 128 large tiles the 512 small ones run in one round, two
    // workgroups to a unit, and the two shapes are level (the small one ahead by 10 - 17 % at K <= 1024); from
    // there on the small tiles need a second round and the large tile wins by 10 - 26 % (sparse), 3 - 38 % (dense).
    // The 16-bit dense product, the one that moves the most bytes per instruction, gains 7 - 14 % from 100 tiles on.
    // Convolutions follow the general rule (dense 16-bit at 108 tiles: the large tile 40 % slower; at 154 - 196: 7 - 20 %
    // faster, strided sparse ones 25 - 28 %).
    // -- unless the large tile would be mostly padding: rows and columns it covers beyond M and N are computed all the
    // same, and per product computed the small tile (two workgroups to a unit) costs about a third more
    const int64_t enough = (!a.conv.on && !is8<DT> && !a.sparse) ? 100 : 129;
    const double cover_big = (double)(((a.M + 255) / 256) * 256) * (double)(((a.N + 255) / 256) * 256);
    const double cover_small = (double)(((a.M + 127) / 128) * 128) * (double)(((a.N + 127) / 128) * 128);
    if (big >= enough && cover_big <= 1.35 * cover_small) return run_pipe<DT, OUT, 4, 2, 2, 4, 3, 2>(a, st);
    // 128x128 tiles, four wavefronts.  With few tiles one workgroup per compute unit is all there is, and a short
    // step (a quarter of the large tile's arithmetic) hides little latency: six (dense: four) stages, transfers
    // five (three) steps ahead.  With many tiles three (two) stages leave room for two workgroups per compute unit.
    const int64_t small = ((a.M + 127) / 128) * ((a.N + 127) / 128);
    // At most 128 of them: tiles of 64 rows, two wavefronts, put twice as many compute units to work.  Such a product
    // is bound by what one unit can keep in flight (its LDS ring against the latency of the L2 and of HBM), not
    // by arithmetic; the smaller stages also allow a deeper ring, and with N <= 64 a 64-column tile does not fetch
    // B rows that do not exist.  Measured on 16 shapes per type, operands from HBM: the sparse product 28 - 31 %
    // faster at N <= 64 (8192 x 64 x 8192 bf16: 43.8 -> 31.5 us), 6 - 17 % at N = 96 .. 128, 5 - 14 % on small
    // squarish shapes; the dense one 23 - 34 % and 15 - 25 % in a single column of tiles, but 10 - 15 % (16-bit)
    // slower with several, where halving the rows doubles the traffic of B: it keeps 128 rows there.
    // (Not for a product already split along K, whose slices fill the chip; not for convolutions, where the gather of
    // B is the cost and doubles with it: strided 3x3 layers with 13 - 98 tiles were 20 - 30 % slower.)
    if (small <= 128 && !a.conv.on && a.k_slices <= 1 && (a.sparse || a.N <= 128)) {
        if (a.N <= 64) return run_pipe<DT, OUT, 2, 1, 1, 2, 9, 9, false>(a, st);
        return run_pipe<DT, OUT, 2, 1, 1, 4, 7, 6, false>(a, st);
    }
    if (small <= 256) return run_pipe<DT, OUT, 2, 2, 2, 2, 6, 4>(a, st);
    return run_pipe<DT, OUT, 2, 2, 2, 2, 3, 2>(a, st);
}

} // namespace sp24
