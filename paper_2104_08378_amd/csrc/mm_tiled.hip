// Tiled, software-pipelined matrix-multiply kernels for large shapes.
//
// Sparse product (Sec. 3.2, Fig. 2) on the 32x32 sparse matrix-core
// instructions, and the same-shape dense product on the dense ones.  One
// workgroup of four wavefronts (2 x 2) computes a (64*TM) x (64*TN) tile of D;
// each wavefront owns TM x TN accumulator tiles of 32x32 and, in the 4 x 4
// configuration, the whole register file of its SIMD (256 accumulator
// registers), so nothing but the instruction order hides latencies:
//
//   - a step consumes 128 bytes of every B row (128 int8 / 64 16-bit values of K);
//   - B (and, in the dense kernel, A) travels global -> LDS without passing
//     through registers (global_load_lds, 16 bytes per lane) into a ring of
//     stages, several steps ahead of its use;
//   - the compressed A operand of the sparse kernel (tiled layout) goes
//     straight from global memory into registers, two steps ahead: one
//     contiguous 1 KiB run of values and one 256-byte run of metadata words
//     per 32-row tile (Sec. 3.1: no indirection, full-width reads);
//   - one s_barrier per step and no fence: a wavefront awaits its own
//     transfers with s_waitcnt vmcnt, the barrier then makes all four
//     wavefronts' transfers visible;
//   - memory instructions are dealt out between the matrix-core instructions
//     (sched_group_barrier), because with one wavefront per SIMD their issue
//     time is otherwise not overlapped with arithmetic;
//   - LDS rows are 128 bytes, unpadded (a transfer instruction fills 1 KiB =
//     8 rows contiguously); the 16-byte piece c of row n sits at slot
//     c ^ ((n >> 1) & 7), so that the fragment reads of 16 neighbouring rows
//     hit 16 different 16-byte columns of the 256-byte-wide bank array;
//   - workgroup ids are remapped so that the workgroups resident on one XCD
//     (ids congruent mod 8) cover a compact 8 x n block of tiles and share
//     their A and B panels in that XCD's L2.
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

// Transfer ROWS rows x 128 bytes (row r of the stage = global row min(row0 + r, limit - 1)) into a stage.
// Offsets of the NJ = ROWS/32 transfer instructions of this wavefront, relative to the first row.
template <int ROWS>
__device__ __forceinline__ void dma_offsets(int64_t row0, int64_t limit, int64_t ld_bytes, int wave, int lane, uint32_t (&off)[ROWS / 32])
{
#pragma unroll
    for (int j = 0; j < ROWS / 32; ++j) {
        const int row = (wave * (ROWS / 32) + j) * 8 + (lane >> 3);
        int64_t g = row0 + row;
        if (g >= limit) g = limit - 1;                       // ragged edge: fetch a valid row, never stored
        const int piece = (lane & 7) ^ ((row >> 1) & 7);
        off[j] = (uint32_t)((g - row0) * ld_bytes + piece * 16);
    }
}

template <int ROWS>
__device__ __forceinline__ void dma_rows(const uint8_t* base, const uint32_t (&off)[ROWS / 32], uint8_t* stage, int wave)
{
#pragma unroll
    for (int j = 0; j < ROWS / 32; ++j)
        __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint4v*>(base + off[j]), (lds_ptr)(stage + (wave * (ROWS / 32) + j) * 1024), 16, 0, 0);
}

// ---------------------------------------------------------------------------
// Sparse kernel.
// ---------------------------------------------------------------------------
template <int DT, int OUT, int TM, int TN>
__global__ __launch_bounds__(256, 1) void k_spmm_pipe(MmArgs a, int tiles_m, int tiles_n)
{
    constexpr int ES = (DT == SP24_I8) ? 1 : 2;
    constexpr int BK = kRowBytes / ES;        // K elements per step
    constexpr int T64 = BK / 64;              // 32x64 A tiles per step and row block (2 for int8, 1 for 16-bit)
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int NJ = BN / 32;               // B transfer instructions per wavefront and step
    constexpr int NA = TM * (2 + T64);        // A load instructions per wavefront and step
    constexpr int NMFMA = 2 * TM * TN;
    constexpr int kStageBytes = BN * kRowBytes;
    using acc_t = typename acc_of<DT>::type;
    __shared__ __attribute__((aligned(1024))) uint8_t st0[kStageBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t st1[kStageBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t st2[kStageBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t st3[kStageBytes];

    int tm, tn;
    tile_of_workgroup(tiles_m, tiles_n, tm, tn);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 31, q = lane >> 5;
    const int64_t KB64 = a.K / 64;
    const int nsteps = (int)(a.K / BK);
    const int64_t rb_total = a.M / 32;

    // A operand (tiled layout): first tile of each of this wavefront's row blocks
    const uint4v* __restrict__ Vp = reinterpret_cast<const uint4v*>(a.A);
    const uint32_t* __restrict__ Mp = reinterpret_cast<const uint32_t*>(a.meta);
    int64_t a_tile0[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int64_t rb = (int64_t)tm * (BM / 32) + wm * TM + i;
        if (rb >= rb_total) rb = rb_total - 1;               // ragged M: compute on a valid row block, never stored
        a_tile0[i] = rb * KB64;
    }

    // B transfers
    const int64_t ldb_bytes = a.ldb * ES;
    const uint8_t* b_blk = reinterpret_cast<const uint8_t*>(a.B) + (int64_t)tn * BN * ldb_bytes;
    uint32_t b_off[NJ];
    dma_offsets<BN>((int64_t)tn * BN, a.N, ldb_bytes, wave, lane, b_off);

    acc_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = acc_t{};

    uint4v a_reg[4][TM][2];
    uint32_t m_reg[4][TM][T64];

    auto stage_ptr = [&](int u) -> uint8_t* { return u == 0 ? st0 : u == 1 ? st1 : u == 2 ? st2 : st3; };
    auto load_a = [&](int step, int set) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if constexpr (DT == SP24_I8) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int64_t tile = a_tile0[i] + (int64_t)step * 2 + j;
                    a_reg[set][i][j] = (Vp + tile * 64)[lane];
                    m_reg[set][i][j] = (Mp + tile * 64)[lane];
                }
            } else {
                const int64_t tile = a_tile0[i] + step;
#pragma unroll
                for (int j = 0; j < 2; ++j) a_reg[set][i][j] = (Vp + (tile * 2 + j) * 64)[lane];
                m_reg[set][i][0] = (Mp + tile * 64)[lane];
            }
        }
    };
    auto dma_b = [&](int step, int u) { dma_rows<BN>(b_blk + (int64_t)step * kRowBytes, b_off, stage_ptr(u), wave); };

    // fragment read offsets inside a stage: row (wn*32*TN + nj*32 + r), piece c at slot c ^ ((r >> 1) & 7);
    // c = 2*c2 + q
    int frag_off[4];
#pragma unroll
    for (int c2 = 0; c2 < 4; ++c2) frag_off[c2] = (wn * 32 * TN + r) * kRowBytes + ((((2 * c2) | q) ^ ((r >> 1) & 7)) << 4);

    auto compute = [&](int u, int set) {
        const uint8_t* base = stage_ptr(u);
        auto read_frag = [&](int t, int8v& bv) {
            const int j = t / TN, nj = t % TN;
            // K-byte offset of the two pieces of instruction j: (int8) 64j + 32h + 16q, (16-bit) 64h + 32j + 16q
            const int c2lo = (DT == SP24_I8) ? 2 * j : j, c2hi = (DT == SP24_I8) ? 2 * j + 1 : 2 + j;
            uint4v lo = *reinterpret_cast<const uint4v*>(base + frag_off[c2lo] + nj * 32 * kRowBytes);
            uint4v hi = *reinterpret_cast<const uint4v*>(base + frag_off[c2hi] + nj * 32 * kRowBytes);
            bv[0] = lo[0]; bv[1] = lo[1]; bv[2] = lo[2]; bv[3] = lo[3];
            bv[4] = hi[0]; bv[5] = hi[1]; bv[6] = hi[2]; bv[7] = hi[3];
        };
        int8v f[2];
        read_frag(0, f[0]);
#pragma unroll
        for (int t = 0; t < 2 * TN; ++t) {
            // the next fragment is requested before, and awaited after, this fragment's TM instructions
            if (t + 1 < 2 * TN) read_frag(t + 1, f[(t + 1) & 1]);
            const int j = t / TN, nj = t % TN;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int4v av = __builtin_bit_cast(int4v, a_reg[set][i][j]);
                if constexpr (DT == SP24_I8) acc[i][nj] = smfmac32<DT, 0>(av, f[t & 1], acc[i][nj], (int)m_reg[set][i][j]);
                else if (j == 0) acc[i][nj] = smfmac32<DT, 0>(av, f[t & 1], acc[i][nj], (int)m_reg[set][i][0]);
                else acc[i][nj] = smfmac32<DT, 1>(av, f[t & 1], acc[i][nj], (int)m_reg[set][i][0]);
            }
        }
    };

    // One step.  Transfers issued during step s: A(s+2) into the register set two ahead and B(s+3) into the
    // stage three ahead.  vmcnt counts in order, so letting only the NA + NJ transfers of the previous step stay
    // in flight on entry means that everything issued up to two steps ago -- A(s) and B(s) among it -- has landed.
    constexpr int kWait = waitcnt_vm(NA + NJ);
    constexpr int kVmemPerMfma = (NA + NJ + NMFMA - 1) / NMFMA;
    auto do_step = [&](int step, int u, int as) {
        __builtin_amdgcn_s_waitcnt(kWait);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // past the end the same addresses are fetched again into stages nobody reads: keeps the counts uniform
        load_a(min(step + 2, nsteps - 1), (as + 2) & 3);
        dma_b(min(step + 3, nsteps - 1), (u + 3) & 3);
        compute(u, as);
        // issue order of this region: two fragment reads, then TM x { matrix-core instruction, transfers }
        __builtin_amdgcn_sched_group_barrier(kSgDsRead, 2, 0);
#pragma unroll
        for (int t = 0; t < 2 * TN; ++t) {
            if (t + 1 < 2 * TN) __builtin_amdgcn_sched_group_barrier(kSgDsRead, 2, 0);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                __builtin_amdgcn_sched_group_barrier(kSgMfma, 1, 0);
                __builtin_amdgcn_sched_group_barrier(kSgVmem, kVmemPerMfma, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // prologue, in the steady-state order: B(0) A(0) B(1) A(1) B(2)
    dma_b(0, 0);
    load_a(0, 0);
    dma_b(min(1, nsteps - 1), 1);
    load_a(min(1, nsteps - 1), 1);
    dma_b(min(2, nsteps - 1), 2);
    __builtin_amdgcn_sched_barrier(0);
    // four steps per iteration in one basic block, so that stage and register-set indices are static and the
    // compiler's wait-count bookkeeping stays exact; the remainder runs after the loop
    int step = 0;
    for (; step + 4 <= nsteps; step += 4) {
        do_step(step, 0, 0);
        do_step(step + 1, 1, 1);
        do_step(step + 2, 2, 2);
        do_step(step + 3, 3, 3);
    }
    if (step < nsteps) do_step(step, 0, 0);
    if (step + 1 < nsteps) do_step(step + 1, 1, 1);
    if (step + 2 < nsteps) do_step(step + 2, 2, 2);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));  // drain the surplus transfers before the stages go away

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int64_t row0 = (int64_t)tm * BM + (wm * TM + i) * 32;
            int64_t col0 = (int64_t)tn * BN + (wn * TN + j) * 32;
            store_tile<DT, OUT>(a.D, a.ldd, row0, col0, a.M, a.N, acc[i][j], lane);
        }
}

// ---------------------------------------------------------------------------
// Dense kernel: the speedup denominator (Sec. 3.2, Fig. 3).  A and B both go
// through LDS (A is plain row-major, so its fragments are not contiguous in
// memory); two stages, transfers one step ahead -- a dense step holds twice
// the arithmetic of a sparse one, which is what hides the latency here.
// ---------------------------------------------------------------------------
template <int DT, int OUT, int TM, int TN>
__global__ __launch_bounds__(256, 1) void k_gemm_pipe(MmArgs a, int tiles_m, int tiles_n)
{
    constexpr int ES = (DT == SP24_I8) ? 1 : 2;
    constexpr int BK = kRowBytes / ES;
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int NJA = BM / 32, NJB = BN / 32;
    constexpr int kStageBytes = (BM + BN) * kRowBytes;
    using acc_t = typename acc_of<DT>::type;
    __shared__ __attribute__((aligned(1024))) uint8_t st0[kStageBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t st1[kStageBytes];

    int tm, tn;
    tile_of_workgroup(tiles_m, tiles_n, tm, tn);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 31, q = lane >> 5;
    const int nsteps = (int)(a.K / BK);

    const int64_t lda_bytes = a.lda * ES, ldb_bytes = a.ldb * ES;
    const uint8_t* a_blk = reinterpret_cast<const uint8_t*>(a.A) + (int64_t)tm * BM * lda_bytes;
    const uint8_t* b_blk = reinterpret_cast<const uint8_t*>(a.B) + (int64_t)tn * BN * ldb_bytes;
    uint32_t a_off[NJA], b_off[NJB];
    dma_offsets<BM>((int64_t)tm * BM, a.M, lda_bytes, wave, lane, a_off);
    dma_offsets<BN>((int64_t)tn * BN, a.N, ldb_bytes, wave, lane, b_off);

    acc_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = acc_t{};

    auto stage_ptr = [&](int u) -> uint8_t* { return u == 0 ? st0 : st1; };
    auto dma = [&](int step, int u) {
        dma_rows<BM>(a_blk + (int64_t)step * kRowBytes, a_off, stage_ptr(u), wave);
        dma_rows<BN>(b_blk + (int64_t)step * kRowBytes, b_off, stage_ptr(u) + BM * kRowBytes, wave);
    };

    // fragment of instruction jj (k-bytes 32*jj .. +31 of the step): lane reads piece 2*jj + q of its row
    int fa_off[4], fb_off[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        const int slot = (((2 * jj) | q) ^ ((r >> 1) & 7)) << 4;
        fa_off[jj] = (wm * 32 * TM + r) * kRowBytes + slot;
        fb_off[jj] = (BM + wn * 32 * TN + r) * kRowBytes + slot;
    }

    auto compute = [&](int u) {
        const uint8_t* base = stage_ptr(u);
        int4v fa[2][TM], fb[2][TN];
        auto read_frags = [&](int jj, int4v (&xa)[TM], int4v (&xb)[TN]) {
#pragma unroll
            for (int i = 0; i < TM; ++i) xa[i] = *reinterpret_cast<const int4v*>(base + fa_off[jj] + i * 32 * kRowBytes);
#pragma unroll
            for (int j = 0; j < TN; ++j) xb[j] = *reinterpret_cast<const int4v*>(base + fb_off[jj] + j * 32 * kRowBytes);
        };
        read_frags(0, fa[0], fb[0]);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            if (jj + 1 < 4) read_frags(jj + 1, fa[(jj + 1) & 1], fb[(jj + 1) & 1]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i) acc[i][j] = mfma32<DT>(fa[jj & 1][i], fb[jj & 1][j], acc[i][j]);
        }
    };

    constexpr int NMFMA = 4 * TM * TN, NV = NJA + NJB;
    auto do_step = [&](int step, int u) {
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // this wavefront's share of stage u has landed
        __builtin_amdgcn_s_barrier();                // ... and everybody's; stage u^1 is no longer being read
        __builtin_amdgcn_sched_barrier(0);
        dma(min(step + 1, nsteps - 1), u ^ 1);
        compute(u);
        __builtin_amdgcn_sched_group_barrier(kSgDsRead, TM + TN, 0);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            if (jj + 1 < 4) __builtin_amdgcn_sched_group_barrier(kSgDsRead, TM + TN, 0);
#pragma unroll
            for (int i = 0; i < TM * TN; ++i) {
                __builtin_amdgcn_sched_group_barrier(kSgMfma, 1, 0);
                if ((jj * TM * TN + i) % (NMFMA / NV) == 0) __builtin_amdgcn_sched_group_barrier(kSgVmem, 1, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    dma(0, 0);
    __builtin_amdgcn_sched_barrier(0);
    int step = 0;
    for (; step + 2 <= nsteps; step += 2) {
        do_step(step, 0);
        do_step(step + 1, 1);
    }
    if (step < nsteps) do_step(step, 0);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int64_t row0 = (int64_t)tm * BM + (wm * TM + i) * 32;
            int64_t col0 = (int64_t)tn * BN + (wn * TN + j) * 32;
            store_tile<DT, OUT>(a.D, a.ldd, row0, col0, a.M, a.N, acc[i][j], lane);
        }
}

// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------
template <int DT, int OUT, int TM, int TN>
static sp24_status run_pipe(const MmArgs& a, hipStream_t st)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(256);
    if (a.sparse) k_spmm_pipe<DT, OUT, TM, TN><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
    else k_gemm_pipe<DT, OUT, TM, TN><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
    return hipGetLastError() == hipSuccess ? SP24_OK : SP24_ERR_LAUNCH;
}

template <int DT, int OUT>
static sp24_status pick_tile(const MmArgs& a, hipStream_t st)
{
    // 256x256 tiles when they still fill the 256 compute units, else 128x128
    const int64_t big = ((a.M + 255) / 256) * ((a.N + 255) / 256);
    if (big >= 200) return run_pipe<DT, OUT, 4, 4>(a, st);
    return run_pipe<DT, OUT, 2, 2>(a, st);
}

sp24_status launch_mm_tiled(const MmArgs& a, hipStream_t st, bool* handled)
{
    *handled = false;
    const int es = esize_of(a.in);
    bool ok = a.bo == SP24_B_KMAJOR && a.K % (kRowBytes / es) == 0 && (reinterpret_cast<uintptr_t>(a.B) & 15u) == 0 &&
              (a.ldb * es) % 16 == 0 && a.N >= 32 && a.M >= 64 && a.M <= ((int64_t)1 << 30) && a.N <= ((int64_t)1 << 30) &&
              a.ldb * es < ((int64_t)1 << 22) && ((a.M + 127) / 128) * ((a.N + 127) / 128) < ((int64_t)1 << 30);
    if (a.sparse) ok = ok && a.layout == SP24_LAYOUT_TILED;
    else ok = ok && a.lda * es < ((int64_t)1 << 22);
    if (!ok) return SP24_OK;
    *handled = true;
    if (a.in == SP24_I8) return pick_tile<SP24_I8, SP24_I32>(a, st);
    if (a.in == SP24_F16) {
        if (a.out == SP24_F32) return pick_tile<SP24_F16, SP24_F32>(a, st);
        if (a.out == SP24_F16) return pick_tile<SP24_F16, SP24_F16>(a, st);
        return pick_tile<SP24_F16, SP24_BF16>(a, st);
    }
    if (a.out == SP24_F32) return pick_tile<SP24_BF16, SP24_F32>(a, st);
    if (a.out == SP24_F16) return pick_tile<SP24_BF16, SP24_F16>(a, st);
    return pick_tile<SP24_BF16, SP24_BF16>(a, st);
}

} // namespace sp24
