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
//   - two s_barriers per step and no fence: a wavefront awaits its own
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

template <int ROWS, int NW>
__device__ __forceinline__ void dma_rows(const uint8_t* base, const uint32_t (&off)[ROWS / 8 / NW], uint8_t* stage, int wave)
{
#pragma unroll
    for (int j = 0; j < ROWS / 8 / NW; ++j)
        __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint4v*>(base + off[j]), (lds_ptr)(stage + (wave * (ROWS / 8 / NW) + j) * 1024), 16, 0, 0);
}

// Issue order of the first part of a sparse step, as a compile-time recursion (the sizes of
// sched_group_barrier must be constants): matrix-core instruction M of NMFMA is preceded, at the start of a
// fragment, by the two reads of the next fragment (and, in fragment 0, by the DSA1 reads of the second
// instruction's A operands) and followed by its share of the NV transfers.
template <int M, int NMFMA, int NV, int TM, int DSA1>
__device__ __forceinline__ void sparse_issue_order()
{
    if constexpr (M < NMFMA) {
        constexpr int t = M / TM, i = M % TM;
        if constexpr (i == 0) __builtin_amdgcn_sched_group_barrier(kSgDsRead, 2, 0);
        if constexpr (i == 0 && t == 0 && DSA1 > 0) __builtin_amdgcn_sched_group_barrier(kSgDsRead, DSA1, 0);
        __builtin_amdgcn_sched_group_barrier(kSgMfma, 1, 0);
        constexpr int nv = (M + 1) * NV / NMFMA - M * NV / NMFMA;
        if constexpr (nv > 0) __builtin_amdgcn_sched_group_barrier(kSgVmem, nv, 0);
        sparse_issue_order<M + 1, NMFMA, NV, TM, DSA1>();
    }
}

// ---------------------------------------------------------------------------
// Sparse kernel.  Stage layout: [B: BN rows x 128 B, swizzled][V: 2 KiB per
// 32-row block, in the tiled layout's own order][meta: 256 B per 32x64 tile].
// Three stages; the transfers for step s+2 are issued during step s, and the
// first operands of step s+1 are read from LDS during the tail of step s.
// ---------------------------------------------------------------------------
template <int DT, int OUT, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(64 * WM * WN, 1) void k_spmm_pipe(MmArgs a, int tiles_m, int tiles_n)
{
    constexpr int ES = (DT == SP24_I8) ? 1 : 2;
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
    __shared__ __attribute__((aligned(1024))) uint8_t st0[kStageBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t st1[kStageBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t st2[kStageBytes];

    int tm, tn;
    tile_of_workgroup(tiles_m, tiles_n, tm, tn);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int r = lane & 31, q = lane >> 5;
    const int64_t KB64 = a.K / 64;
    const int nsteps = (int)(a.K / BK);
    const int64_t rb_total = a.M / 32;

    // ---- transfers of this wavefront ----
    const int64_t ldb_bytes = a.ldb * ES;
    const uint8_t* b_blk = reinterpret_cast<const uint8_t*>(a.B) + (int64_t)tn * BN * ldb_bytes;
    uint32_t b_off[NJB];
    dma_offsets<BN, NW>((int64_t)tn * BN, a.N, ldb_bytes, wave, lane, b_off);
    // V: transfer x of this wavefront is 1 KiB number (wave*NJV + x) of the RB*2 of a step: row block /2, half %2
    const uint8_t* v_src[NJV];
#pragma unroll
    for (int x = 0; x < NJV; ++x) {
        const int id = wave * NJV + x;
        int64_t rb = (int64_t)tm * RB + (id >> 1);
        if (rb >= rb_total) rb = rb_total - 1;             // ragged M: compute on a valid row block, never stored
        v_src[x] = reinterpret_cast<const uint8_t*>(a.A) + rb * KB64 * (1024 * ES) + (id & 1) * 1024 + lane * 16;
    }
    // metadata: transfer x is 256-byte tile number (wave*NJM + x) of the RB*T64 of a step
    const uint8_t* m_src[NJM];
#pragma unroll
    for (int x = 0; x < NJM; ++x) {
        const int id = wave * NJM + x;
        int64_t rb = (int64_t)tm * RB + id / T64;
        if (rb >= rb_total) rb = rb_total - 1;
        m_src[x] = reinterpret_cast<const uint8_t*>(a.meta) + (rb * KB64 + id % T64) * 256 + lane * 4;
    }

    auto stage_ptr = [&](int u) -> uint8_t* { return u == 0 ? st0 : u == 1 ? st1 : st2; };
    auto dma = [&](int step, int u) {
        uint8_t* stg = stage_ptr(u);
        dma_rows<BN, NW>(b_blk + (int64_t)step * kRowBytes, b_off, stg, wave);
#pragma unroll
        for (int x = 0; x < NJV; ++x)
            __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint4v*>(v_src[x] + (int64_t)step * 2048),
                                             (lds_ptr)(stg + kVOff + (wave * NJV + x) * 1024), 16, 0, 0);
#pragma unroll
        for (int x = 0; x < NJM; ++x)
            __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(m_src[x] + (int64_t)step * (T64 * 256)),
                                             (lds_ptr)(stg + kMOff + (wave * NJM + x) * 256), 4, 0, 0);
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
    const int va_off = kVOff + wm * TM * 2048 + lane * 16;
    const int ma_off = kMOff + wm * TM * T64 * 256 + lane * 4;

    // Operand reads from a stage.  A operands of matrix-core instruction j of the step: values (row block i,
    // half j), codes (int8: tile j; 16-bit: the one tile, the instruction picks its half through abid).
    auto read_a = [&](const uint8_t* base, int j, int4v (&xa)[TM], int (&xm)[TM], bool with_codes) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            xa[i] = *reinterpret_cast<const int4v*>(base + va_off + (i * 2 + j) * 1024);
            if (with_codes) xm[i] = *reinterpret_cast<const int*>(base + ma_off + (i * T64 + (DT == SP24_I8 ? j : 0)) * 256);
        }
    };
    auto read_frag = [&](const uint8_t* base, int t, int8v& bv) {
        const int j = t / TN, nj = t % TN;
        // K-byte offset of the two pieces of instruction j: (int8) 64j + 32h + 16q, (16-bit) 64h + 32j + 16q
        const int c2lo = (DT == SP24_I8) ? 2 * j : j, c2hi = (DT == SP24_I8) ? 2 * j + 1 : 2 + j;
        uint4v lo = *reinterpret_cast<const uint4v*>(base + frag_off[c2lo] + nj * 32 * kRowBytes);
        uint4v hi = *reinterpret_cast<const uint4v*>(base + frag_off[c2hi] + nj * 32 * kRowBytes);
        bv[0] = lo[0]; bv[1] = lo[1]; bv[2] = lo[2]; bv[3] = lo[3];
        bv[4] = hi[0]; bv[5] = hi[1]; bv[6] = hi[2]; bv[7] = hi[3];
    };

    // Operands carried from the tail of one step into the next: A operands of instruction 0 and fragment 0.
    int4v a_first[TM];
    int m_first[TM];
    int8v f_first;

    // One step (stage u holds its operands; fragments t = 0 .. 2*TN-1, TM instructions each).
    //   barrier 0: every wavefront has finished the previous step, so the stage it read is free:
    //              the transfers for step s+2 go there, dealt out between the instructions of t < T1;
    //   barrier 1 (before t = T1): this wavefront's transfers for step s+1 have landed (vmcnt counts in order:
    //              only the NV just issued may still be in flight), the barrier makes everybody's visible;
    //   t >= T1:   the first operands of step s+1 are read while the last instructions of step s run, so that
    //              no wavefront starts a step waiting for LDS.
    constexpr int NF = 2 * TN, T1 = NF - 2;
    constexpr int kWait = waitcnt_vm(NV);
    constexpr int kCodeReads = (DT == SP24_I8) ? TM : 0;    // LDS reads of the codes of instruction 1
    auto do_step = [&](int step, int u) {
        const uint8_t* cur = stage_ptr(u);
        const uint8_t* nxt = stage_ptr((u + 1) % 3);
        int4v av[2][TM];
        int mv[2][TM];
        int8v f[2];
#pragma unroll
        for (int i = 0; i < TM; ++i) { av[0][i] = a_first[i]; mv[0][i] = m_first[i]; }
        f[0] = f_first;
        auto mfmas = [&](int t) {
            const int j = t / TN, nj = t % TN;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if constexpr (DT == SP24_I8) acc[i][nj] = smfmac32<DT, 0>(av[j][i], f[t & 1], acc[i][nj], mv[j][i]);
                else if (j == 0) acc[i][nj] = smfmac32<DT, 0>(av[0][i], f[t & 1], acc[i][nj], mv[0][i]);
                else acc[i][nj] = smfmac32<DT, 1>(av[1][i], f[t & 1], acc[i][nj], mv[0][i]);
            }
        };
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // past the end the last step is fetched again into a stage nobody reads: keeps the counts uniform
        dma(min(step + 2, nsteps - 1), (u + 2) % 3);
#pragma unroll
        for (int t = 0; t < T1; ++t) {
            read_frag(cur, t + 1, f[(t + 1) & 1]);
            if (t == 0) read_a(cur, 1, av[1], mv[1], DT == SP24_I8);
            mfmas(t);
        }
        sparse_issue_order<0, T1 * TM, NV, TM, TM + kCodeReads>();
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(kWait);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        read_frag(cur, T1 + 1, f[(T1 + 1) & 1]);
        read_a(nxt, 0, a_first, m_first, true);
        mfmas(T1);
        read_frag(nxt, 0, f_first);
        mfmas(T1 + 1);
        __builtin_amdgcn_sched_group_barrier(kSgDsRead, 2, 0);
        __builtin_amdgcn_sched_group_barrier(kSgMfma, 1, 0);
        __builtin_amdgcn_sched_group_barrier(kSgDsRead, 2 * TM, 0);
        __builtin_amdgcn_sched_group_barrier(kSgMfma, TM - 1, 0);
        __builtin_amdgcn_sched_group_barrier(kSgDsRead, 2, 0);
        __builtin_amdgcn_sched_group_barrier(kSgMfma, TM, 0);
        __builtin_amdgcn_sched_barrier(0);
    };

    // prologue: stages 0 and 1 on their way; first operands of step 0 once stage 0 has landed
    dma(0, 0);
    dma(min(1, nsteps - 1), 1);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(kWait);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    read_a(st0, 0, a_first, m_first, true);
    read_frag(st0, 0, f_first);
    __builtin_amdgcn_sched_barrier(0);
    // three steps per iteration in one basic block, so that stage indices are static and the compiler's
    // wait-count bookkeeping stays exact; the remainder runs after the loop
    int step = 0;
    for (; step + 3 <= nsteps; step += 3) {
        do_step(step, 0);
        do_step(step + 1, 1);
        do_step(step + 2, 2);
    }
    if (step < nsteps) do_step(step, 0);
    if (step + 1 < nsteps) do_step(step + 1, 1);
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
template <int DT, int OUT, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(64 * WM * WN, 1) void k_gemm_pipe(MmArgs a, int tiles_m, int tiles_n)
{
    constexpr int ES = (DT == SP24_I8) ? 1 : 2;
    constexpr int BK = kRowBytes / ES;
    constexpr int NW = WM * WN;
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    constexpr int NJA = BM / 8 / NW, NJB = BN / 8 / NW;
    constexpr int kStageBytes = (BM + BN) * kRowBytes;
    using acc_t = typename acc_of<DT>::type;
    __shared__ __attribute__((aligned(1024))) uint8_t st0[kStageBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t st1[kStageBytes];

    int tm, tn;
    tile_of_workgroup(tiles_m, tiles_n, tm, tn);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int r = lane & 31, q = lane >> 5;
    const int nsteps = (int)(a.K / BK);

    const int64_t lda_bytes = a.lda * ES, ldb_bytes = a.ldb * ES;
    const uint8_t* a_blk = reinterpret_cast<const uint8_t*>(a.A) + (int64_t)tm * BM * lda_bytes;
    const uint8_t* b_blk = reinterpret_cast<const uint8_t*>(a.B) + (int64_t)tn * BN * ldb_bytes;
    uint32_t a_off[NJA], b_off[NJB];
    dma_offsets<BM, NW>((int64_t)tm * BM, a.M, lda_bytes, wave, lane, a_off);
    dma_offsets<BN, NW>((int64_t)tn * BN, a.N, ldb_bytes, wave, lane, b_off);

    acc_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = acc_t{};

    auto stage_ptr = [&](int u) -> uint8_t* { return u == 0 ? st0 : st1; };
    auto dma = [&](int step, int u) {
        dma_rows<BM, NW>(a_blk + (int64_t)step * kRowBytes, a_off, stage_ptr(u), wave);
        dma_rows<BN, NW>(b_blk + (int64_t)step * kRowBytes, b_off, stage_ptr(u) + BM * kRowBytes, wave);
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
template <int DT, int OUT, int WM, int WN, int TM, int TN>
static sp24_status run_pipe(const MmArgs& a, hipStream_t st)
{
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(64 * WM * WN);
    if (a.sparse) k_spmm_pipe<DT, OUT, WM, WN, TM, TN><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
    else k_gemm_pipe<DT, OUT, WM, WN, TM, TN><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
    return hipGetLastError() == hipSuccess ? SP24_OK : SP24_ERR_LAUNCH;
}

template <int DT, int OUT>
static sp24_status pick_tile(const MmArgs& a, hipStream_t st)
{
    // 256x256 tiles when they still fill the 256 compute units, else 128x128
    const int64_t big = ((a.M + 255) / 256) * ((a.N + 255) / 256);
    // eight wavefronts of 64x128 each (two per SIMD, so that one computes while the other waits); measured
    // faster than four of 128x128 on the short-K transformer shape and equal on the long-K square one
    if (big >= 200) return run_pipe<DT, OUT, 4, 2, 2, 4>(a, st);
    return run_pipe<DT, OUT, 2, 2, 2, 2>(a, st);
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
