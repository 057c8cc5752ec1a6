// Tiled matrix-multiply kernels for large aligned shapes.
//
// Sparse product (Sec. 3.2, Fig. 2) on the 32x32 sparse matrix-core
// instructions.  One workgroup of four wavefronts (2 x 2) computes a
// (64*TM) x (64*TN) tile of D; each wavefront owns TM x TN accumulator tiles
// of 32x32.  Per step of 128 bytes of a B row (128 int8 or 64 16-bit values
// of K):
//   - the compressed A operand (tiled layout) goes straight from global
//     memory into registers: one contiguous 1 KiB run of values and one
//     256-byte run of metadata words per 32-row tile, no LDS;
//   - the B tile (K-major rows) is staged through LDS, double-buffered, with
//     a row pitch of 144 bytes so that 16-byte fragment reads of 8
//     neighbouring rows fall in distinct banks;
//   - workgroup ids are remapped so that the workgroups resident on one XCD
//     (ids congruent mod 8) cover a compact 8 x n block of tiles and share
//     their A and B panels in that XCD's L2.
#include "common.hpp"
#include "launch.hpp"
#include "mfma.hpp"

namespace sp24 {

constexpr int kRowBytes = 128;           // bytes of one B row consumed per step
constexpr int kPitch = kRowBytes + 16;   // LDS row pitch

template <int DT, int OUT, int TM, int TN>
__global__ __launch_bounds__(256, 1) void k_spmm_tiled(MmArgs a, int tiles_m, int tiles_n)
{
    constexpr int ES = (DT == SP24_I8) ? 1 : 2;
    constexpr int BK = kRowBytes / ES;        // K elements per step
    constexpr int T64 = BK / 64;              // 32x64 A tiles per step and row block (2 for int8, 1 for 16-bit)
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int NLOAD = BN * (kRowBytes / 16) / 256; // 16-byte B loads per thread and step
    using acc_t = typename acc_of<DT>::type;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    // ---- workgroup -> tile, XCD-aware ----
    const int nwg = tiles_m * tiles_n;
    int wg = blockIdx.x;
    {
        // hardware deals consecutive ids round-robin over 8 XCDs: give each XCD a contiguous range
        const int per = (nwg + 7) / 8;
        const int xcd = wg & 7, idx = wg >> 3;
        const int full = nwg - (per - 1) * 8;   // XCDs that own `per` ids (the rest own per-1)
        wg = (xcd < full) ? xcd * per + idx : full * per + (xcd - full) * (per - 1) + idx;
    }
    // sweep tiles in groups of 8 along M, then along N
    constexpr int GM = 8;
    const int group = wg / (GM * tiles_n);
    const int first_m = group * GM;
    const int gsz = min(tiles_m - first_m, GM);
    const int in_group = wg - group * GM * tiles_n;
    const int tm = first_m + in_group % gsz, tn = in_group / gsz;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 31, q = lane >> 5;
    const int64_t KB64 = a.K / 64;
    const int nsteps = (int)(a.K / BK);
    const int64_t rb_total = a.M / 32;

    // ---- A operand addresses (tiled layout) ----
    const uint4v* __restrict__ Vp = reinterpret_cast<const uint4v*>(a.A);
    const uint32_t* __restrict__ Mp = reinterpret_cast<const uint32_t*>(a.meta);
    int64_t a_tile0[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int64_t rb = (int64_t)tm * (BM / 32) + wm * TM + i;
        if (rb >= rb_total) rb = rb_total - 1;          // ragged M: clamp loads, stores are predicated
        a_tile0[i] = rb * KB64;
    }

    // ---- B staging addresses ----
    const uint8_t* __restrict__ Bp = reinterpret_cast<const uint8_t*>(a.B);
    const int64_t ldb_bytes = a.ldb * ES;
    const uint8_t* b_src[NLOAD];
    int b_dst[NLOAD];
#pragma unroll
    for (int j = 0; j < NLOAD; ++j) {
        int id = tid + 256 * j;
        int row = id >> 3, c = id & 7;
        int64_t n = (int64_t)tn * BN + row;
        if (n >= a.N) n = a.N - 1;
        b_src[j] = Bp + n * ldb_bytes + c * 16;
        b_dst[j] = row * kPitch + c * 16;
    }
    constexpr int kBufBytes = BN * kPitch;

    acc_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = acc_t{};

    uint4v a_cur[TM][2], a_nxt[TM][2];
    uint32_t m_cur[TM][T64], m_nxt[TM][T64];
    uint4v b_stage[NLOAD];

    auto load_a = [&](int step, uint4v (&av)[TM][2], uint32_t (&mv)[TM][T64]) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if constexpr (DT == SP24_I8) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    int64_t tile = a_tile0[i] + (int64_t)step * 2 + j;
                    av[i][j] = Vp[tile * 64 + lane];
                    mv[i][j] = Mp[tile * 64 + lane];
                }
            } else {
                int64_t tile = a_tile0[i] + step;
#pragma unroll
                for (int j = 0; j < 2; ++j) av[i][j] = Vp[(tile * 2 + j) * 64 + lane];
                mv[i][0] = Mp[tile * 64 + lane];
            }
        }
    };
    auto load_b = [&](int step) {
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) b_stage[j] = *reinterpret_cast<const uint4v*>(b_src[j] + (int64_t)step * kRowBytes);
    };
    auto store_b = [&](int buf) {
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) *reinterpret_cast<uint4v*>(lds + buf * kBufBytes + b_dst[j]) = b_stage[j];
    };

    // prologue
    load_b(0);
    load_a(0, a_cur, m_cur);
    store_b(0);
    __syncthreads();

    for (int step = 0; step < nsteps; ++step) {
        const int buf = step & 1;
        const bool more = step + 1 < nsteps;
        if (more) {
            load_b(step + 1);
            load_a(step + 1, a_nxt, m_nxt);
        }
        const uint8_t* bt = lds + buf * kBufBytes + (wn * TN * 32 + r) * kPitch + 16 * q;
#pragma unroll
        for (int j = 0; j < 2; ++j) {           // the two matrix-core instructions of a step
#pragma unroll
            for (int nj = 0; nj < TN; ++nj) {
                // fragment: 16-byte pieces at K-byte offsets (int8) 64j + 32h + 16q, (16-bit) 64h + 32j + 16q
                const uint8_t* p = bt + nj * 32 * kPitch + ((DT == SP24_I8) ? 64 * j : 32 * j);
                constexpr int hstride = (DT == SP24_I8) ? 32 : 64;
                uint4v lo = *reinterpret_cast<const uint4v*>(p);
                uint4v hi = *reinterpret_cast<const uint4v*>(p + hstride);
                int8v bv;
                bv[0] = lo[0]; bv[1] = lo[1]; bv[2] = lo[2]; bv[3] = lo[3];
                bv[4] = hi[0]; bv[5] = hi[1]; bv[6] = hi[2]; bv[7] = hi[3];
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    int4v av = __builtin_bit_cast(int4v, a_cur[i][j]);
                    if constexpr (DT == SP24_I8) acc[i][nj] = smfmac32<DT, 0>(av, bv, acc[i][nj], (int)m_cur[i][j]);
                    else if (j == 0) acc[i][nj] = smfmac32<DT, 0>(av, bv, acc[i][nj], (int)m_cur[i][0]);
                    else acc[i][nj] = smfmac32<DT, 1>(av, bv, acc[i][nj], (int)m_cur[i][0]);
                }
            }
        }
        if (more) {
            store_b(buf ^ 1);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int j = 0; j < 2; ++j) a_cur[i][j] = a_nxt[i][j];
#pragma unroll
                for (int j = 0; j < T64; ++j) m_cur[i][j] = m_nxt[i][j];
            }
        }
        __syncthreads();
    }

    // ---- epilogue ----
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int64_t row0 = (int64_t)tm * BM + (wm * TM + i) * 32;
            int64_t col0 = (int64_t)tn * BN + (wn * TN + j) * 32;
            store_tile<DT, OUT>(a.D, a.ldd, row0, col0, a.M, a.N, acc[i][j], lane);
        }
}

template <int DT, int OUT, int TM, int TN>
static sp24_status run_spmm(const MmArgs& a, hipStream_t st)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    size_t lds_bytes = 2 * (size_t)BN * kPitch;
    auto kern = k_spmm_tiled<DT, OUT, TM, TN>;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
            return SP24_ERR_LAUNCH;
        attr_set = true;
    }
    kern<<<dim3((unsigned)(tiles_m * tiles_n)), dim3(256), lds_bytes, st>>>(a, tiles_m, tiles_n);
    return hipGetLastError() == hipSuccess ? SP24_OK : SP24_ERR_LAUNCH;
}

template <int DT, int OUT>
static sp24_status pick_tile(const MmArgs& a, hipStream_t st)
{
    // large tiles when they still fill the chip, else smaller ones
    int64_t big = ((a.M + 255) / 256) * ((a.N + 255) / 256);
    if (big >= 200) return run_spmm<DT, OUT, 4, 4>(a, st);
    return run_spmm<DT, OUT, 2, 2>(a, st);
}

sp24_status launch_mm_tiled(const MmArgs& a, hipStream_t st, bool* handled)
{
    *handled = false;
    if (!a.sparse) return SP24_OK;
    const int es = esize_of(a.in);
    const bool ok = a.layout == SP24_LAYOUT_TILED && a.bo == SP24_B_KMAJOR && a.K % (kRowBytes / es) == 0 &&
                    (reinterpret_cast<uintptr_t>(a.B) & 15u) == 0 && (a.ldb * es) % 16 == 0 && a.N >= 32 && a.M >= 64 &&
                    a.M * a.N < (int64_t)1 << 40;
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
