// Matrix multiply with a skinny second operand (N <= 32): the decode-like
// shape, bound by streaming the first operand from HBM once.
//
// One workgroup of 8 wavefronts per 32 rows of A.  The wavefronts split K in
// an interleaved way (64-column tile kb goes to wavefront kb % 8, so the
// workgroup as a whole reads A front to back), each keeps one 32x32
// accumulator tile (columns >= N are fed zeros), and the 8 partial tiles are
// summed through LDS in a fixed order.  The sparse variant reads the
// compressed operand in its tiled layout: per tile one contiguous 1 KiB (int8)
// or 2 KiB (16-bit) run of values and one 256-byte run of metadata words, 56 %
// (16-bit) or 62.5 % (8-bit) of the dense bytes -- the bandwidth saving of
// Sec. 3.1.  B is small (K x N) and is read straight from cache.
//
// In the dense variant every workgroup starts its sweep over K at a different
// tile and wraps around: with all of them at the same K at the same time, the
// rows of the row-major A -- a power-of-two pitch apart -- fall into the same
// memory channels.  Measured on 8192 x 8192 x 16 bf16: 29 -> 22 us inside the
// kernel.  The sparse variant reads one contiguous stream per workgroup front
// to back, with the tile addresses of a batch a constant apart (a start tile
// per workgroup cost it 10 %: an address computation per load).
#include "common.hpp"
#include "launch.hpp"
#include "mfma.hpp"

namespace sp24 {

constexpr int kSkinnyWaves = 8;
constexpr int kSkinnyUnroll = 4;   // tiles whose loads are in flight together, per wavefront

template <int DT, int OUT, bool SPARSE>
__global__ __launch_bounds__(64 * kSkinnyWaves) void k_mm_skinny(MmArgs a)
{
    constexpr int ES = is8<DT> ? 1 : 2;
    constexpr int TB = 64 * ES;                      // bytes of a B (or dense A) row per 64-column tile
    constexpr int NI = SPARSE ? (is8<DT> ? 1 : 2) : TB / 32;   // matrix-core instructions per tile
    using acc_t = typename acc_of<DT>::type;
    __shared__ uint32_t red[kSkinnyWaves][16][64];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, q = lane >> 5;
    const int64_t rb = blockIdx.x;
    // This workgroup's share of the inner dimension, in 64-column tiles: all of them, or (K split across gridDim.y
    // workgroups per row block) slice blockIdx.y, whose partial product goes to image blockIdx.y of D.  The operand
    // pointers below start at the share's first tile, and tile numbers and byte offsets count from there.
    int64_t kb_first = 0, KB64 = (a.K + 63) / 64;
    if (a.k_slices > 1) {
        kb_first = min((int64_t)blockIdx.y * a.slice_steps, KB64);
        KB64 = min((int64_t)a.slice_steps, KB64 - kb_first);
        a.D = reinterpret_cast<uint8_t*>(a.D) + (int64_t)blockIdx.y * a.M * a.ldd * 4;
    }
    const int64_t Kbytes = a.K * ES - kb_first * TB;
    const int64_t k_start = (SPARSE || KB64 == 0) ? 0 : (rb * 37) % KB64;   // this workgroup's first tile (dense only)

    const bool n_ok = r < a.N;
    const uint8_t* brow = reinterpret_cast<const uint8_t*>(a.B) + (int64_t)(n_ok ? r : 0) * a.ldb * ES + kb_first * TB;
    int64_t m = rb * 32 + r;
    if (m >= a.M) m = a.M - 1;                       // ragged M (dense only): rows past the end are never stored
    const uint8_t* arow = reinterpret_cast<const uint8_t*>(a.A) + m * a.lda * ES + kb_first * TB;
    const uint4v* Vp = reinterpret_cast<const uint4v*>(a.A);
    const uint32_t* Mp = reinterpret_cast<const uint32_t*>(a.meta);
    const int64_t tile_first = rb * (a.K / 64) + kb_first;   // tiled layout: this row block's first tile of the share
    // canonical layout: lane (m % 32, h) reads its slot's 16 bytes of values and 4 bytes of codes from row m
    const bool canonical = SPARSE && a.layout == SP24_LAYOUT_CANONICAL;
    const uint8_t* vrow = reinterpret_cast<const uint8_t*>(a.A) + m * (a.K / 2 * ES) + (ES == 1 ? 16 : 32) * q + kb_first * 32 * ES;
    const uint8_t* mrow = reinterpret_cast<const uint8_t*>(a.meta) + m * (a.K / 8) + 4 * q + kb_first * 8;

    acc_t acc = {};
    const uint4v zero4 = {0u, 0u, 0u, 0u};
    for (int64_t kb0 = wave; kb0 < KB64; kb0 += kSkinnyWaves * kSkinnyUnroll) {
        uint4v va[kSkinnyUnroll][SPARSE ? (ES == 1 ? 1 : 2) : NI];
        uint4v vb[kSkinnyUnroll][TB / 32];           // this lane's 16 bytes of every 32-byte piece of the tile's B row
        uint32_t codes[kSkinnyUnroll];
#pragma unroll
        for (int u = 0; u < kSkinnyUnroll; ++u) {
            const int64_t kbl = kb0 + (int64_t)u * kSkinnyWaves;
            const bool ok = kbl < KB64;
            int64_t kb = kbl;
            if constexpr (!SPARSE) {
                kb += k_start;                       // (with !ok nothing is loaded)
                if (kb >= KB64) kb -= KB64;
            }
            if constexpr (SPARSE) {
                const int64_t tile = tile_first + kb;
                if (canonical) {
                    codes[u] = ok ? *reinterpret_cast<const uint32_t*>(mrow + kb * 8) : 0u;
                    if constexpr (is8<DT>) va[u][0] = ok ? *reinterpret_cast<const uint4v*>(vrow + kb * 32) : zero4;
                    else {
                        va[u][0] = ok ? *reinterpret_cast<const uint4v*>(vrow + kb * 64) : zero4;
                        va[u][1] = ok ? *reinterpret_cast<const uint4v*>(vrow + kb * 64 + 16) : zero4;
                    }
                } else {
                    // the compressed operand passes once: loads marked as such leave B, which every workgroup re-reads,
                    // in the L2 (8192 x 8192 x 16 bf16 with the operand streamed from HBM: 21.1 -> 19.3 us)
                    codes[u] = ok ? __builtin_nontemporal_load(Mp + tile * 64 + lane) : 0u;
                    if constexpr (is8<DT>) va[u][0] = ok ? __builtin_nontemporal_load(Vp + tile * 64 + lane) : zero4;
                    else {
                        va[u][0] = ok ? __builtin_nontemporal_load(Vp + (tile * 2) * 64 + lane) : zero4;
                        va[u][1] = ok ? __builtin_nontemporal_load(Vp + (tile * 2 + 1) * 64 + lane) : zero4;
                    }
                }
            } else {
#pragma unroll
                for (int jj = 0; jj < NI; ++jj) {
                    const int64_t off = kb * TB + 32 * jj + 16 * q;
                    va[u][jj] = (ok && off < Kbytes) ? *reinterpret_cast<const uint4v*>(arow + off) : zero4;
                }
            }
            // B: every 16-byte piece of the tile's row that this lane may need (piece index 2*p + q)
#pragma unroll
            for (int p = 0; p < TB / 32; ++p) {
                const int64_t off = kb * TB + 32 * p + 16 * q;
                vb[u][p] = (ok && n_ok && off < Kbytes) ? *reinterpret_cast<const uint4v*>(brow + off) : zero4;
            }
        }
#pragma unroll
        for (int u = 0; u < kSkinnyUnroll; ++u) {
            if constexpr (SPARSE) {
                // instruction j takes the pieces at K-byte offsets (int8) 32h + 16q, (16-bit) 64h + 32j + 16q
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    const uint4v lo = is8<DT> ? vb[u][0] : vb[u][j];
                    const uint4v hi = is8<DT> ? vb[u][1] : vb[u][2 + j];
                    int8v bv;
                    bv[0] = lo[0]; bv[1] = lo[1]; bv[2] = lo[2]; bv[3] = lo[3];
                    bv[4] = hi[0]; bv[5] = hi[1]; bv[6] = hi[2]; bv[7] = hi[3];
                    const int4v av = __builtin_bit_cast(int4v, va[u][j]);
                    if (j == 0) acc = smfmac32<DT, 0>(av, bv, acc, (int)codes[u]);
                    else acc = smfmac32<DT, 1>(av, bv, acc, (int)codes[u]);
                }
            } else {
#pragma unroll
                for (int jj = 0; jj < NI; ++jj)
                    acc = mfma32<DT>(__builtin_bit_cast(int4v, va[u][jj]), __builtin_bit_cast(int4v, vb[u][jj]), acc);
            }
        }
    }

    // fixed-order sum of the partial tiles
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if constexpr (DT == SP24_I8) red[wave][i][lane] = (uint32_t)acc[i];
        else red[wave][i][lane] = __float_as_uint(acc[i]);
    }
    __syncthreads();
    for (int i = tid >> 6; i < 16; i += kSkinnyWaves) {   // accumulator registers handled by this thread
        const int64_t row = rb * 32 + 8 * (i / 4) + 4 * q + (i % 4);
        const int64_t col = r;
        if (row < a.M && col < a.N) {
            if constexpr (DT == SP24_I8) {
                int s = 0;
#pragma unroll
                for (int w = 0; w < kSkinnyWaves; ++w) s += (int)red[w][i][lane];
                float es = 0.0f, eb = 0.0f;
                if constexpr (OUT != SP24_I32) epilogue_row(a.epi, row, es, eb);
                store_bits<OUT>(a.D, row * a.ldd + col, output_bits<OUT>(s, es, eb, a.epi));
            } else {
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < kSkinnyWaves; ++w) s += __uint_as_float(red[w][i][lane]);
                store_out<OUT>(a.D, row * a.ldd + col, s);
            }
        }
    }
}

template <int DT, int OUT>
static sp24_status run_skinny(const MmArgs& a, hipStream_t st)
{
    const dim3 grid((unsigned)((a.M + 31) / 32), (unsigned)(a.k_slices > 1 ? a.k_slices : 1)), block(64 * kSkinnyWaves);
    if (a.sparse) k_mm_skinny<DT, OUT, true><<<grid, block, 0, st>>>(a);
    else k_mm_skinny<DT, OUT, false><<<grid, block, 0, st>>>(a);
    return hipGetLastError() == hipSuccess ? SP24_OK : SP24_ERR_LAUNCH;
}

sp24_status launch_mm_skinny(const MmArgs& a, hipStream_t st, bool* handled)
{
    *handled = false;
    const int es = esize_of(a.in);
    bool ok = a.N <= 32 && a.bo == SP24_B_KMAJOR && (reinterpret_cast<uintptr_t>(a.B) & 15u) == 0 && (a.ldb * es) % 16 == 0 &&
              a.M >= 32 && (a.M + 31) / 32 < ((int64_t)1 << 31);
    if (a.sparse && a.layout == SP24_LAYOUT_CANONICAL) ok = ok && a.K % 64 == 0;
    if (!ok) return SP24_OK;
    *handled = true;
    if (a.in == SP24_I8) {
        if (a.out == SP24_I32) return run_skinny<SP24_I8, SP24_I32>(a, st);
        if (a.out == SP24_I8) return run_skinny<SP24_I8, SP24_I8>(a, st);
        if (a.out == SP24_F32) return run_skinny<SP24_I8, SP24_F32>(a, st);
        if (a.out == SP24_F16) return run_skinny<SP24_I8, SP24_F16>(a, st);
        return run_skinny<SP24_I8, SP24_BF16>(a, st);
    }
    if (a.in == SP24_F8) {
        if (a.out == SP24_F32) return run_skinny<SP24_F8, SP24_F32>(a, st);
        if (a.out == SP24_F16) return run_skinny<SP24_F8, SP24_F16>(a, st);
        return run_skinny<SP24_F8, SP24_BF16>(a, st);
    }
    if (a.in == SP24_F16) {
        if (a.out == SP24_F32) return run_skinny<SP24_F16, SP24_F32>(a, st);
        if (a.out == SP24_F16) return run_skinny<SP24_F16, SP24_F16>(a, st);
        return run_skinny<SP24_F16, SP24_BF16>(a, st);
    }
    if (a.out == SP24_F32) return run_skinny<SP24_BF16, SP24_F32>(a, st);
    if (a.out == SP24_F16) return run_skinny<SP24_BF16, SP24_F16>(a, st);
    return run_skinny<SP24_BF16, SP24_BF16>(a, st);
}

} // namespace sp24
