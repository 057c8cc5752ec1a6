// Sparse 3 x 3 convolution as an implicit GEMM with the input staged as a patch and the compressed filters read
// straight into registers (Sec. 3.2: convolutions are GEMM-like with the sparse tensor first; Sec. 4.2: inner
// dimension C x R x S; Sec. 3.1: the compressed operand needs no indirection and is read with full-width accesses).
//
// The kernel was written for outputs with too few tiles for the 256 x 256 shape: 128 x 128 tiles, one workgroup of
// four wavefronts per compute unit, i.e. ONE wavefront per SIMD (it serves larger outputs too: it turned out no
// slower per product than the 256 x 256 kernels).  A lone wavefront issues at most one instruction every
// four clocks, and the 8 matrix instructions of a step (16-bit inputs) occupy the matrix core for 256 clocks: a
// step stays at that pace only while it has well under 64 instructions.  Counters of the general implicit-GEMM
// path on a shape of 196 tiles show where its 0.34 us (820 clocks) per step go: the matrix cores are busy a fifth of the
// time, and more than half of all wavefront cycles are instruction issue -- the per-tap gather addresses, the LDS
// transfers with their M0 writes, 18 LDS operand reads, the counters.  Three properties of the problem remove
// most of that work:
//
//   * for unit-stride convolutions the pixels a tile of consecutive output pixels needs for ALL filter taps form
//     one short run of the NHWC input: output pixel n = (img, oy, ox) meets, for tap (r, s), the input pixel with
//     linear index lin0(n) + r*W + s, lin0(n) = (img*H + oy - pad_h)*W + ox - pad_w, and lin0 grows with n when
//     the output is no larger than the input.  Per chunk of channels (one 128-byte step of K) that run -- the
//     patch, at most 192 or 256 pixels x 128 bytes -- is put into LDS once per chunk, and every tap reads its B
//     fragments from it at a row offset of r*W + s.  Rows are 144 bytes apart, which keeps 16-byte reads of
//     consecutive rows on distinct banks without an address swizzle, so the 8 fragments of a step sit at
//     immediate offsets from one row address per output pixel; taps in the padding read a row of zeros;
//   * with the nine taps fixed at compile time the loop body is two chunks of nine steps, written out: the row
//     address of every (tap, pixel) is formed once per lane, buffers and register sets are constants, and no
//     position counter is left in the loop;
//   * the compressed A in its tiled layout is already in the lane order of the matrix instruction, so a
//     wavefront loads its A operands from memory into registers -- buffer loads with a lane offset formed once
//     and the step as a scalar offset -- two steps ahead, and A takes no part in the LDS traffic at all (the two
//     wavefronts that share rows of A read them twice from the L2 instead).
//
// The inner dimension is walked chunk by chunk, taps innermost: K step (tap, chunk) of A is column block
// tap*C + chunk*BK.  The patches alternate between two buffers.  A wavefront loads its share of patch c + 2
// into registers in step 6 of chunk c and writes it in the first step of chunk c + 1; the one barrier per
// chunk, before the B fragments of the next chunk's first step are read in the last step of a chunk, orders
// both the writes before the reads and the last reads of a buffer before its refill.  All memory waits are the
// compiler's own.
#pragma once
#include "mm_tiled.hpp"
#include <utility>

namespace sp24 {

constexpr int kPatchRowsSmall = 192, kPatchRowsLarge = 256;   // pixels a patch holds: two sizes of the kernel
constexpr int kPatchPitch = 144;                   // bytes from one patch row to the next in LDS

// f(integral_constant<int, I>) for every I of the sequence, in order: a loop whose index is a constant in its body
template <int... I, class F>
__device__ __forceinline__ void for_each_index(std::integer_sequence<int, I...>, F&& f)
{
    (f(std::integral_constant<int, I>{}), ...);
}

// The pixels a tile's patch may span if the patch kernel can take this convolution, else 0.  (The caller has checked
// what the tiled kernels need.)
inline int64_t conv_patch_span(const MmArgs& a)
{
    const ConvGeom& g = a.conv;
    if (!g.on || !a.sparse || a.layout != SP24_LAYOUT_TILED) return 0;
    if (g.R != 3 || g.S != 3 || g.stride_h != 1 || g.stride_w != 1 || g.OH > g.H || g.OW > g.W) return 0;
    // the compressed rows of one wavefront's two row blocks, as a buffer load's 32-bit offset
    if (a.K * 64 >= (int64_t)1 << 31) return 0;
    // rows a tile's patch spans at most: 128 consecutive output pixels, the extra input pixels at every change of
    // output row and image among them, and the reach of the filter
    const int64_t row_changes = 127 / g.OW + 1, img_changes = 127 / ((int64_t)g.OH * g.OW) + 1;
    const int64_t span = 128 + row_changes * (g.W - g.OW) + img_changes * (int64_t)(g.H - g.OH) * g.W + (int64_t)(g.R - 1) * g.W + g.S - 1;
    return span <= kPatchRowsLarge ? span : 0;
}

template <int DT, int OUT, int kPatchRows>
__global__ __launch_bounds__(256, kPatchRows <= kPatchRowsSmall ? 2 : 1) void k_conv_patch(MmArgs a, int tiles_m, int tiles_n)
{
    constexpr int ES = is8<DT> ? 1 : 2;
    constexpr int BK = kRowBytes / ES;                 // K elements (channels) per step
    constexpr int T64 = BK / 64;
    constexpr int WN = 2, TM = 2, TN = 2, BM = 128, BN = 128, RB = BM / 32;
    constexpr int NF = 2 * TN;                         // B fragments of a step: instruction j = f / TN, block nj = f % TN
    constexpr int XP = kPatchRows / 8 / 4;             // 1 KiB parts (8 pixels) of a patch per wavefront
    constexpr int kLoadsA = TM * (is8<DT> ? 4 : 3);    // loads of a step's A per wavefront: values twice, codes once (twice for 8-bit)
    constexpr int TAPS = 9, PF = 3;                    // PF: steps of A in registers, the one in use and two ahead; divides TAPS
    constexpr int kPitch = kPatchPitch;
    // LDS: two buffers, each the patch's rows and behind them a row of zeros: a row address is formed for buffer 0
    // and reaches buffer 1 by an immediate offset, whichever row it is.  55 KiB with the smaller patch, so that two
    // workgroups share a compute unit where the grid has them; 74 KiB with the larger
    constexpr int kPatchBytes = (kPatchRows + 1) * kPitch;
    constexpr int kZeroOff = kPatchRows * kPitch;
    constexpr int kLdsBytes = 2 * kPatchBytes;
    using acc_t = typename acc_of<DT>::type;
    static_assert(4 * epilogue_geometry<OUT, TN>::kWaveBytes <= kLdsBytes, "store scratch");
    static_assert(kPatchBytes + 96 + 16 <= 65536 && kLdsBytes <= 160 * 1024, "the second buffer and a fragment's place in a row as a 16-bit immediate");
    __shared__ __attribute__((aligned(1024))) uint8_t lds_all[kLdsBytes];

    int tm, tn;
    tile_of_workgroup(tiles_m, tiles_n, tm, tn);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int r = lane & 31, q = lane >> 5;
    const ConvGeom g = a.conv;
    const int nchunks = g.C / BK;
    const uint8_t* X = reinterpret_cast<const uint8_t*>(a.B);
    const int64_t pixel_bytes = (int64_t)g.C * ES;
    const int64_t n_pixels = (a.N / ((int64_t)g.OH * g.OW)) * g.H * g.W;      // input pixels in all images

    // linear index of the input pixel that tap (0, 0) meets for output pixel n (may lie before the image: padding)
    auto lin0_of = [&](int64_t n, int& iy, int& ix) -> int64_t {
        const int64_t t = n / g.OW;
        const int ox = (int)(n - t * g.OW);
        const int64_t img = t / g.OH;
        const int oy = (int)(t - img * g.OH);
        iy = oy - g.pad_h;
        ix = ox - g.pad_w;
        return (img * g.H + iy) * (int64_t)g.W + ix;
    };
    const int64_t n0 = (int64_t)tn * BN;
    int unused_y, unused_x;
    int64_t patch_first = lin0_of(n0, unused_y, unused_x);                     // wave-uniform
    if (patch_first < 0) patch_first = 0;

    // LDS address (in buffer 0) of this lane's row of B, 16-byte column q, for each tap and each of the lane's two
    // output pixels (one per 32-column block of the wavefront's tile); the row of zeros where the tap falls outside
    // the image or the pixel is past the last one (those columns are never stored)
    uint32_t b_row[TAPS][TN];
#pragma unroll
    for (int nj = 0; nj < TN; ++nj) {
        const int64_t n = n0 + wn * 32 * TN + nj * 32 + r;
        int iy0 = 0, ix0 = 0;
        const int prow = n < a.N ? (int)(lin0_of(n, iy0, ix0) - patch_first) : 0;
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            const int tr = t / 3, ts = t % 3;
            const bool in = n < a.N && (unsigned)(iy0 + tr) < (unsigned)g.H && (unsigned)(ix0 + ts) < (unsigned)g.W;
            b_row[t][nj] = (uint32_t)(in ? (prow + tr * g.W + ts) * kPitch : kZeroOff) + q * 16;
        }
    }
    struct BOps {
        int8v f[NF];
    };
    // B fragments out of buffer BUF for the row addresses of one tap
    auto read_b = [&](auto buf_c, const uint32_t (&row)[TN], BOps& o) {
        constexpr int BUF = decltype(buf_c)::value;
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            const int j = f / TN, nj = f % TN;
            // instruction j takes the 16-byte pieces at K-byte offsets (8-bit) 64j + 32h + 16q, (16-bit) 64h + 32j + 16q
            const int lo_off = is8<DT> ? 64 * j : 32 * j, hi_off = is8<DT> ? 64 * j + 32 : 64 + 32 * j;
            const uint8_t* base = lds_all + row[nj] + BUF * kPatchBytes;
            const uint4v lo = *reinterpret_cast<const uint4v*>(base + lo_off);
            const uint4v hi = *reinterpret_cast<const uint4v*>(base + hi_off);
            o.f[f][0] = lo[0]; o.f[f][1] = lo[1]; o.f[f][2] = lo[2]; o.f[f][3] = lo[3];
            o.f[f][4] = hi[0]; o.f[f][5] = hi[1]; o.f[f][6] = hi[2]; o.f[f][7] = hi[3];
        }
    };

    // ---- the patch: part x (0 .. XP-1) of this wavefront is patch rows (wave*XP + x)*8 .. +7; lane l carries
    // piece l % 8 of row l / 8.  Rows past the input fetch the last pixel (no tap inside the image reads them) ----
    const int64_t last_rel = n_pixels - 1 - patch_first;
    const uint8_t* patch_base = X + patch_first * pixel_bytes;                // wave-uniform
    uint32_t part_src[XP];
#pragma unroll
    for (int x = 0; x < XP; ++x) {
        const int prow_t = (wave * XP + x) * 8 + (lane >> 3);
        const int64_t rel = prow_t < last_rel ? prow_t : last_rel;
        part_src[x] = (uint32_t)(rel * pixel_bytes) + (lane & 7) * 16;
    }
    const uint32_t part_dst = (uint32_t)((wave * XP * 8 + (lane >> 3)) * kPitch + (lane & 7) * 16);
    struct Patch {
        uint4v part[XP];
    };
    auto load_patch = [&](int chunk, Patch& p) {
        const uint8_t* src = patch_base + (int64_t)chunk * kRowBytes;
#pragma unroll
        for (int x = 0; x < XP; ++x) p.part[x] = *reinterpret_cast<const uint4v*>(src + part_src[x]);
    };
    auto store_patch = [&](const Patch& p, int buf) {
#pragma unroll
        for (int x = 0; x < XP; ++x) *reinterpret_cast<uint4v*>(lds_all + buf * kPatchBytes + part_dst + x * 8 * kPitch) = p.part[x];
    };

    // ---- A: this wavefront's TM row blocks, straight from the tiled layout (a 32x64 tile's values are 1 KiB runs
    // in lane order, its codes a 256-byte run): buffer loads from the first row block's start, the lane's place as
    // the vector offset, the K step as the scalar offset ----
    struct AOps {
        int4v av[2][TM];
        int mv[2][TM];
    };
    const int64_t KB64 = a.K / 64, rb_total = a.M / 32;
    int64_t rb0 = (int64_t)tm * RB + wm * TM;
    if (rb0 >= rb_total) rb0 = rb_total - 1;            // ragged M: a valid row block, never stored
    const uint8_t* v_base = reinterpret_cast<const uint8_t*>(a.A) + rb0 * KB64 * (1024 * ES);
    const uint8_t* m_base = reinterpret_cast<const uint8_t*>(a.meta) + rb0 * KB64 * 256;
    const int rbs = rb0 + 1 < rb_total ? 2 : 1;         // row blocks from rb0 on that exist
    const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(wave_uniform(v_base)), 0, __builtin_amdgcn_readfirstlane((int)(rbs * KB64 * (1024 * ES))), 0x00020000);
    const __amdgpu_buffer_rsrc_t m_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(wave_uniform(m_base)), 0, __builtin_amdgcn_readfirstlane((int)(rbs * KB64 * 256)), 0x00020000);
    int v_off[TM], m_off[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int64_t di = i < rbs ? i : 0;
        v_off[i] = (int)(di * KB64 * (1024 * ES)) + lane * 16;
        m_off[i] = (int)(di * KB64 * 256) + lane * 4;
    }
    auto load_a = [&](int kstep, AOps& o) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                o.av[j][i] = __builtin_bit_cast(int4v, __builtin_amdgcn_raw_buffer_load_b128(v_rsrc, v_off[i] + j * 1024, kstep * 2048, 0));
                if (j == 0 || is8<DT>) o.mv[j][i] = __builtin_amdgcn_raw_buffer_load_b32(m_rsrc, m_off[i] + (is8<DT> ? j : 0) * 256, kstep * (T64 * 256), 0);
            }
    };

    acc_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = acc_t{};

    // ---- prologue: the row of zeros, the first patch, the second patch in flight, A of steps 0 and 1, B of step 0 ----
    if (tid < 2 * (kPitch / 4)) reinterpret_cast<uint32_t*>(lds_all + kZeroOff + (tid / (kPitch / 4)) * kPatchBytes)[tid % (kPitch / 4)] = 0u;
    Patch pp;
    load_patch(0, pp);
    store_patch(pp, 0);
    load_patch(nchunks > 1 ? 1 : 0, pp);
    AOps ao[PF];
#pragma unroll
    for (int u = 0; u < PF - 1; ++u) load_a(u * nchunks, ao[u]);              // steps (tap u, chunk 0)
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(63) & ~(15 << 8));                  // this wavefront's LDS writes are done (lgkmcnt 0)
    __builtin_amdgcn_s_barrier();
    BOps bo[2];
    read_b(std::integral_constant<int, 0>{}, b_row[0], bo[0]);
    __builtin_amdgcn_sched_barrier(0);

    // chunk c, PAR = c % 2: its patch is in buffer PAR; step t uses ring slot t % PF of A and register set
    // (9*PAR + t) % 2 of B
    auto do_chunk = [&](auto par_c, int c) {
        constexpr int PAR = decltype(par_c)::value;
        for_each_index(std::make_integer_sequence<int, TAPS>{}, [&](auto t_c) {
            constexpr int t = decltype(t_c)::value;
            if (t == 0) {
                // the patch of chunk c + 1 goes into the buffer chunk c - 1 used: everybody passed the barrier in that
                // chunk's last step, after its last reads
                store_patch(pp, PAR ^ 1);
            }
            if (t == 6) load_patch(c + 2 < nchunks ? c + 2 : nchunks - 1, pp);
            if (t == TAPS - 1) {
                // the next step's fragments come from the patch of chunk c + 1, written by all wavefronts in this
                // chunk's first step; and whoever passes here has finished the reads of this chunk's earlier steps
                __builtin_amdgcn_s_waitcnt(waitcnt_vm(63) & ~(15 << 8));
                __builtin_amdgcn_s_barrier();
            }
            __builtin_amdgcn_sched_barrier(0);
            {
                // A of the step two ahead, (tap, chunk) = (t + 2, c) or (t + 2 - 9, c + 1); past the last chunk that is
                // a step of the matrix all the same (tap 0 or 1 of "chunk nchunks" is K step nchunks or 2*nchunks), unused
                constexpr int t2 = (t + PF - 1) % TAPS;
                const int c2 = t + PF - 1 < TAPS ? c : c + 1;
                load_a(t2 * nchunks + c2, ao[(t + PF - 1) % PF]);
            }
            {
                constexpr int t1 = (t + 1) % TAPS;
                constexpr int buf1 = t + 1 < TAPS ? PAR : PAR ^ 1;
                read_b(std::integral_constant<int, buf1>{}, b_row[t1], bo[(9 * PAR + t + 1) & 1]);
            }
            const AOps& A = ao[t % PF];
            const BOps& B = bo[(9 * PAR + t) & 1];
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                const int j = f / TN, nj = f % TN;
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    if constexpr (is8<DT>) acc[i][nj] = smfmac32<DT, 0>(A.av[j][i], B.f[f], acc[i][nj], A.mv[j][i]);
                    else if (j == 0) acc[i][nj] = smfmac32<DT, 0>(A.av[0][i], B.f[f], acc[i][nj], A.mv[0][i]);
                    else acc[i][nj] = smfmac32<DT, 1>(A.av[1][i], B.f[f], acc[i][nj], A.mv[0][i]);
                }
            }
            // a wavefront issues in order, and a matrix instruction that finds the core busy holds up whatever follows
            // it: one LDS read and one load go into the shadow of each matrix instruction rather than ahead of all
#pragma unroll
            for (int k = 0; k < NF * TM; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);               // one matrix instruction
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);               // one LDS read
                if (k < kLoadsA) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // one load
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    int c = 0;
    for (; c + 2 <= nchunks; c += 2) {
        do_chunk(std::integral_constant<int, 0>{}, c);
        do_chunk(std::integral_constant<int, 1>{}, c + 1);
    }
    if (c < nchunks) do_chunk(std::integral_constant<int, 0>{}, c);

    // every wavefront is done with the patches: LDS becomes store scratch
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(63) & ~(15 << 8));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    store_wave_tile<DT, OUT, TM, TN>(a, acc, lds_all + wave * epilogue_geometry<OUT, TN>::kWaveBytes,
                                     (int64_t)tm * BM + wm * TM * 32, (int64_t)tn * BN + wn * TN * 32, lane);
}

template <int DT, int OUT>
static sp24_status run_conv_patch(const MmArgs& a, hipStream_t st)
{
    const int tiles_m = (int)((a.M + 127) / 128), tiles_n = (int)((a.N + 127) / 128);
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(256);
    if (conv_patch_span(a) <= kPatchRowsSmall) k_conv_patch<DT, OUT, kPatchRowsSmall><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
    else k_conv_patch<DT, OUT, kPatchRowsLarge><<<grid, block, 0, st>>>(a, tiles_m, tiles_n);
    return hipGetLastError() == hipSuccess ? SP24_OK : SP24_ERR_LAUNCH;
}

// The tiled kernel for a problem: the patch kernel for every sparse convolution it fits -- measured against the general
// kernels from 52 to 1568 tiles (7x7 to 56x56 images, 64 to 1024 output channels) it is 3 to 70 % faster throughout,
// most where M <= 128 leaves a 256-row tile half empty -- else the general choice.
template <int DT, int OUT>
static sp24_status pick_tile(const MmArgs& a, hipStream_t st)
{
    if (a.conv.on && conv_patch_span(a) > 0) return run_conv_patch<DT, OUT>(a, st);
    return pick_tile_general<DT, OUT>(a, st);
}

} // namespace sp24
