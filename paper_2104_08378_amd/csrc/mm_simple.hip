// General matrix-multiply kernel: one wavefront per 32x32 tile of D, operands
// gathered element by element with bounds checks.  It accepts every legal
// shape, both compressed layouts and both orders of B; the tiled kernels take
// over for the large aligned shapes.  Sparse (Sec. 3.2, Fig. 2: the metadata
// selects the rows of B that meet kept values of A) and dense variants share
// the operand gather and the store.
#include "common.hpp"
#include "launch.hpp"
#include "mfma.hpp"

#include <type_traits>

namespace sp24 {

template <int ES>
__device__ __forceinline__ uint32_t load_elem(const void* p, int64_t idx)
{
    if constexpr (ES == 2) return reinterpret_cast<const uint16_t*>(p)[idx];
    else return reinterpret_cast<const uint8_t*>(p)[idx];
}

// Gather COUNT consecutive-k elements starting at (k0) of row/column `fixed`
// into packed dwords.  stride_k / stride_f give the element strides.
template <int ES, int COUNT>
__device__ __forceinline__ void gather(const void* p, int64_t k0, int64_t kmax, bool fixed_ok, int64_t base_f, int64_t stride_k,
                                       int* dst)
{
    constexpr int PER = 4 / ES;
#pragma unroll
    for (int d = 0; d < COUNT / PER; ++d) {
        uint32_t w = 0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            int64_t k = k0 + d * PER + j;
            uint32_t x = (fixed_ok && k < kmax) ? load_elem<ES>(p, base_f + k * stride_k) : 0u;
            w |= x << (8 * ES * j);
        }
        dst[d] = (int)w;
    }
}

// Output pixel of a convolution column n: image and the input coordinates of filter tap (0, 0).
struct ConvPixel {
    int64_t img;
    int iy0, ix0;
};

// The same gather for a convolution read as an implicit GEMM: COUNT consecutive k (16 bytes, starting at a
// multiple of 16 bytes) lie inside one filter tap because C * element size is a multiple of 16 bytes.
template <int ES, int COUNT>
__device__ __forceinline__ void gather_conv(const MmArgs& a, int64_t k0, int64_t kmax, bool n_ok, const ConvPixel& px, int* dst)
{
    const ConvGeom& g = a.conv;
    const int64_t tap = k0 / g.C;
    const int c = (int)(k0 - tap * g.C);
    const int r = (int)(tap / g.S), s = (int)(tap - (int64_t)r * g.S);
    const int iy = px.iy0 + r, ix = px.ix0 + s;
    const bool ok = n_ok && k0 < kmax && (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
    const int64_t base = ((px.img * g.H + iy) * g.W + ix) * g.C + c;
    gather<ES, COUNT>(a.B, 0, COUNT, ok, base, 1, dst);
}

template <int DT, int OUT, bool SPARSE>
__global__ __launch_bounds__(64) void k_mm_simple(MmArgs a)
{
    constexpr int ES = is8<DT> ? 1 : 2;
    using acc_t = typename acc_of<DT>::type;
    const int lane = threadIdx.x, r = lane & 31, q = lane >> 5;
    const int64_t row0 = (int64_t)blockIdx.y * 32, col0 = (int64_t)blockIdx.x * 32;
    const int64_t m = row0 + r, n = col0 + r;
    const bool m_ok = m < a.M, n_ok = n < a.N;
    const int64_t K = a.K;
    // element (k, n) of B
    const int64_t b_stride_k = (a.bo == SP24_B_KMAJOR) ? 1 : a.ldb;
    const int64_t b_base = (a.bo == SP24_B_KMAJOR) ? n * a.ldb : n;
    ConvPixel px = {0, 0, 0};
    if (a.conv.on && n_ok) {
        const int64_t t = n / a.conv.OW;
        px.img = t / a.conv.OH;
        px.iy0 = (int)(t - px.img * a.conv.OH) * a.conv.stride_h - a.conv.pad_h;
        px.ix0 = (int)(n - t * a.conv.OW) * a.conv.stride_w - a.conv.pad_w;
    }
    // COUNT values of column n of B starting at row k0, packed into dwords
    auto load_b = [&](auto es_tag, auto count_tag, int64_t k0, int* dst) {
        constexpr int E = decltype(es_tag)::value, CNT = decltype(count_tag)::value;
        if (a.conv.on) gather_conv<E, CNT>(a, k0, K, n_ok, px, dst);
        else gather<E, CNT>(a.B, k0, K, n_ok, b_base, b_stride_k, dst);
    };
    using i1 = std::integral_constant<int, 1>;
    using i2 = std::integral_constant<int, 2>;
    using i8c = std::integral_constant<int, 8>;
    using i16c = std::integral_constant<int, 16>;
    acc_t acc = {};
    const int64_t KB = (K + 63) / 64;
    for (int64_t kb = 0; kb < KB; ++kb) {
        if constexpr (SPARSE) {
            uint32_t codes = 0;
            const int64_t K2 = K / 2;
            if (a.layout == SP24_LAYOUT_TILED) {
                codes = reinterpret_cast<const uint32_t*>(a.meta)[(((int64_t)blockIdx.y) * (K / 64) + kb) * 64 + lane];
            } else {
                const uint8_t* mrow = reinterpret_cast<const uint8_t*>(a.meta) + m * (K / 8);
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    int64_t byte = kb * 8 + 4 * q + b;
                    if (m_ok && byte < K / 8) codes |= (uint32_t)mrow[byte] << (8 * b);
                }
            }
            if constexpr (is8<DT>) {
                int4v av;
                int8v bv;
                int tmp[8];
                if (a.layout == SP24_LAYOUT_TILED)
                    av = reinterpret_cast<const int4v*>(a.A)[(((int64_t)blockIdx.y) * (K / 64) + kb) * 64 + lane];
                else {
                    gather<1, 16>(a.A, kb * 32 + 16 * q, K2, m_ok, m * K2, 1, tmp);
                    for (int i = 0; i < 4; ++i) av[i] = tmp[i];
                }
                load_b(i1{}, i16c{}, kb * 64 + 16 * q, tmp);
                load_b(i1{}, i16c{}, kb * 64 + 32 + 16 * q, tmp + 4);
                for (int i = 0; i < 8; ++i) bv[i] = tmp[i];
                acc = smfmac32<DT, 0>(av, bv, acc, (int)codes);
            } else {
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    int4v av;
                    int8v bv;
                    int tmp[8];
                    if (a.layout == SP24_LAYOUT_TILED)
                        av = reinterpret_cast<const int4v*>(a.A)[((((int64_t)blockIdx.y) * (K / 64) + kb) * 2 + s) * 64 + lane];
                    else {
                        gather<2, 8>(a.A, kb * 32 + 16 * q + 8 * s, K2, m_ok, m * K2, 1, tmp);
                        for (int i = 0; i < 4; ++i) av[i] = tmp[i];
                    }
                    load_b(i2{}, i8c{}, kb * 64 + 16 * s + 8 * q, tmp);
                    load_b(i2{}, i8c{}, kb * 64 + 32 + 16 * s + 8 * q, tmp + 4);
                    for (int i = 0; i < 8; ++i) bv[i] = tmp[i];
                    if (s == 0) acc = smfmac32<DT, 0>(av, bv, acc, (int)codes);
                    else acc = smfmac32<DT, 1>(av, bv, acc, (int)codes);
                }
            }
        } else {
            constexpr int PERK = is8<DT> ? 32 : 16; // k per dense instruction (the 8-bit float form takes its 16 bytes as two)
#pragma unroll
            for (int j = 0; j < 64 / PERK; ++j) {
                int4v av, bv;
                int ta[4], tb[4];
                int64_t k0 = kb * 64 + j * PERK + (PERK / 2) * q;
                gather<ES, PERK / 2>(a.A, k0, K, m_ok, m * a.lda, 1, ta);
                load_b(std::integral_constant<int, ES>{}, std::integral_constant<int, PERK / 2>{}, k0, tb);
                for (int i = 0; i < 4; ++i) { av[i] = ta[i]; bv[i] = tb[i]; }
                acc = mfma32<DT>(av, bv, acc);
            }
        }
    }
    store_tile<DT, OUT>(a.D, a.ldd, row0, col0, a.M, a.N, acc, lane, a.epi);
}

template <int DT, int OUT>
static sp24_status launch_t(const MmArgs& a, hipStream_t st)
{
    dim3 grid((unsigned)((a.N + 31) / 32), (unsigned)((a.M + 31) / 32));
    if (a.sparse) k_mm_simple<DT, OUT, true><<<grid, 64, 0, st>>>(a);
    else k_mm_simple<DT, OUT, false><<<grid, 64, 0, st>>>(a);
    return hipGetLastError() == hipSuccess ? SP24_OK : SP24_ERR_LAUNCH;
}

sp24_status launch_mm_simple(const MmArgs& a, hipStream_t st)
{
    if (a.M == 0 || a.N == 0) return SP24_OK;
    if ((a.M + 31) / 32 > 65535) return SP24_ERR_SHAPE;
    if (a.in == SP24_I8) {
        if (a.out == SP24_I32) return launch_t<SP24_I8, SP24_I32>(a, st);
        if (a.out == SP24_I8) return launch_t<SP24_I8, SP24_I8>(a, st);
        if (a.out == SP24_F32) return launch_t<SP24_I8, SP24_F32>(a, st);
        if (a.out == SP24_F16) return launch_t<SP24_I8, SP24_F16>(a, st);
        return launch_t<SP24_I8, SP24_BF16>(a, st);
    }
    if (a.in == SP24_F8) {
        if (a.out == SP24_F32) return launch_t<SP24_F8, SP24_F32>(a, st);
        if (a.out == SP24_F16) return launch_t<SP24_F8, SP24_F16>(a, st);
        return launch_t<SP24_F8, SP24_BF16>(a, st);
    }
    if (a.in == SP24_F16) {
        if (a.out == SP24_F32) return launch_t<SP24_F16, SP24_F32>(a, st);
        if (a.out == SP24_F16) return launch_t<SP24_F16, SP24_F16>(a, st);
        return launch_t<SP24_F16, SP24_BF16>(a, st);
    }
    if (a.out == SP24_F32) return launch_t<SP24_BF16, SP24_F32>(a, st);
    if (a.out == SP24_F16) return launch_t<SP24_BF16, SP24_F16>(a, st);
    return launch_t<SP24_BF16, SP24_BF16>(a, st);
}

} // namespace sp24
