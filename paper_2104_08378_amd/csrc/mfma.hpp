// Thin typed wrappers over the gfx950 32x32 matrix-core instructions.
//
// Register layouts (64 lanes; r = lane % 32, q = lane / 32), as measured on
// the device for the sparse forms and as documented for the dense ones:
//
//   D / C (all forms): 16 values per lane; value i is row 8*(i/4) + 4*q + i%4,
//       column r of the 32x32 tile.
//
//   dense  v_mfma_f32_32x32x16_{f16,bf16}: A and B hold 8 values per lane,
//       k = 8*q + e.     v_mfma_i32_32x32x32_i8: 16 values, k = 16*q + e.
//
//   sparse v_smfmac_f32_32x32x32_{f16,bf16} (A is 32 x 32, stored 32 x 16):
//       A: 8 compressed values per lane = 4 groups: group 4*q + e/2, i.e.
//          columns 16*q .. 16*q+15 of the instruction's 32 columns of A;
//       idx: 4 codes x 4 bits (pos0 | pos1<<2), code p for values 2p, 2p+1,
//          taken from bits 0..15 (abid = 0) or 16..31 (abid = 1) of the lane;
//       B: 16 values per lane: value e is row k = 16*(e/8) + 8*q + e%8.
//   sparse v_smfmac_i32_32x32x64_i8 and v_smfmac_f32_32x32x64_fp8_fp8 (A is 32 x 64, stored 32 x 32):
//       A: 16 compressed values per lane = 8 groups: columns 32*q .. 32*q+31;
//       idx: 8 codes in all 32 bits of the lane;
//       B: 32 values per lane: value e is row k = 32*(e/16) + 16*q + e%16.
//
// The sparse forms implement the selection step of Fig. 2: the codes pick,
// for each kept value of A, the matching row of B inside its group of four.
#pragma once
#include "common.hpp"

namespace sp24 {

template <int DT> struct acc_of { using type = float16v; };
template <> struct acc_of<SP24_I8> { using type = int16v; };

// A operand: 4 dwords, B operand: 8 dwords (sparse) / 4 dwords (dense), raw bits.
template <int DT, int ABID>
__device__ __forceinline__ typename acc_of<DT>::type smfmac32(const int4v& a, const int8v& b, typename acc_of<DT>::type c, int idx)
{
    if constexpr (DT == SP24_F16)
        return __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half16, b), c, idx, 0, ABID);
    else if constexpr (DT == SP24_BF16)
        return __builtin_amdgcn_smfmac_f32_32x32x32_bf16(__builtin_bit_cast(bf8, a), __builtin_bit_cast(bf16x16, b), c, idx, 0, ABID);
    else if constexpr (DT == SP24_F8)
        return __builtin_amdgcn_smfmac_f32_32x32x64_fp8_fp8(a, b, c, idx, 0, ABID);
    else
        return __builtin_amdgcn_smfmac_i32_32x32x64_i8(a, b, c, idx, 0, ABID);
}

template <int DT>
__device__ __forceinline__ typename acc_of<DT>::type mfma32(const int4v& a, const int4v& b, typename acc_of<DT>::type c)
{
    if constexpr (DT == SP24_F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
    else if constexpr (DT == SP24_BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf8, a), __builtin_bit_cast(bf8, b), c, 0, 0, 0);
    else if constexpr (DT == SP24_F8) {
        // the 16 bytes per lane are two operands of the 8-byte form; which 8 values of K a lane holds does not
        // matter as long as A and B pair up the same bytes
        typedef long long2v __attribute__((ext_vector_type(2)));
        const long2v a2 = __builtin_bit_cast(long2v, a), b2 = __builtin_bit_cast(long2v, b);
        c = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a2[0], b2[0], c, 0, 0, 0);
        return __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a2[1], b2[1], c, 0, 0, 0);
    } else
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
}

// Store one 32x32 accumulator tile, predicated on the matrix edge; int8 inputs with a scaled output type go
// through the quantised path's epilogue.
template <int DT, int OUT>
__device__ __forceinline__ void store_tile(void* D, int64_t ldd, int64_t row0, int64_t col0, int64_t M, int64_t N,
                                           const typename acc_of<DT>::type& c, int lane, const Epilogue& epi)
{
    int r = lane & 31, q = lane >> 5;
    int64_t col = col0 + r;
    if (col >= N) return;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        int64_t row = row0 + 8 * (i / 4) + 4 * q + (i % 4);
        if (row < M) {
            float s = 0.0f, b = 0.0f;
            if constexpr (DT == SP24_I8 && OUT != SP24_I32) epilogue_row(epi, row, s, b);
            auto v = c[i];
            store_bits<OUT>(D, row * ldd + col, output_bits<OUT>(v, s, b, epi));
        }
    }
}

} // namespace sp24
