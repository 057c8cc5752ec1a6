// Shared device-side helpers of libsp24 (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "../../include/sp24.h"

namespace sp24 {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef int int4v __attribute__((ext_vector_type(4)));
typedef int int8v __attribute__((ext_vector_type(8)));
typedef int int16v __attribute__((ext_vector_type(16)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));

__host__ __device__ inline int esize_of(sp24_dtype t)
{
    return (t == SP24_I8 || t == SP24_F8) ? 1 : (t == SP24_F16 || t == SP24_BF16) ? 2 : 4;
}

// one-byte input types: they share every data path (64 columns of A per 32x32 sparse instruction, 32 bytes of
// compressed values per row and 64 columns); they differ in the magnitude that pruning compares and in the
// matrix-core instruction (integer or float accumulation)
template <int DT> constexpr bool is8 = (DT == SP24_I8 || DT == SP24_F8);

// ---------------------------------------------------------------------------
// Selection rule (Sec. 4.1 Step 2: drop the two smallest magnitudes of four).
// Magnitudes are compared through an unsigned key: for 16-bit floats the bit
// pattern without its sign, with every NaN clamped to one key just above
// infinity; for int8 the absolute value in a wider type (|-128| = 128).
// Equal keys: the lower column wins.
// ---------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ uint32_t mag_key16(uint32_t bits)
{
    constexpr uint32_t inf = (DT == SP24_F16) ? 0x7C00u : 0x7F80u;
    uint32_t a = bits & 0x7FFFu;
    return a > inf ? inf + 1u : a;
}

__device__ __forceinline__ uint32_t mag_key8(uint32_t byte)
{
    int v = (int)(int8_t)byte;
    return (uint32_t)(v < 0 ? -v : v);
}

// 8-bit float (4 exponent bits, bias 7, 3 fraction bits, no infinities): the bit pattern without its sign orders
// the magnitudes, and the one NaN pattern (0x7F) is the largest key by itself
__device__ __forceinline__ uint32_t mag_key_f8(uint32_t byte) { return byte & 0x7Fu; }

// its magnitude as a number (NaN counts as +infinity, as for the other float types where sums of magnitudes are formed)
__device__ __forceinline__ float magnitude_f8(uint32_t byte)
{
    const uint32_t a = byte & 0x7Fu, e = a >> 3, f = a & 7u;
    if (a == 0x7Fu) return __builtin_inff();
    if (e == 0u) return (float)f * 0.001953125f;                       // subnormal: f * 2^-9
    return __uint_as_float(((e + 120u) << 23) | (f << 20));             // 2^(e - 7) * (1 + f / 8)
}

// Returns the 4-bit keep mask (bit i set = column i survives); exactly two bits set.
__device__ __forceinline__ uint32_t keep_mask(uint32_t k0, uint32_t k1, uint32_t k2, uint32_t k3)
{
    // c_ab = 1 when column a outranks column b (a < b, so a also wins ties)
    uint32_t c01 = k0 >= k1, c02 = k0 >= k2, c03 = k0 >= k3;
    uint32_t c12 = k1 >= k2, c13 = k1 >= k3, c23 = k2 >= k3;
    uint32_t ahead0 = 3u - c01 - c02 - c03;
    uint32_t ahead1 = c01 + 2u - c12 - c13;
    uint32_t ahead2 = c02 + c12 + 1u - c23;
    uint32_t ahead3 = c03 + c13 + c23;
    return (ahead0 < 2u) | ((ahead1 < 2u) << 1) | ((ahead2 < 2u) << 2) | ((ahead3 < 2u) << 3);
}

// Metadata code pos0 | pos1 << 2 for a keep mask with two bits set (Sec. 3.1:
// 2 bits per kept value, positions in ascending order).
__device__ __forceinline__ uint32_t code_of_mask(uint32_t mask)
{
    // nibble table indexed by mask: 0011->0x4 0101->0x8 0110->0x9 1001->0xC 1010->0xD 1100->0xE
    constexpr uint64_t table = (0x4ull << (4 * 0x3)) | (0x8ull << (4 * 0x5)) | (0x9ull << (4 * 0x6)) |
                               (0xCull << (4 * 0x9)) | (0xDull << (4 * 0xA)) | (0xEull << (4 * 0xC));
    return (uint32_t)(table >> (4 * mask)) & 0xFu;
}

// ---------------------------------------------------------------------------
// fp32 -> 16-bit storage, round to nearest even.
// ---------------------------------------------------------------------------
// float -> 16-bit output, round to nearest even, as the hardware converts (v_cvt_pk_bf16_f32 / v_cvt_f16_f32:
// one instruction, no branch on NaN)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    __bf16 h = (__bf16)f;
    return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ uint16_t f32_to_f16_bits(float f)
{
    _Float16 h = (_Float16)f;
    return __builtin_bit_cast(uint16_t, h);
}

// two floats -> two 16-bit outputs in one register (lo in bits 0-15), one packed conversion
template <int OUT>
__device__ __forceinline__ uint32_t pack_out16(float lo, float hi)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    if constexpr (OUT == SP24_BF16) {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    } else {
        typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
    }
}

// ---------------------------------------------------------------------------
// Epilogue of the quantised path (int8 inputs; Sec. 5: one scaling factor per
// row of the weight matrix -- per output channel -- and one per activation
// tensor).  For accumulator acc of row m:
//     s = w_scale[m] * x_scale;  y = fma(float(acc), s, bias[m]);  y = max(y, 0) if relu
// written as F32 / F16 / BF16 (one rounding), or re-quantised with a
// per-tensor output scale: q = clamp(rint(y * inv_y_scale), -128, 127), every
// step one binary32 operation (the rounding decision is defined in binary32).
// ---------------------------------------------------------------------------
struct Epilogue {
    const float* w_scale;   // device, M values
    const float* bias;      // device, M values, or null
    float x_scale;
    float inv_y_scale;      // used when the output type is SP24_I8
    int relu;
    int on;                 // 0: plain int32 / float output
};

// scale and bias of row m (m clamped by the caller to a valid row)
__device__ __forceinline__ void epilogue_row(const Epilogue& e, int64_t m, float& s, float& b)
{
    s = e.w_scale[m] * e.x_scale;
    b = e.bias ? e.bias[m] : 0.0f;
}

__device__ __forceinline__ float dequant_value(int acc, float s, float b, int relu)
{
    const float y = __builtin_fmaf((float)acc, s, b);
    return relu ? fmaxf(y, 0.0f) : y;
}

__device__ __forceinline__ int quantise_i8(float y, float inv_y_scale)
{
    float r = __builtin_rintf(y * inv_y_scale);         // v_rndne_f32: ties to even
    r = fminf(fmaxf(r, -128.0f), 127.0f);
    return (int)r;
}

// Bits of one output element (in the low bytes of the result) for an accumulator value: the integer itself,
// the float converted to the output type, or the quantised epilogue's result.  ACC is int (int8 inputs) or float.
template <int OUT, typename ACC>
__device__ __forceinline__ uint32_t output_bits(ACC acc, float s, float b, const Epilogue& e)
{
    if constexpr (std::is_same<ACC, int>::value) {
        if constexpr (OUT == SP24_I32) return (uint32_t)acc;
        else {
            const float y = dequant_value(acc, s, b, e.relu);
            if constexpr (OUT == SP24_I8) return (uint32_t)quantise_i8(y, e.inv_y_scale) & 0xFFu;
            else if constexpr (OUT == SP24_F32) return __float_as_uint(y);
            else if constexpr (OUT == SP24_F16) return f32_to_f16_bits(y);
            else return f32_to_bf16_bits(y);
        }
    } else {
        if constexpr (OUT == SP24_F32) return __float_as_uint(acc);
        else if constexpr (OUT == SP24_F16) return f32_to_f16_bits(acc);
        else return f32_to_bf16_bits(acc);
    }
}

template <int OUT>
constexpr int out_size() { return (OUT == SP24_F32 || OUT == SP24_I32) ? 4 : (OUT == SP24_I8) ? 1 : 2; }

// store the low out_size<OUT>() bytes of `bits` at element idx of D
template <int OUT>
__device__ __forceinline__ void store_bits(void* D, int64_t idx, uint32_t bits)
{
    if constexpr (out_size<OUT>() == 4) reinterpret_cast<uint32_t*>(D)[idx] = bits;
    else if constexpr (out_size<OUT>() == 2) reinterpret_cast<uint16_t*>(D)[idx] = (uint16_t)bits;
    else reinterpret_cast<uint8_t*>(D)[idx] = (uint8_t)bits;
}

template <int OUT>
__device__ __forceinline__ void store_out(void* D, int64_t idx, float v)
{
    if constexpr (OUT == SP24_F32) reinterpret_cast<float*>(D)[idx] = v;
    else if constexpr (OUT == SP24_F16) reinterpret_cast<uint16_t*>(D)[idx] = f32_to_f16_bits(v);
    else reinterpret_cast<uint16_t*>(D)[idx] = f32_to_bf16_bits(v);
}

} // namespace sp24
