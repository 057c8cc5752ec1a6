// Tiled product kernels: which problems they take, and the per-type entry points.  The kernels themselves are
// templates in mm_tiled.hpp; each pair of input and output type is instantiated in a
// translation unit of its own (mm_tiled_<in>_<out>.hip) so that they compile side by side.
#include "common.hpp"
#include "launch.hpp"

namespace sp24 {

sp24_status tiled_f16_f32(const MmArgs& a, hipStream_t st);
sp24_status tiled_f16_f16(const MmArgs& a, hipStream_t st);
sp24_status tiled_f16_bf16(const MmArgs& a, hipStream_t st);
sp24_status tiled_bf16_f32(const MmArgs& a, hipStream_t st);
sp24_status tiled_bf16_f16(const MmArgs& a, hipStream_t st);
sp24_status tiled_bf16_bf16(const MmArgs& a, hipStream_t st);
sp24_status tiled_i8_i32(const MmArgs& a, hipStream_t st);
sp24_status tiled_i8_i8(const MmArgs& a, hipStream_t st);
sp24_status tiled_i8_f32(const MmArgs& a, hipStream_t st);
sp24_status tiled_i8_f16(const MmArgs& a, hipStream_t st);
sp24_status tiled_i8_bf16(const MmArgs& a, hipStream_t st);
sp24_status tiled_f8_f32(const MmArgs& a, hipStream_t st);
sp24_status tiled_f8_f16(const MmArgs& a, hipStream_t st);
sp24_status tiled_f8_bf16(const MmArgs& a, hipStream_t st);

constexpr int kStepBytes = 128;   // bytes of one operand row consumed per step (kRowBytes of the kernels)

sp24_status launch_mm_tiled(const MmArgs& a, hipStream_t st, bool* handled)
{
    *handled = false;
    const int es = esize_of(a.in);
    // K: whole 32-byte runs (a last, partial step is filled up with zeros)
    bool ok = a.bo == SP24_B_KMAJOR && (a.K * es) % 32 == 0 && (reinterpret_cast<uintptr_t>(a.B) & 15u) == 0 &&
              (a.ldb * es) % 16 == 0 && a.N >= 1 && a.M >= 1 && a.M <= ((int64_t)1 << 30) && a.N <= ((int64_t)1 << 30) &&
              a.ldb * es < ((int64_t)1 << 22) && ((a.M + 127) / 128) * ((a.N + 127) / 128) < ((int64_t)1 << 30);
    if (!a.conv.on && a.bo == SP24_B_NMAJOR) {
        // N-major B: whole 16-byte chunks of columns, rows 16-byte aligned, 32-bit row offsets within a step
        ok = (a.K * es) % 32 == 0 && (reinterpret_cast<uintptr_t>(a.B) & 15u) == 0 && (a.ldb * es) % 16 == 0 &&
             (a.N * es) % 16 == 0 && a.N >= 1 && a.M >= 1 && a.M <= ((int64_t)1 << 30) && a.N <= ((int64_t)1 << 30) &&
             a.ldb * es < ((int64_t)1 << 22) && ((a.M + 127) / 128) * ((a.N + 127) / 128) < ((int64_t)1 << 30);
    }
    if (a.conv.on) {
        // implicit GEMM: a step must lie inside one filter tap, and byte offsets into the input must fit 31 bits
        // (N / (OH*OW) images of H*W*C elements, plus the virtual pixels of the padding)
        const ConvGeom& g = a.conv;
        const int64_t n_img = a.N / ((int64_t)g.OH * g.OW);
        const int64_t span = ((n_img * g.H + g.pad_h + g.R) * (int64_t)g.W + g.pad_w + g.S) * g.C * es;
        ok = (reinterpret_cast<uintptr_t>(a.B) & 15u) == 0 && a.N >= 32 && a.M >= 1 && a.M <= ((int64_t)1 << 30) &&
             ((int64_t)g.C * es) % kStepBytes == 0 && span < ((int64_t)1 << 31) &&
             ((a.M + 127) / 128) * ((a.N + 127) / 128) < ((int64_t)1 << 30);
    }
    // compressed operand: the tiled layout, or the canonical one gathered row by row (32-bit offsets inside a tile)
    // (canonical codes are fetched as 4-byte words = 32 columns)
    if (a.sparse && a.layout == SP24_LAYOUT_CANONICAL) ok = ok && a.K % 32 == 0 && (a.K / 2 * es) * 256 < ((int64_t)1 << 31);
    else ok = ok && a.lda * es < ((int64_t)1 << 22);
    if (!ok) return SP24_OK;
    *handled = true;
    if (a.in == SP24_I8) {
        if (a.out == SP24_I32) return tiled_i8_i32(a, st);
        if (a.out == SP24_I8) return tiled_i8_i8(a, st);
        if (a.out == SP24_F32) return tiled_i8_f32(a, st);
        if (a.out == SP24_F16) return tiled_i8_f16(a, st);
        return tiled_i8_bf16(a, st);
    }
    if (a.in == SP24_F8) {
        if (a.out == SP24_F32) return tiled_f8_f32(a, st);
        if (a.out == SP24_F16) return tiled_f8_f16(a, st);
        return tiled_f8_bf16(a, st);
    }
    if (a.in == SP24_F16) {
        if (a.out == SP24_F32) return tiled_f16_f32(a, st);
        if (a.out == SP24_F16) return tiled_f16_f16(a, st);
        return tiled_f16_bf16(a, st);
    }
    if (a.out == SP24_F32) return tiled_bf16_f32(a, st);
    if (a.out == SP24_F16) return tiled_bf16_f16(a, st);
    return tiled_bf16_bf16(a, st);
}

} // namespace sp24
