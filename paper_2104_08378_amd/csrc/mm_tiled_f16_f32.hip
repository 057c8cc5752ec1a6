// Tiled product kernels instantiated for f16 inputs and f32 output (one translation unit per type
// pair so that they compile side by side).
#include "conv_patch.hpp"

namespace sp24 {

sp24_status tiled_f16_f32(const MmArgs& a, hipStream_t st) { return pick_tile<SP24_F16, SP24_F32>(a, st); }

} // namespace sp24
