// Tiled product kernels instantiated for i8 inputs and f16 output (one translation unit per type
// pair so that they compile side by side).
#include "conv_patch.hpp"

namespace sp24 {

sp24_status tiled_i8_f16(const MmArgs& a, hipStream_t st) { return pick_tile<SP24_I8, SP24_F16>(a, st); }

} // namespace sp24
