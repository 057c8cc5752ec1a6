// Tiled product kernels instantiated for f8 inputs and bf16 output (one translation unit per type
// pair so that they compile side by side).
#include "conv_patch.hpp"

namespace sp24 {

sp24_status tiled_f8_bf16(const MmArgs& a, hipStream_t st) { return pick_tile<SP24_F8, SP24_BF16>(a, st); }

} // namespace sp24
