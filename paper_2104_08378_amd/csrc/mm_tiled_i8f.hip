// Tiled product kernels instantiated for int8 inputs with the quantised path's floating-point outputs.
#include "mm_tiled.hpp"

namespace sp24 {

sp24_status tiled_i8_scaled(const MmArgs& a, hipStream_t st)
{
    if (a.out == SP24_F32) return pick_tile<SP24_I8, SP24_F32>(a, st);
    if (a.out == SP24_F16) return pick_tile<SP24_I8, SP24_F16>(a, st);
    return pick_tile<SP24_I8, SP24_BF16>(a, st);
}

} // namespace sp24
