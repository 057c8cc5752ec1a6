// Tiled product kernels instantiated for int8 inputs with integer outputs: the plain int32 result and the
// quantised path's int8 output.
#include "mm_tiled.hpp"

namespace sp24 {

sp24_status tiled_i8_scaled(const MmArgs& a, hipStream_t st);

sp24_status tiled_i8(const MmArgs& a, hipStream_t st)
{
    if (a.out == SP24_I32) return pick_tile<SP24_I8, SP24_I32>(a, st);
    if (a.out == SP24_I8) return pick_tile<SP24_I8, SP24_I8>(a, st);
    return tiled_i8_scaled(a, st);
}

} // namespace sp24
