// Tiled product kernels instantiated for int8 inputs.
#include "mm_tiled.hpp"

namespace sp24 {

sp24_status tiled_i8(const MmArgs& a, hipStream_t st)
{
    return pick_tile<SP24_I8, SP24_I32>(a, st);
}

} // namespace sp24
