// Tiled product kernels instantiated for f16 inputs.
#include "mm_tiled.hpp"

namespace sp24 {

sp24_status tiled_f16(const MmArgs& a, hipStream_t st)
{
    if (a.out == SP24_F32) return pick_tile<SP24_F16, SP24_F32>(a, st);
    if (a.out == SP24_F16) return pick_tile<SP24_F16, SP24_F16>(a, st);
    return pick_tile<SP24_F16, SP24_BF16>(a, st);
}

} // namespace sp24
