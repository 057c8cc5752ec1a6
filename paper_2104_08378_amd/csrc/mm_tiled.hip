// Tiled matrix-multiply kernels for large aligned shapes (placeholder: nothing handled yet).
#include "common.hpp"
#include "launch.hpp"
#include "mfma.hpp"

namespace sp24 {

sp24_status launch_mm_tiled(const MmArgs&, hipStream_t, bool* handled)
{
    *handled = false;
    return SP24_OK;
}

} // namespace sp24
