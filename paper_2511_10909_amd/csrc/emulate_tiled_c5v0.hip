// Tiled emulation kernels: accumulation mode MMAEMU_C_AFTER_RD with the split into quarters, value mode 0
// (see emulate_tiled.hpp).
#include "emulate_tiled.hpp"

namespace mmaemu {
template MMAEMU_TILED_SIG(CM_RD_QUARTERS, 0);
} // namespace mmaemu
