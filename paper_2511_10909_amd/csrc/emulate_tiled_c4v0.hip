// Tiled emulation kernels: accumulation mode MMAEMU_C_AFTER_RD with the first / second half split, value mode 0
// (see emulate_tiled.hpp).
#include "emulate_tiled.hpp"

namespace mmaemu {
template MMAEMU_TILED_SIG(CM_RD_HALVES, 0);
} // namespace mmaemu
