// Tiled emulation kernels: accumulation mode MMAEMU_C_AFTER_RD, value mode 2 (see emulate_tiled.hpp).
#include "emulate_tiled.hpp"

namespace mmaemu {
template MMAEMU_TILED_SIG(MMAEMU_C_AFTER_RD, 2);
} // namespace mmaemu
