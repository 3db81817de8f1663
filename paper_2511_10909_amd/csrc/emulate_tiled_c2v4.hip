// Tiled emulation kernels: accumulation mode MMAEMU_C_AFTER_RD, value mode 4 (TF32 operands; see emulate_tiled.hpp).
#include "emulate_tiled.hpp"

namespace mmaemu {
template MMAEMU_TILED_SIG(MMAEMU_C_AFTER_RD, 4);
} // namespace mmaemu
