// Tiled emulation kernels: accumulation mode MMAEMU_C_AFTER_RD with the first / second half split, value mode 3 (binary32 values with E8M0 block scales;
// see emulate_tiled.hpp).
#include "emulate_tiled.hpp"

namespace mmaemu {
template MMAEMU_TILED_SIG(CM_RD_HALVES, 3);
} // namespace mmaemu
