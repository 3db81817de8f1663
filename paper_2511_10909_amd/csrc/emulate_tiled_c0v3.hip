// Tiled emulation kernels: accumulation mode MMAEMU_C_IN_GROUP, value mode 3 (binary32 values with E8M0 block scales;
// see emulate_tiled.hpp).
#include "emulate_tiled.hpp"

namespace mmaemu {
template MMAEMU_TILED_SIG(MMAEMU_C_IN_GROUP, 3);
} // namespace mmaemu
