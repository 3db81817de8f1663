// Tiled emulation kernels that run several models per launch, value mode 0 (see emulate_tiled.hpp).
#include "emulate_tiled.hpp"

namespace mmaemu {
template MMAEMU_MULTI_SIG(0);
} // namespace mmaemu
