// Tiled emulation kernels that run several models per launch, value mode 1 (see emulate_tiled.hpp).
#include "emulate_tiled.hpp"

namespace mmaemu {
template MMAEMU_MULTI_SIG(1);
} // namespace mmaemu
