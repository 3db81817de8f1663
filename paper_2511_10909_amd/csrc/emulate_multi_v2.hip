// Tiled emulation kernels that run several models per launch, value mode 2 (see emulate_tiled.hpp).
#include "emulate_tiled.hpp"

namespace mmaemu {
template MMAEMU_MULTI_SIG(2);
} // namespace mmaemu
