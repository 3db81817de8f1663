// Tiled emulation kernels, accumulation mode MMAEMU_C_IN_GROUP (see emulate_tiled.hpp).
#include "emulate_tiled.hpp"

namespace mmaemu {
template mmaemu_status launch_tiled_shape<MMAEMU_C_IN_GROUP>(const TiledArgs &, const void *, const void *, const void *, void *, uint32_t,
                                              uint32_t, uint32_t, uint64_t, hipStream_t, bool &);
} // namespace mmaemu
