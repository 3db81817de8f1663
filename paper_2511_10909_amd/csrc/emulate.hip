// Dispatch of the emulation entry point to a kernel family.
#include "common.hpp"

namespace mmaemu {

mmaemu_status launch_emulate(const ModelArgs &p, const void *A, const void *B, const void *C, void *D,
                             uint32_t m, uint32_t n, uint32_t k, uint64_t batch, uint32_t ta, uint32_t tb,
                             hipStream_t s)
{
    return launch_emulate_generic(p, A, B, C, D, m, n, k, batch, ta, tb, s);
}

} // namespace mmaemu
