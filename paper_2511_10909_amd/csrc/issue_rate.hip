// Issue-rate probes: for each vector-ALU instruction that the emulation kernels' hot loops are made of, a kernel of
// eight independent dependency chains per lane.  Timed from outside (events around the launch), they give the
// instruction's lane-instructions per second on this chip: the measured counterpart of the ALU peak that the
// benchmark's roofline is quoted against (256 CUs x 4 SIMDs x 16 lanes x clock).
#include "common.hpp"

namespace mmaemu {

constexpr int CHAINS = 8;

#define PROBE32(NAME, ASM)                                                                             \
    __global__ void __launch_bounds__(256) NAME(uint32_t *out, uint32_t seed, uint32_t iters)           \
    {                                                                                                  \
        uint32_t x[CHAINS], y = seed + threadIdx.x, z = seed ^ 0x1234567u;                             \
        for (int i = 0; i < CHAINS; ++i) x[i] = seed * (i + 1) + threadIdx.x;                          \
        for (uint32_t it = 0; it < iters; ++it) {                                                      \
            _Pragma("unroll") for (int i = 0; i < CHAINS; ++i) asm volatile(ASM : "+v"(x[i]) : "v"(y), "v"(z)); \
        }                                                                                              \
        uint32_t s = 0;                                                                                \
        for (int i = 0; i < CHAINS; ++i) s ^= x[i];                                                    \
        if (s == 0x9999999u) out[threadIdx.x] = s;                                                     \
    }

#define PROBE64(NAME, ASM)                                                                             \
    __global__ void __launch_bounds__(256) NAME(uint32_t *out, uint32_t seed, uint32_t iters)           \
    {                                                                                                  \
        double x[CHAINS], y = (double)(seed + threadIdx.x + 3), z = (double)(seed ^ 0x1234567u);       \
        uint32_t w = seed & 7;                                                                         \
        for (int i = 0; i < CHAINS; ++i) x[i] = (double)(seed * (i + 1) + threadIdx.x + 1);            \
        for (uint32_t it = 0; it < iters; ++it) {                                                      \
            _Pragma("unroll") for (int i = 0; i < CHAINS; ++i) asm volatile(ASM : "+v"(x[i]) : "v"(y), "v"(z), "v"(w)); \
        }                                                                                              \
        double s = 0;                                                                                  \
        for (int i = 0; i < CHAINS; ++i) s += x[i];                                                    \
        if (s == 1234.5) out[threadIdx.x] = 1;                                                         \
    }

PROBE32(probe_add_u32, "v_add_u32 %0, %1, %0")
PROBE32(probe_add3_u32, "v_add3_u32 %0, %0, %1, %2")
PROBE32(probe_max_u32, "v_max_u32 %0, %1, %0")
PROBE32(probe_max3_i32, "v_max3_i32 %0, %0, %1, %2")
PROBE32(probe_lshlrev_b32, "v_lshlrev_b32 %0, %1, %0")
PROBE32(probe_mul_u32_u24, "v_mul_u32_u24 %0, %1, %0")
PROBE32(probe_xad_u32, "v_xad_u32 %0, %0, %1, %2")
PROBE32(probe_pk_add_u16, "v_pk_add_u16 %0, %1, %0")
PROBE32(probe_pk_max_u16, "v_pk_max_u16 %0, %1, %0")
PROBE32(probe_mul_f32, "v_mul_f32 %0, %1, %0")
PROBE32(probe_cvt_i32_f32, "v_cvt_i32_f32 %0, %0")
PROBE32(probe_cvt_f32_i32, "v_cvt_f32_i32 %0, %0")
PROBE32(probe_ldexp_f32, "v_ldexp_f32 %0, %0, %1")
PROBE32(probe_med3_i32, "v_med3_i32 %0, %0, %1, %2")
PROBE64(probe_mul_f64, "v_mul_f64 %0, %1, %0")
PROBE64(probe_add_f64, "v_add_f64 %0, %1, %0")
PROBE64(probe_ldexp_f64, "v_ldexp_f64 %0, %0, %3")
PROBE64(probe_trunc_f64, "v_trunc_f64 %0, %0")
PROBE64(probe_cvt_f64_i32, "v_cvt_f64_i32 %0, %3")

typedef void (*ProbeKernel)(uint32_t *, uint32_t, uint32_t);
static const struct { const char *name; ProbeKernel fn; } PROBES[] = {
    {"v_add_u32", probe_add_u32},         {"v_add3_u32", probe_add3_u32},       {"v_max_u32", probe_max_u32},
    {"v_max3_i32", probe_max3_i32},       {"v_lshlrev_b32", probe_lshlrev_b32}, {"v_mul_u32_u24", probe_mul_u32_u24},
    {"v_xad_u32", probe_xad_u32},         {"v_pk_add_u16", probe_pk_add_u16},   {"v_pk_max_u16", probe_pk_max_u16},
    {"v_mul_f32", probe_mul_f32},         {"v_cvt_i32_f32", probe_cvt_i32_f32}, {"v_cvt_f32_i32", probe_cvt_f32_i32},
    {"v_ldexp_f32", probe_ldexp_f32},     {"v_med3_i32", probe_med3_i32},       {"v_mul_f64", probe_mul_f64},
    {"v_add_f64", probe_add_f64},         {"v_ldexp_f64", probe_ldexp_f64},     {"v_trunc_f64", probe_trunc_f64},
    {"v_cvt_f64_i32", probe_cvt_f64_i32},
};
constexpr uint32_t N_PROBES = sizeof(PROBES) / sizeof(PROBES[0]);

uint32_t issue_probe_count() { return N_PROBES; }
const char *issue_probe_name(uint32_t op) { return op < N_PROBES ? PROBES[op].name : nullptr; }

mmaemu_status launch_issue_probe(uint32_t op, uint32_t iters, uint32_t workgroups, uint32_t *out, hipStream_t s)
{
    hipLaunchKernelGGL(PROBES[op].fn, dim3(workgroups), dim3(256), 0, s, out, 12345u, iters);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

} // namespace mmaemu
