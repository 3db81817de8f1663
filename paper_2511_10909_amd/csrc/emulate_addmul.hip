// The model built from binary flush-to-zero operations (paper Sec. 4.1.1): Algorithm "Phi_FTZ-AddMul" around
// Algorithm "FTZ-Add and FTZ-Mul".  One thread per output element.  The device's binary32 multiply and add are
// IEEE-754 basic operations (RNE of the exact result; this file is compiled without contraction), which is what
// FTZ-Mul and FTZ-Add ask for before their flush; the flush of results below 2^-126 (sign kept), the flush of
// subnormal inputs to +0.0 and the model's NaN encoding are applied explicitly.
#include "fdpa_int.hpp"

namespace mmaemu {

// operand -> binary32 value (every supported operand value is a binary32 number); subnormals become +0.0
template <int T>
__device__ __forceinline__ float flushed_operand(uint32_t bits)
{
    const Dec x = decode<T>(bits, 1u);               // ftz_in = 1: FlushSubnormal
    if (x.cls == CLS_NAN) return __uint_as_float(0x7FC00000u);
    if (x.cls == CLS_INF) return __uint_as_float(x.sign ? 0xFF800000u : 0x7F800000u);
    const float mag = ldexpf((float)x.sig, x.exp - Fmt<T>::MB);      // exact
    return __uint_as_float(__float_as_uint(mag) | (x.sign << 31));
}

__device__ __forceinline__ float ftz_fix(float z, uint32_t nan_bits)
{
    uint32_t b = __float_as_uint(z);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) b = nan_bits;
    else if ((b & 0x7F800000u) == 0) b &= 0x80000000u;                // |z| < 2^-126: zero of the same sign
    return __uint_as_float(b);
}

template <int TA, int TB>
__global__ void __launch_bounds__(256)
emulate_addmul_kernel(uint32_t P, uint32_t nan_bits, const typename Fmt<TA>::elem *__restrict__ A,
                      const typename Fmt<TB>::elem *__restrict__ B, const uint32_t *C, uint32_t *D,
                      uint32_t m, uint32_t n, uint32_t k, uint64_t total)
{
    const uint64_t mn = (uint64_t)m * n;
    for (uint64_t o = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total;
         o += (uint64_t)gridDim.x * blockDim.x) {
        const uint64_t t = o / mn;
        const uint32_t r = (uint32_t)(o - t * mn);
        const uint32_t i = r / n, j = r - i * n;
        const typename Fmt<TA>::elem *a = A + (t * m + i) * (uint64_t)k;
        const typename Fmt<TB>::elem *b = B + (t * n + j) * (uint64_t)k;
        uint32_t cb = C[o];
        if ((cb & 0x7F800000u) == 0) cb &= (cb & 0x007FFFFFu) ? 0u : 0x80000000u;     // subnormal accumulator -> +0.0
        float d = ftz_fix(__uint_as_float(cb), nan_bits);
        for (uint32_t k0 = 0; k0 < k; k0 += P) {
            float p[4];
            for (uint32_t l = 0; l < P; ++l)
                p[l] = ftz_fix(__fmul_rn(flushed_operand<TA>(a[k0 + l]), flushed_operand<TB>(b[k0 + l])), nan_bits);
            float s = ftz_fix(__fadd_rn(p[0], p[1]), nan_bits);
            if (P == 4) {
                const float s2 = ftz_fix(__fadd_rn(p[2], p[3]), nan_bits);
                s = ftz_fix(__fadd_rn(s, s2), nan_bits);
            }
            d = ftz_fix(__fadd_rn(d, s), nan_bits);
        }
        D[o] = __float_as_uint(d);
    }
}

template <int TA, int TB>
static mmaemu_status launch_t(const ModelArgs &p, const void *A, const void *B, const void *C, void *D,
                              uint32_t m, uint32_t n, uint32_t k, uint64_t batch, hipStream_t s)
{
    const uint64_t total = batch * m * n;
    uint64_t blocks = (total + 255) / 256;
    if (blocks > (1ull << 22)) blocks = 1ull << 22;
    hipLaunchKernelGGL((emulate_addmul_kernel<TA, TB>), dim3((uint32_t)blocks), dim3(256), 0, s, p.L, p.nan_bits,
                       (const typename Fmt<TA>::elem *)A, (const typename Fmt<TB>::elem *)B,
                       (const uint32_t *)C, (uint32_t *)D, m, n, k, total);
    MMAEMU_HIP(hipGetLastError());
    set_last_kernel("ftz-addmul P=%u", p.L);
    return MMAEMU_OK;
}

mmaemu_status launch_emulate_addmul(const ModelArgs &p, const void *A, const void *B, const void *C, void *D,
                                    uint32_t m, uint32_t n, uint32_t k, uint64_t batch, uint32_t ta,
                                    uint32_t tb, hipStream_t s)
{
#define CASE(X, Y) if (ta == X && tb == Y) return launch_t<X, Y>(p, A, B, C, D, m, n, k, batch, s)
    CASE(MMAEMU_FP8_E4M3, MMAEMU_FP8_E4M3); CASE(MMAEMU_FP8_E4M3, MMAEMU_FP8_E5M2);
    CASE(MMAEMU_FP8_E4M3, MMAEMU_FP16);     CASE(MMAEMU_FP8_E4M3, MMAEMU_BF16);
    CASE(MMAEMU_FP8_E5M2, MMAEMU_FP8_E4M3); CASE(MMAEMU_FP8_E5M2, MMAEMU_FP8_E5M2);
    CASE(MMAEMU_FP8_E5M2, MMAEMU_FP16);     CASE(MMAEMU_FP8_E5M2, MMAEMU_BF16);
    CASE(MMAEMU_FP16, MMAEMU_FP8_E4M3);     CASE(MMAEMU_FP16, MMAEMU_FP8_E5M2);
    CASE(MMAEMU_FP16, MMAEMU_FP16);         CASE(MMAEMU_FP16, MMAEMU_BF16);
    CASE(MMAEMU_BF16, MMAEMU_FP8_E4M3);     CASE(MMAEMU_BF16, MMAEMU_FP8_E5M2);
    CASE(MMAEMU_BF16, MMAEMU_FP16);         CASE(MMAEMU_BF16, MMAEMU_BF16);
#undef CASE
    set_error("unsupported operand types a=%u b=%u", ta, tb);
    return MMAEMU_ERR_UNSUPPORTED;
}

} // namespace mmaemu
