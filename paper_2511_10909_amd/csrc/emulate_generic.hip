// General-purpose emulation kernel: one thread per output element, integer arithmetic
// throughout, every operand type, every supported parameter value, special values
// included.  It is the path taken by shapes and parameters that the tiled kernels do not
// cover, and by tiles that hold NaN or infinities.
//
// Per element it runs the chained FDPA model (paper Algorithm "Phi_FDPA") around the
// truncated fused dot-product-add (Algorithm "T-FDPA"): two passes over each group of L
// products -- first the special-value scan (Sec. 4.2) and e_max, then alignment with
// truncation toward zero to F fractional bits and the exact integer sum -- followed by
// the conversion rho and the optional output flush (Algorithm "FTZ-Add/FTZ-Mul").
#include "common.hpp"

namespace mmaemu {

enum { CLS_ZERO = 0, CLS_SUB = 1, CLS_NORMAL = 2, CLS_INF = 3, CLS_NAN = 4 };

struct Dec {
    uint32_t sig;
    int exp;
    uint32_t sign;
    int cls;
};

template <int T>
__device__ __forceinline__ Dec decode(uint32_t bits, uint32_t ftz_in)
{
    using F = Fmt<T>;
    constexpr uint32_t EMASK = (1u << F::EB) - 1u, MMASK = (1u << F::MB) - 1u;
    const uint32_t E = (bits >> F::MB) & EMASK, M = bits & MMASK;
    Dec d;
    d.sign = (bits >> (F::EB + F::MB)) & 1u;
    d.exp = (E ? (int)E : 1) - F::BIAS;
    d.sig = E ? (M | (1u << F::MB)) : M;
    d.cls = E ? CLS_NORMAL : (M ? CLS_SUB : CLS_ZERO);
    if (F::IEEE) {
        if (E == EMASK) d.cls = M ? CLS_NAN : CLS_INF;
    } else {
        if (E == EMASK && M == MMASK) d.cls = CLS_NAN;
    }
    if (ftz_in && d.cls == CLS_SUB) { d.cls = CLS_ZERO; d.sig = 0; d.sign = 0; }   // FlushSubnormal: -> +0.0
    return d;
}

template <int TA, int TB>
__device__ uint32_t fdpa_group(const ModelArgs &p, const typename Fmt<TA>::elem *a,
                               const typename Fmt<TB>::elem *b, uint32_t L, uint32_t c)
{
    constexpr int FA = Fmt<TA>::MB, FB = Fmt<TB>::MB;
    const Dec dc = decode<MMAEMU_FP32>(c, p.ftz_in);

    // pass 1: special values and the maximum exponent
    bool any_nan = dc.cls == CLS_NAN, pinf = false, ninf = false;
    int emax = -100000;
    for (uint32_t k = 0; k < L; ++k) {
        const Dec x = decode<TA>(a[k], p.ftz_in), y = decode<TB>(b[k], p.ftz_in);
        if (x.cls == CLS_NAN || y.cls == CLS_NAN) any_nan = true;
        else if (x.cls == CLS_INF || y.cls == CLS_INF) {
            if (x.cls == CLS_ZERO || y.cls == CLS_ZERO) any_nan = true;      // inf * 0
            else if (x.sign ^ y.sign) ninf = true;
            else pinf = true;
        } else {
            const int e = x.exp + y.exp;
            emax = e > emax ? e : emax;
        }
    }
    if (dc.cls == CLS_INF) { if (dc.sign) ninf = true; else pinf = true; }
    if (any_nan || (pinf && ninf)) return p.nan_bits;
    if (pinf) return 0x7F800000u;
    if (ninf) return 0xFF800000u;

    if (p.c_mode == MMAEMU_C_IN_GROUP && dc.exp > emax) emax = dc.exp;
    const int unit = emax - p.F;            // aligned terms count multiples of 2^unit

    // pass 2: align, truncate toward zero, sum exactly
    int64_t S = 0;
    for (uint32_t k = 0; k < L; ++k) {
        const Dec x = decode<TA>(a[k], p.ftz_in), y = decode<TB>(b[k], p.ftz_in);
        const uint64_t prod = (uint64_t)(x.sig * y.sig);                    // <= 22 bits
        const int sh = (x.exp + y.exp - FA - FB) - unit;                    // <= F
        const uint64_t al = sh >= 0 ? (prod << sh) : (sh > -32 ? (prod >> (-sh)) : 0ull);
        S += (x.sign ^ y.sign) ? -(int64_t)al : (int64_t)al;
    }
    uint32_t d;
    if (p.c_mode == MMAEMU_C_IN_GROUP) {
        const int sh = (dc.exp - 23) - unit;
        const uint64_t al = sh >= 0 ? ((uint64_t)dc.sig << sh) : (sh > -32 ? ((uint64_t)dc.sig >> (-sh)) : 0ull);
        S += dc.sign ? -(int64_t)al : (int64_t)al;
        const uint32_t neg = S < 0;
        const uint64_t mag = (uint64_t)(neg ? -S : S);
        d = mag ? round_to_fp32(neg, mag, unit, 0, p.out_round) : 0u;
    } else {
        const uint32_t neg = S < 0;
        d = add_exact_round(neg, (uint64_t)(neg ? -S : S), unit, dc.sign, (uint64_t)dc.sig, dc.exp - 23, p.out_round);
    }
    if (p.ftz_out && (d & 0x7F800000u) == 0) d &= 0x80000000u;
    return d;
}

template <int TA, int TB>
__global__ void __launch_bounds__(256)
emulate_generic_kernel(ModelArgs p, const typename Fmt<TA>::elem *__restrict__ A,
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
        uint32_t d = C[o];
        for (uint32_t k0 = 0; k0 < k; k0 += p.L) d = fdpa_group<TA, TB>(p, a + k0, b + k0, p.L, d);
        D[o] = d;
    }
}

template <int TA, int TB>
static mmaemu_status launch_t(const ModelArgs &p, const void *A, const void *B, const void *C, void *D,
                              uint32_t m, uint32_t n, uint32_t k, uint64_t batch, hipStream_t s)
{
    const uint64_t total = batch * m * n;
    uint64_t blocks = (total + 255) / 256;
    if (blocks > (1ull << 22)) blocks = 1ull << 22;     // grid-stride beyond that
    hipLaunchKernelGGL((emulate_generic_kernel<TA, TB>), dim3((uint32_t)blocks), dim3(256), 0, s, p,
                       (const typename Fmt<TA>::elem *)A, (const typename Fmt<TB>::elem *)B,
                       (const uint32_t *)C, (uint32_t *)D, m, n, k, total);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

mmaemu_status launch_emulate_generic(const ModelArgs &p, const void *A, const void *B, const void *C, void *D,
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
