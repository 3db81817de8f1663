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
#include "fdpa_int.hpp"
#include "efdpa_pair.hpp"

namespace mmaemu {

// EXACT: Algorithm "E-FDPA" (its 640-bit accumulator sits in private memory, so it gets instantiations of its own and the
// other modes stay free of scratch memory)
template <int TA, int TB, bool EXACT>
__global__ void __launch_bounds__(256)
emulate_generic_kernel(ModelArgs p, const typename Fmt<TA>::elem *__restrict__ A,
                       const typename Fmt<TB>::elem *__restrict__ B, const uint32_t *C, uint32_t *D,
                       uint32_t m, uint32_t n, uint32_t k, uint64_t total, const uint8_t *__restrict__ SA,
                       const uint8_t *__restrict__ SB, uint32_t block)
{
    const uint64_t mn = (uint64_t)m * n;
    for (uint64_t o = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total;
         o += (uint64_t)gridDim.x * blockDim.x) {
        const uint64_t t = o / mn;
        const uint32_t r = (uint32_t)(o - t * mn);
        const uint32_t i = r / n, j = r - i * n;
        const typename Fmt<TA>::elem *a = A + (t * m + i) * (uint64_t)k;
        const typename Fmt<TB>::elem *b = B + (t * n + j) * (uint64_t)k;
        const bool acc16 = (p.flags & FL_ACC16) != 0;
        uint32_t d = acc16 ? half_bits_to_float_bits(reinterpret_cast<const uint16_t *>(C)[o]) : C[o];
        if (acc16 && (d & 0x7FFFFFFFu) > 0x7F800000u) d = p.nan_bits;
        ScaleRef sr = no_scales();
        if (SA) {                                   // Algorithm "ST-FDPA": this row's and this column's block scales
            sr.sa = SA + (t * m + i) * (uint64_t)(k / block);
            sr.sb = SB + (t * n + j) * (uint64_t)(k / block);
            sr.block = block;
        }
        for (uint32_t k0 = 0; k0 < k; k0 += p.L) {
            sr.k0 = k0;
            if constexpr (EXACT) {
                // first in a pair of binary64 numbers, which holds the exact sum of most groups; the 640-bit accumulator
                // only where it does not (the payload variation goes there directly)
                if (!(p.flags & FL_NAN_PROPAGATE)) {
                    const StaticFmt<TA> fa{};
                    const StaticFmt<TB> fb{};
                    ExactPair sum;
                    sum.start((p.ftz_in && (d & 0x7F800000u) == 0) ? 0u : d);
                    for (uint32_t kk = 0; kk < p.L; ++kk)
                        sum.add(dec_value(fa, decode_as(fa, fa.load(a + k0, kk), p.ftz_in)), dec_value(fb, decode_as(fb, fb.load(b + k0, kk), p.ftz_in)));
                    uint32_t out;
                    if (sum.finish(p, out)) { d = out; continue; }
                }
            }
            d = fdpa_group<EXACT>(p, StaticFmt<TA>{}, StaticFmt<TB>{}, a + k0, b + k0, p.L, d, sr);
        }
        if (acc16) reinterpret_cast<uint16_t *>(D)[o] = (uint16_t)((d & 0x7FFFFFFFu) > 0x7F800000u ? p.nan16 : float_bits_to_half_bits(d));
        else D[o] = d;
    }
}

template <int TA, int TB>
static mmaemu_status launch_t(const ModelArgs &p, const void *A, const void *B, const void *C, void *D,
                              uint32_t m, uint32_t n, uint32_t k, uint64_t batch, hipStream_t s, const uint8_t *SA,
                              const uint8_t *SB, uint32_t block)
{
    const uint64_t total = batch * m * n;
    uint64_t blocks = (total + 255) / 256;
    if (blocks > (1ull << 22)) blocks = 1ull << 22;     // grid-stride beyond that
    if (p.c_mode == MMAEMU_C_EXACT)
        hipLaunchKernelGGL((emulate_generic_kernel<TA, TB, true>), dim3((uint32_t)blocks), dim3(256), 0, s, p,
                           (const typename Fmt<TA>::elem *)A, (const typename Fmt<TB>::elem *)B,
                           (const uint32_t *)C, (uint32_t *)D, m, n, k, total, SA, SB, block);
    else
        hipLaunchKernelGGL((emulate_generic_kernel<TA, TB, false>), dim3((uint32_t)blocks), dim3(256), 0, s, p,
                           (const typename Fmt<TA>::elem *)A, (const typename Fmt<TB>::elem *)B,
                           (const uint32_t *)C, (uint32_t *)D, m, n, k, total, SA, SB, block);
    MMAEMU_HIP(hipGetLastError());
    set_last_kernel(p.c_mode == MMAEMU_C_EXACT ? "general, exact sum" : (SA ? "general, block-scaled" : "general"));
    return MMAEMU_OK;
}

mmaemu_status launch_emulate_generic(const ModelArgs &p, const void *A, const void *B, const void *C, void *D,
                                     uint32_t m, uint32_t n, uint32_t k, uint64_t batch, uint32_t ta,
                                     uint32_t tb, hipStream_t s, const uint8_t *SA, const uint8_t *SB, uint32_t block)
{
#define CASE(X, Y) if (ta == X && tb == Y) return launch_t<X, Y>(p, A, B, C, D, m, n, k, batch, s, SA, SB, block)
    CASE(MMAEMU_FP8_E4M3, MMAEMU_FP8_E4M3); CASE(MMAEMU_FP8_E4M3, MMAEMU_FP8_E5M2);
    CASE(MMAEMU_FP8_E4M3, MMAEMU_FP16);     CASE(MMAEMU_FP8_E4M3, MMAEMU_BF16);
    CASE(MMAEMU_FP8_E5M2, MMAEMU_FP8_E4M3); CASE(MMAEMU_FP8_E5M2, MMAEMU_FP8_E5M2);
    CASE(MMAEMU_FP8_E5M2, MMAEMU_FP16);     CASE(MMAEMU_FP8_E5M2, MMAEMU_BF16);
    CASE(MMAEMU_FP16, MMAEMU_FP8_E4M3);     CASE(MMAEMU_FP16, MMAEMU_FP8_E5M2);
    CASE(MMAEMU_FP16, MMAEMU_FP16);         CASE(MMAEMU_FP16, MMAEMU_BF16);
    CASE(MMAEMU_BF16, MMAEMU_FP8_E4M3);     CASE(MMAEMU_BF16, MMAEMU_FP8_E5M2);
    CASE(MMAEMU_BF16, MMAEMU_FP16);         CASE(MMAEMU_BF16, MMAEMU_BF16);
    CASE(MMAEMU_TF32, MMAEMU_TF32);         CASE(MMAEMU_FP32, MMAEMU_FP32);
    // FP6 / FP4 with each other and with FP8
#define NARROW_ROW(X) CASE(X, MMAEMU_FP8_E4M3); CASE(X, MMAEMU_FP8_E5M2); CASE(X, MMAEMU_FP6_E2M3); CASE(X, MMAEMU_FP6_E3M2); CASE(X, MMAEMU_FP4_E2M1)
#define NARROW_COL(Y) CASE(MMAEMU_FP8_E4M3, Y); CASE(MMAEMU_FP8_E5M2, Y)
    NARROW_ROW(MMAEMU_FP6_E2M3); NARROW_ROW(MMAEMU_FP6_E3M2); NARROW_ROW(MMAEMU_FP4_E2M1);
    NARROW_COL(MMAEMU_FP6_E2M3); NARROW_COL(MMAEMU_FP6_E3M2); NARROW_COL(MMAEMU_FP4_E2M1);
#undef NARROW_ROW
#undef NARROW_COL
#undef CASE
    set_error("unsupported operand types a=%u b=%u", ta, tb);
    return MMAEMU_ERR_UNSUPPORTED;
}

} // namespace mmaemu
