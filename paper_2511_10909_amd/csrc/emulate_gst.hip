// Group-scaled truncated FDPA (paper Algorithm "GST-FDPA", Sec. 4.1.3): FP4 operands with one scale factor pair per
// block, an exact dot product per group of G products, then the truncated fused sum of the group terms and the
// accumulator.  One thread per output element, integer arithmetic: an FP4 value is sig 2^(Exp - 1) with sig in 0..3,
// so a product counts units of 2^-2; a scale significand counts units of 2^-3 (E8M0's 1.0 is eight of them); a group
// term s_g = p_g sig(alpha) sig(beta) therefore counts units of 2^-8 and stays below 2^22.
#include "fdpa_int.hpp"

namespace mmaemu {

// scale code -> significand in units of 2^-3 and exponent; false for a NaN code
__device__ __forceinline__ bool gst_scale(uint32_t code, uint32_t fmt, int &sig8, int &exp)
{
    if (fmt == MMAEMU_SCALE_FORMAT_E8M0) { sig8 = 8; exp = (int)code - 127; return code != 0xFFu; }
    const Dec d = decode<MMAEMU_FP8_E4M3>(code & 0x7Fu, 0);
    sig8 = (int)d.sig;
    exp = d.exp;
    return d.cls != CLS_NAN;
}

__device__ __forceinline__ int64_t gst_align(int64_t s, int lsb, int unit)      // truncation toward zero
{
    const int sh = lsb - unit;
    const uint64_t mag = (uint64_t)(s < 0 ? -s : s);
    const uint64_t al = sh >= 0 ? (mag << sh) : (sh > -64 ? (mag >> (-sh)) : 0ull);
    return s < 0 ? -(int64_t)al : (int64_t)al;
}

__global__ void __launch_bounds__(256)
emulate_gst_kernel(GstArgs g, const uint8_t *__restrict__ A, const uint8_t *__restrict__ B, const uint32_t *C, uint32_t *D,
                   const uint8_t *__restrict__ SA, const uint8_t *__restrict__ SB, uint32_t m, uint32_t n, uint32_t k, uint64_t total)
{
    const uint64_t mn = (uint64_t)m * n;
    const uint32_t nblk = k / g.block, ng = g.L / g.G;
    const int F = (int)g.F;
    for (uint64_t o = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total; o += (uint64_t)gridDim.x * blockDim.x) {
        const uint64_t t = o / mn;
        const uint32_t r = (uint32_t)(o - t * mn), i = r / n, j = r - i * n;
        const uint8_t *a = A + (t * m + i) * (uint64_t)k, *b = B + (t * n + j) * (uint64_t)k;
        const uint8_t *al = SA + (t * m + i) * (uint64_t)nblk, *be = SB + (t * n + j) * (uint64_t)nblk;
        uint32_t d = C[o];
        for (uint32_t k0 = 0; k0 < k; k0 += g.L) {
            const Dec dc = decode<MMAEMU_FP32>(d, 0);
            if (dc.cls == CLS_NAN) { d = g.nan_bits; continue; }
            // first sweep: a NaN scale, and the maximum exponent
            bool nan = false;
            int emax = dc.exp;
            for (uint32_t q = 0; q < ng; ++q) {
                const uint32_t blk = (k0 + q * g.G) / g.block;
                int sa, ea, sb, eb;
                nan |= !gst_scale(al[blk], g.scale_format, sa, ea);
                nan |= !gst_scale(be[blk], g.scale_format, sb, eb);
                emax = ea + eb > emax ? ea + eb : emax;
            }
            if (nan) { d = g.nan_bits; continue; }
            if (dc.cls == CLS_INF) continue;                                  // an infinite accumulator stays
            // second sweep: exact dot product per group, aligned at e_max with F fractional bits, summed
            const int unit = emax - F;
            int64_t S = 0;
            for (uint32_t q = 0; q < ng; ++q) {
                const uint32_t kq = k0 + q * g.G, blk = kq / g.block;
                int sa, ea, sb, eb;
                gst_scale(al[blk], g.scale_format, sa, ea);
                gst_scale(be[blk], g.scale_format, sb, eb);
                int32_t p = 0;
                for (uint32_t kk = kq; kk < kq + g.G; ++kk) {
                    const Dec x = decode<MMAEMU_FP4_E2M1>(a[kk], 0), y = decode<MMAEMU_FP4_E2M1>(b[kk], 0);
                    const int32_t tq = (int32_t)(x.sig * y.sig) << (x.exp + y.exp);                // units of 2^-2
                    p += (x.sign ^ y.sign) ? -tq : tq;
                }
                S += gst_align((int64_t)p * sa * sb, ea + eb - 8, unit);
            }
            S += gst_align(dc.sign ? -(int64_t)dc.sig : (int64_t)dc.sig, dc.exp - 23, unit);
            const uint32_t neg = S < 0;
            const uint64_t mag = (uint64_t)(neg ? -S : S);
            d = mag ? round_to_fp32(neg, mag, unit, 0, g.out_round) : 0u;
        }
        D[o] = d;
    }
}

mmaemu_status launch_emulate_gst(const GstArgs &g, const void *A, const void *B, const void *C, void *D, const uint8_t *SA,
                                 const uint8_t *SB, uint32_t m, uint32_t n, uint32_t k, uint64_t batch, hipStream_t s)
{
    const uint64_t total = batch * m * n;
    uint64_t blocks = (total + 255) / 256;
    if (blocks > (1ull << 22)) blocks = 1ull << 22;
    hipLaunchKernelGGL(emulate_gst_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, g, (const uint8_t *)A, (const uint8_t *)B,
                       (const uint32_t *)C, (uint32_t *)D, SA, SB, m, n, k, total);
    MMAEMU_HIP(hipGetLastError());
    set_last_kernel("gst-fdpa");
    return MMAEMU_OK;
}

} // namespace mmaemu
