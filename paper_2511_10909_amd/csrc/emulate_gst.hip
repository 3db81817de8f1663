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

// The same model with operand sharing: a workgroup owns 16 x 16 blocks of D (one output per thread).  Per operation (L
// values of k) the block's rows of A and of B are decoded once into LDS as signed 8-bit integers counting units of 2^-1
// (an FP4 value is 0, 1, 2, 3, 4, 6, 8 or 12 of them), four to a dword, so a group's exact dot product in units of 2^-2 is
// a run of v_dot4_i32_i8; the scale codes are decoded once per row and block as well (significand in units of 2^-3,
// exponent, NaN flag).  Alignment, summation and rounding are those of the kernel above.
constexpr int GST_LMAX = 256;                                     // values of k per operation this kernel stages
constexpr uint32_t GST_NAN_SCALE = 0xFFFFFFFFu;

__device__ __forceinline__ uint32_t fp4_units(uint32_t code)      // -> value in units of 2^-1 as a signed byte
{
    const uint32_t mag = code & 7u;
    const uint32_t v = mag < 2u ? mag : (2u | (mag & 1u)) << ((mag >> 1) - 1u);
    return ((code & 8u) ? 0u - v : v) & 0xFFu;
}

__global__ void __launch_bounds__(256)
emulate_gst_blocks_kernel(GstArgs g, const uint8_t *__restrict__ A, const uint8_t *__restrict__ B, const uint32_t *C, uint32_t *D,
                          const uint8_t *__restrict__ SA, const uint8_t *__restrict__ SB, uint32_t m, uint32_t n, uint32_t k, uint64_t nblocks)
{
    constexpr int VS = GST_LMAX / 4 + 4;                          // dwords per staged row (16-byte aligned, rows spread over the banks)
    __shared__ __attribute__((aligned(16))) uint32_t Av[16][VS], Bv[16][VS];
    __shared__ uint32_t As[16][GST_LMAX / 16 + 1], Bs[16][GST_LMAX / 16 + 1];          // per row and scale block: (exp + 512) << 8 | sig8, or the NaN mark
    const uint32_t tid = threadIdx.x, i = tid / 16u, j = tid % 16u;
    const uint32_t bpr = n / 16u, bpt = (m / 16u) * bpr;
    const uint32_t nblk = k / g.block, ng = g.L / g.G, bpo = g.L / g.block;              // scale blocks per row / groups and scale blocks per operation
    const int F = (int)g.F;
    for (uint64_t w = blockIdx.x; w < nblocks; w += gridDim.x) {
        const uint64_t t = w / bpt;
        const uint32_t r = (uint32_t)(w - t * bpt), bi = r / bpr, bj = r - bi * bpr;
        const uint64_t arow0 = t * m + 16u * bi, brow0 = t * n + 16u * bj;
        const uint64_t o = (arow0 + i) * (uint64_t)n + 16u * bj + j;
        uint32_t d = C[o];
        for (uint32_t k0 = 0; k0 < k; k0 += g.L) {
            __syncthreads();                                      // (the previous operation's readers)
            for (uint32_t e = tid; e < 16u * (g.L / 4u); e += 256u) {
                const uint32_t row = e / (g.L / 4u), q = e - row * (g.L / 4u);
                const uint32_t ra = *reinterpret_cast<const uint32_t *>(A + (arow0 + row) * (uint64_t)k + k0 + 4u * q);
                const uint32_t rb = *reinterpret_cast<const uint32_t *>(B + (brow0 + row) * (uint64_t)k + k0 + 4u * q);
                Av[row][q] = fp4_units(ra) | (fp4_units(ra >> 8) << 8) | (fp4_units(ra >> 16) << 16) | (fp4_units(ra >> 24) << 24);
                Bv[row][q] = fp4_units(rb) | (fp4_units(rb >> 8) << 8) | (fp4_units(rb >> 16) << 16) | (fp4_units(rb >> 24) << 24);
            }
            for (uint32_t e = tid; e < 32u * bpo; e += 256u) {
                const uint32_t which = e / (16u * bpo), rem = e - which * 16u * bpo, row = rem / bpo, q = rem - row * bpo;
                const uint8_t *src = which ? SB + (brow0 + row) * (uint64_t)nblk : SA + (arow0 + row) * (uint64_t)nblk;
                int sig8, ex;
                const bool ok = gst_scale(src[k0 / g.block + q], g.scale_format, sig8, ex);
                (which ? Bs : As)[row][q] = ok ? ((uint32_t)(ex + 512) << 8) | (uint32_t)sig8 : GST_NAN_SCALE;
            }
            __syncthreads();
            const Dec dc = decode<MMAEMU_FP32>(d, 0);
            if (dc.cls == CLS_NAN) { d = g.nan_bits; continue; }
            // first sweep: a NaN scale, and the maximum exponent
            bool nan = false;
            int emax = dc.exp;
            for (uint32_t q = 0; q < bpo; ++q) {
                const uint32_t x = As[i][q], y = Bs[j][q];
                nan |= x == GST_NAN_SCALE || y == GST_NAN_SCALE;
                const int e = (int)(x >> 8) + (int)(y >> 8) - 1024;
                emax = e > emax ? e : emax;
            }
            if (nan) { d = g.nan_bits; continue; }
            if (dc.cls == CLS_INF) continue;                                  // an infinite accumulator stays
            // second sweep: exact dot product per group, aligned at e_max with F fractional bits, summed
            const int unit = emax - F;
            int64_t S = 0;
            for (uint32_t q = 0; q < ng; ++q) {
                const uint32_t kq = q * g.G, blk = kq / g.block;
                const uint32_t x = As[i][blk], y = Bs[j][blk];
                int32_t p = 0;
                for (uint32_t kk = kq / 4u; kk < (kq + g.G) / 4u; ++kk) p = __builtin_amdgcn_sdot4((int)Av[i][kk], (int)Bv[j][kk], p, false);
                S += gst_align((int64_t)p * (int)(x & 0xFFu) * (int)(y & 0xFFu), (int)(x >> 8) + (int)(y >> 8) - 1024 - 8, unit);
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
    if (m % 16 == 0 && n % 16 == 0 && g.G % 4 == 0 && g.L <= (uint32_t)GST_LMAX && g.block >= 16 &&
        ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 3) == 0) {
        const uint64_t nblocks = total / 256;
        const uint64_t grid = nblocks < (1ull << 16) ? nblocks : (1ull << 16);
        hipLaunchKernelGGL(emulate_gst_blocks_kernel, dim3((uint32_t)grid), dim3(256), 0, s, g, (const uint8_t *)A, (const uint8_t *)B,
                           (const uint32_t *)C, (uint32_t *)D, SA, SB, m, n, k, nblocks);
        MMAEMU_HIP(hipGetLastError());
        set_last_kernel("gst-fdpa, 16x16 blocks through LDS");
        return MMAEMU_OK;
    }
    uint64_t blocks = (total + 255) / 256;
    if (blocks > (1ull << 22)) blocks = 1ull << 22;
    hipLaunchKernelGGL(emulate_gst_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, g, (const uint8_t *)A, (const uint8_t *)B,
                       (const uint32_t *)C, (uint32_t *)D, SA, SB, m, n, k, total);
    MMAEMU_HIP(hipGetLastError());
    set_last_kernel("gst-fdpa");
    return MMAEMU_OK;
}

} // namespace mmaemu
