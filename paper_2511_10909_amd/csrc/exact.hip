// Exact dot products on a sample of outputs and the error of an emulated D against them
// (methodology of the paper's Sec. 6.2.4: deviation of a model's output from the real
// result; the real result here is the exact integer dot product of the FP8 operands).
//
// One wavefront per sampled output: lanes stride over k, each accumulating exact products
// in units of 2^LSB0 (LSB0 = the smallest last-place exponent a product can have); an FP8
// product is below 2^33 in value and a multiple of 2^-32, so it needs at most 66 bits;
// per-lane sums are kept in two binary64 numbers that split every product at 2^(LSB0 + 32),
// both exact, and combined into a two-limb (128-bit) signed value that is exact for any
// k <= 2^20.
#include "common.hpp"

namespace mmaemu {

struct I128 { uint64_t lo; int64_t hi; };

__device__ __forceinline__ I128 add128(I128 a, I128 b)
{
    I128 r;
    r.lo = a.lo + b.lo;
    r.hi = a.hi + b.hi + (r.lo < a.lo ? 1 : 0);
    return r;
}

__device__ __forceinline__ I128 neg128(I128 a)
{
    I128 r;
    r.lo = ~a.lo + 1ull;
    r.hi = ~a.hi + (r.lo == 0 ? 1 : 0);
    return r;
}

// a << s for 0 <= s < 128 (two's complement)
__device__ __forceinline__ I128 shl128(I128 a, int s)
{
    I128 r;
    if (s == 0) return a;
    if (s >= 64) { r.lo = 0; r.hi = (int64_t)(a.lo << (s - 64)); return r; }
    r.lo = a.lo << s;
    r.hi = (int64_t)(((uint64_t)a.hi << s) | (a.lo >> (64 - s)));
    return r;
}

template <int T> __device__ __forceinline__ void dec8(uint32_t bits, uint32_t &sig, int &exp, uint32_t &sign, bool &special)
{
    using F = Fmt<T>;
    constexpr uint32_t EMASK = (1u << F::EB) - 1u, MMASK = (1u << F::MB) - 1u;
    const uint32_t E = (bits >> F::MB) & EMASK, M = bits & MMASK;
    sign = (bits >> 7) & 1u;
    exp = (E ? (int)E : 1) - F::BIAS;
    sig = E ? (M | (1u << F::MB)) : M;
    special = F::IEEE ? (E == EMASK) : (E == EMASK && M == MMASK);
}

__global__ void err_stats_reset_kernel(mmaemu_err_stats *st)
{
    uint64_t *w = reinterpret_cast<uint64_t *>(st);
    if (threadIdx.x < sizeof(mmaemu_err_stats) / 8) w[threadIdx.x] = 0ull;   // +0.0 is all-zero bits
}

__device__ __forceinline__ int64_t okey(uint32_t b) { return (b & 0x80000000u) ? -(int64_t)(b & 0x7FFFFFFFu) : (int64_t)b; }

// value of a 128-bit magnitude times 2^lsb as a double (rounded once per limb and once at the sum)
__device__ __forceinline__ double mag_to_double(uint64_t hi, uint64_t lo, int lsb)
{
    return ldexp((double)hi, 64 + lsb) + ldexp((double)lo, lsb);
}

// the four FP8 elements of a word as binary32 numbers (exact), by v_cvt_pk_f32_fp8 / v_cvt_pk_f32_bf8: on gfx950 these
// take the OCP encodings (E4M3 with the single NaN pattern S.1111.111 and no infinity, E5M2 with IEEE-style specials)
typedef float f32x2 __attribute__((ext_vector_type(2)));
template <int T> __device__ __forceinline__ void fp8x4_values(uint32_t w, float (&v)[4])
{
    f32x2 lo, hi;
    if (T == MMAEMU_FP8_E4M3) { lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false); hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true); }
    else { lo = __builtin_amdgcn_cvt_pk_f32_bf8((int)w, false); hi = __builtin_amdgcn_cvt_pk_f32_bf8((int)w, true); }
    v[0] = lo.x; v[1] = lo.y; v[2] = hi.x; v[3] = hi.y;
}

template <int TA, int TB>
__global__ void __launch_bounds__(256)
exact_dot_kernel(const uint8_t *__restrict__ A, const uint8_t *__restrict__ B, const uint32_t *__restrict__ D,
                 uint32_t m, uint32_t n, uint32_t k, uint64_t stride, uint64_t nsamples, mmaemu_err_stats *st)
{
    constexpr int LSB0 = (1 - Fmt<TA>::BIAS - Fmt<TA>::MB) + (1 - Fmt<TB>::BIAS - Fmt<TB>::MB);
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const uint64_t nwaves = ((uint64_t)gridDim.x * blockDim.x) >> 6;
    // statistics are gathered per workgroup in LDS (same layout as mmaemu_err_stats) and
    // flushed once at the end: global atomics on a handful of addresses serialise chip-wide
    constexpr int NW = sizeof(mmaemu_err_stats) / 8;
    __shared__ unsigned long long ls[NW];
    if (threadIdx.x < NW) ls[threadIdx.x] = 0ull;                 // +0.0 is all-zero bits
    __syncthreads();
    unsigned long long *g = ls;
    double *gd = reinterpret_cast<double *>(ls + 5 + 34);
    for (uint64_t sidx = wave; sidx < nsamples; sidx += nwaves) {
        const uint64_t o = sidx * stride;
        const uint32_t i = (uint32_t)(o / n), j = (uint32_t)(o % n);
        const uint8_t *a = A + (uint64_t)i * k, *b = B + (uint64_t)j * k;
        // Per lane: four consecutive k per 32-bit load, decoded by the hardware's own FP8 -> binary32 conversions (two
        // elements per instruction); a product is exact in binary32 (at most 8 significant bits, 2^-32 <= |p| < 2^33).
        // Its binary64 image is split at 2^(LSB0 + 32) by adding and subtracting a constant whose last place that is:
        // the upper part is a multiple of 2^(LSB0 + 32), the lower part a multiple of 2^LSB0 of at most 2^(LSB0 + 31),
        // and with at most 2^14 terms per lane (k <= 2^20) both sums stay below 2^53 of their units, i.e. exact.
        // A NaN or an infinity among the operands makes one of the sums a NaN or an infinity.
        constexpr double SPLIT = 0x1.8p+52 * (LSB0 + 32 >= 0 ? (double)(1ull << (LSB0 + 32 >= 0 ? LSB0 + 32 : 0)) : 1.0 / (double)(1ull << (LSB0 + 32 >= 0 ? 0 : -(LSB0 + 32))));
        double sum_hi = 0.0, sum_lo = 0.0;
        for (uint32_t q = 4 * lane; q < k; q += 256) {
            uint32_t wa, wb;
            if (q + 4 <= k && (((uintptr_t)(a + q) | (uintptr_t)(b + q)) & 3) == 0) {
                wa = *reinterpret_cast<const uint32_t *>(a + q);
                wb = *reinterpret_cast<const uint32_t *>(b + q);
            } else {
                wa = wb = 0;                                                     // (padding bytes are zero: +0.0)
                for (uint32_t u = 0; u < 4 && q + u < k; ++u) { wa |= (uint32_t)a[q + u] << (8 * u); wb |= (uint32_t)b[q + u] << (8 * u); }
            }
            float va[4], vb[4];
            fp8x4_values<TA>(wa, va);
            fp8x4_values<TB>(wb, vb);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const double pd = (double)(va[u] * vb[u]);
                const double upper = (pd + SPLIT) - SPLIT;
                sum_hi += upper;
                sum_lo += pd - upper;
            }
        }
        const double finite_max = 0x1.fffffffffffffp+1023;
        bool bad = !(__builtin_fabs(sum_hi) <= finite_max) || !(__builtin_fabs(sum_lo) <= finite_max);
        const int64_t acc_hi = bad ? 0 : (int64_t)__builtin_ldexp(sum_hi, -(LSB0 + 32));
        const int64_t acc_lo = bad ? 0 : (int64_t)__builtin_ldexp(sum_lo, -LSB0);
        I128 acc = {(uint64_t)acc_lo, acc_lo < 0 ? -1ll : 0ll};
        acc = add128(acc, shl128(I128{(uint64_t)acc_hi, acc_hi < 0 ? -1ll : 0ll}, 32));
        // wavefront reduction of the two-limb sums
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            I128 o2;
            o2.lo = __shfl_xor((unsigned long long)acc.lo, off, 64);
            o2.hi = (int64_t)__shfl_xor((unsigned long long)acc.hi, off, 64);
            acc = add128(acc, o2);
            bad |= (bool)__shfl_xor((int)bad, off, 64);
        }
        if (lane == 0) {
        const uint32_t d = D[o];
        if (bad || (d & 0x7F800000u) == 0x7F800000u) {
            atomicAdd(&g[4], 1ull);
        } else {
        const uint32_t neg = acc.hi < 0;
        const I128 mg = neg ? neg128(acc) : acc;
        // RNE-FP32 of the exact value
        uint32_t r;
        if (mg.hi == 0 && mg.lo == 0) r = 0u;
        else if (mg.hi == 0) r = round_to_fp32(neg, mg.lo, LSB0, 0, MMAEMU_ROUND_RNE);
        else {
            // fold to 64 bits keeping a sticky bit: hi limb != 0 means >= 65 significant bits
            const int sh = 64 - __builtin_clzll((uint64_t)mg.hi);             // 1..63 bits to drop
            const uint64_t top = ((uint64_t)mg.hi << (64 - sh)) | (mg.lo >> sh);
            const uint32_t sticky = (mg.lo & ((1ull << sh) - 1ull)) != 0;
            r = round_to_fp32(neg, top, LSB0 + sh, sticky, MMAEMU_ROUND_RNE);
        }
        atomicAdd(&g[0], 1ull);
        if (d == r) atomicAdd(&g[1], 1ull);
        const int64_t kd = okey(d), kr = okey(r);
        if (kd > kr) atomicAdd(&g[2], 1ull);
        else if (kd < kr) atomicAdd(&g[3], 1ull);
        const uint64_t dist = (uint64_t)(kd > kr ? kd - kr : kr - kd);
        atomicAdd(&g[5 + (dist ? 64 - __builtin_clzll(dist) : 0)], 1ull);
        // D - exact, formed exactly in integers at the finer of the two last places, then
        // converted to binary64
        const uint32_t dE = (d >> 23) & 0xFFu;
        const uint64_t dsig = (d & 0x7FFFFFu) | (dE ? 0x800000u : 0u);
        const int dl = (int)(dE ? dE : 1u) - 127 - 23;
        const int lo_exp = dl < LSB0 ? dl : LSB0;
        double err;
        if (dl - lo_exp <= 100 && LSB0 - lo_exp <= 20 && (mg.hi >> 40) == 0) {
            I128 dv = shl128(I128{dsig, 0}, dl - lo_exp);
            if (d >> 31) dv = neg128(dv);
            const I128 ev = shl128(acc, LSB0 - lo_exp);
            I128 df = add128(dv, neg128(ev));
            const uint32_t eneg = df.hi < 0;
            const I128 dm = eneg ? neg128(df) : df;
            err = mag_to_double((uint64_t)dm.hi, dm.lo, lo_exp);
            if (eneg) err = -err;
        } else {
            // far-apart magnitudes (D wildly off): plain binary64 difference
            const double dv = (d >> 31 ? -1.0 : 1.0) * ldexp((double)dsig, dl);
            const double ev = (neg ? -1.0 : 1.0) * mag_to_double((uint64_t)mg.hi, mg.lo, LSB0);
            err = dv - ev;
        }
        const double ae = err < 0 ? -err : err;
        atomicAdd(&gd[0], ae);
        atomicMax(reinterpret_cast<unsigned long long *>(&gd[1]), (unsigned long long)__double_as_longlong(ae));
        atomicAdd(&gd[4], err);
        if (mg.hi != 0 || mg.lo != 0) {
            const double rel = ae / mag_to_double((uint64_t)mg.hi, mg.lo, LSB0);
            atomicAdd(&gd[2], rel);
            atomicMax(reinterpret_cast<unsigned long long *>(&gd[3]), (unsigned long long)__double_as_longlong(rel));
        }
        }   // finite sample
        }   // lane 0
    }
    __syncthreads();
    if (threadIdx.x < NW && ls[threadIdx.x] != 0ull) {
        unsigned long long *out = reinterpret_cast<unsigned long long *>(st) + threadIdx.x;
        const int w = (int)threadIdx.x - (5 + 34);                 // index among the binary64 fields
        if (w < 0) atomicAdd(out, ls[threadIdx.x]);
        else if (w == 1 || w == 3) atomicMax(out, ls[threadIdx.x]);             // maxima of non-negative doubles
        else atomicAdd(reinterpret_cast<double *>(out), __longlong_as_double((long long)ls[threadIdx.x]));
    }
}

mmaemu_status launch_err_stats_reset(mmaemu_err_stats *st, hipStream_t s)
{
    hipLaunchKernelGGL(err_stats_reset_kernel, dim3(1), dim3(64), 0, s, st);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

template <int TA, int TB>
static mmaemu_status launch_t(const void *A, const void *B, const uint32_t *D, uint32_t m, uint32_t n, uint32_t k,
                              uint64_t stride, mmaemu_err_stats *st, hipStream_t s)
{
    const uint64_t total = (uint64_t)m * n;
    const uint64_t nsamples = (total + stride - 1) / stride;
    uint64_t blocks = (nsamples + 3) / 4;
    if (blocks > 1024) blocks = 1024;                      // wave-stride beyond that
    hipLaunchKernelGGL((exact_dot_kernel<TA, TB>), dim3((uint32_t)blocks), dim3(256), 0, s, (const uint8_t *)A,
                       (const uint8_t *)B, D, m, n, k, stride, nsamples, st);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

mmaemu_status launch_exact_dot_sample(const void *A, const void *B, const uint32_t *D, uint32_t m, uint32_t n,
                                      uint32_t k, uint32_t ta, uint32_t tb, uint64_t stride,
                                      mmaemu_err_stats *st, hipStream_t s)
{
#define CASE(X, Y) if (ta == X && tb == Y) return launch_t<X, Y>(A, B, D, m, n, k, stride, st, s)
    CASE(MMAEMU_FP8_E4M3, MMAEMU_FP8_E4M3); CASE(MMAEMU_FP8_E4M3, MMAEMU_FP8_E5M2);
    CASE(MMAEMU_FP8_E5M2, MMAEMU_FP8_E4M3); CASE(MMAEMU_FP8_E5M2, MMAEMU_FP8_E5M2);
#undef CASE
    set_error("exact_dot_sample: operands must be FP8 (got a=%u b=%u)", ta, tb);
    return MMAEMU_ERR_UNSUPPORTED;
}

} // namespace mmaemu
