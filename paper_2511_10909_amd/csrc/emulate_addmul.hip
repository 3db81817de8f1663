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

// The same model with operand sharing: a workgroup owns 16 x 16 blocks of D (one output per thread), and the rows of A
// and B that a block needs are decoded and flushed once, into LDS, KC values of k at a time; every thread then reads
// its row and its column as 128-bit (64-bit for P = 2) LDS words.  A NaN stays a NaN through every later product and
// sum (the flush leaves it alone), so the model's NaN pattern is written once, at the end of the chain.
__device__ __forceinline__ float flush_tiny(float z)
{
    const uint32_t b = __float_as_uint(z);
    return __uint_as_float((b & 0x7F800000u) == 0 ? (b & 0x80000000u) : b);             // |z| < 2^-126: zero of the same sign
}

template <int TA, int TB, int P, int BM>
__global__ void __launch_bounds__(256)
emulate_addmul_blocks_kernel(uint32_t nan_bits, const typename Fmt<TA>::elem *__restrict__ A, const typename Fmt<TB>::elem *__restrict__ B,
                             const uint32_t *C, uint32_t *D, uint32_t m, uint32_t n, uint32_t k, uint64_t nblocks)
{
    constexpr int Q = BM / 16;                                    // Q x Q outputs per thread, 16 rows / columns apart
    constexpr int KC = 64, VS = KC + 4;                           // row stride: 16-byte aligned, rows spread over the banks
    __shared__ __attribute__((aligned(16))) float As[BM][VS];
    __shared__ __attribute__((aligned(16))) float Bs[BM][VS];
    const uint32_t tid = threadIdx.x, i = tid / 16u, j = tid % 16u;
    const uint32_t bpr = n / BM, bpt = (m / BM) * bpr;
    for (uint64_t w = blockIdx.x; w < nblocks; w += gridDim.x) {
        const uint64_t t = w / bpt;
        const uint32_t r = (uint32_t)(w - t * bpt), bi = r / bpr, bj = r - bi * bpr;
        const typename Fmt<TA>::elem *a0 = A + (t * m + (uint32_t)BM * bi) * (uint64_t)k;
        const typename Fmt<TB>::elem *b0 = B + (t * n + (uint32_t)BM * bj) * (uint64_t)k;
        const uint64_t o = (t * m + (uint32_t)BM * bi + i) * (uint64_t)n + (uint32_t)BM * bj + j;     // + 16 r n + 16 c
        float d[Q][Q];
#pragma unroll
        for (int rr = 0; rr < Q; ++rr)
#pragma unroll
            for (int cc = 0; cc < Q; ++cc) {
                uint32_t cb = C[o + (uint64_t)(16 * rr) * n + 16 * cc];
                if ((cb & 0x7F800000u) == 0) cb &= (cb & 0x007FFFFFu) ? 0u : 0x80000000u;     // subnormal accumulator -> +0.0
                d[rr][cc] = __uint_as_float(cb);
            }
        for (uint32_t k0 = 0; k0 < k; k0 += KC) {
            const uint32_t kc = k - k0 < (uint32_t)KC ? k - k0 : (uint32_t)KC;
            __syncthreads();                                      // (the previous chunk's readers)
            for (uint32_t e = tid; e < (uint32_t)BM * kc; e += 256u) {
                const uint32_t row = e / kc, kk = e - row * kc;
                As[row][kk] = flushed_operand<TA>(a0[(uint64_t)row * k + k0 + kk]);
                Bs[row][kk] = flushed_operand<TB>(b0[(uint64_t)row * k + k0 + kk]);
            }
            __syncthreads();
#pragma unroll 2
            for (uint32_t kk = 0; kk < kc; kk += P) {
                float x[Q][P], y[Q][P];
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    if (P == 4) {
                        const float4 xv = *reinterpret_cast<const float4 *>(&As[i + 16 * q][kk]), yv = *reinterpret_cast<const float4 *>(&Bs[j + 16 * q][kk]);
                        x[q][0] = xv.x; x[q][1] = xv.y; x[q][2 % P] = xv.z; x[q][3 % P] = xv.w;
                        y[q][0] = yv.x; y[q][1] = yv.y; y[q][2 % P] = yv.z; y[q][3 % P] = yv.w;
                    } else {
                        const float2 xv = *reinterpret_cast<const float2 *>(&As[i + 16 * q][kk]), yv = *reinterpret_cast<const float2 *>(&Bs[j + 16 * q][kk]);
                        x[q][0] = xv.x; x[q][1] = xv.y;
                        y[q][0] = yv.x; y[q][1] = yv.y;
                    }
                }
#pragma unroll
                for (int rr = 0; rr < Q; ++rr)
#pragma unroll
                    for (int cc = 0; cc < Q; ++cc) {
                        float p[P];
#pragma unroll
                        for (int l = 0; l < P; ++l) p[l] = flush_tiny(__fmul_rn(x[rr][l], y[cc][l]));
                        float s = flush_tiny(__fadd_rn(p[0], p[1]));
                        if (P == 4) {
                            const float s2 = flush_tiny(__fadd_rn(p[2 % P], p[3 % P]));
                            s = flush_tiny(__fadd_rn(s, s2));
                        }
                        d[rr][cc] = flush_tiny(__fadd_rn(d[rr][cc], s));
                    }
            }
        }
#pragma unroll
        for (int rr = 0; rr < Q; ++rr)
#pragma unroll
            for (int cc = 0; cc < Q; ++cc) {
                uint32_t out = __float_as_uint(d[rr][cc]);
                if ((out & 0x7FFFFFFFu) > 0x7F800000u) out = nan_bits;
                D[o + (uint64_t)(16 * rr) * n + 16 * cc] = out;
            }
    }
}

template <int TA, int TB, int P, int BM>
static mmaemu_status launch_blocks(const ModelArgs &p, const void *A, const void *B, const void *C, void *D, uint32_t m, uint32_t n, uint32_t k,
                                   uint64_t batch, hipStream_t s)
{
    const uint64_t nblocks = batch * (m / BM) * (n / BM);
    const uint64_t grid = nblocks < (1ull << 16) ? nblocks : (1ull << 16);
    hipLaunchKernelGGL((emulate_addmul_blocks_kernel<TA, TB, P, BM>), dim3((uint32_t)grid), dim3(256), 0, s, p.nan_bits, (const typename Fmt<TA>::elem *)A,
                       (const typename Fmt<TB>::elem *)B, (const uint32_t *)C, (uint32_t *)D, m, n, k, nblocks);
    MMAEMU_HIP(hipGetLastError());
    set_last_kernel("ftz-addmul P=%u, %dx%d blocks through LDS", p.L, BM, BM);
    return MMAEMU_OK;
}

template <int TA, int TB>
static mmaemu_status launch_t(const ModelArgs &p, const void *A, const void *B, const void *C, void *D,
                              uint32_t m, uint32_t n, uint32_t k, uint64_t batch, hipStream_t s)
{
    const uint64_t total = batch * m * n;
    if (m % 16 == 0 && n % 16 == 0 && (p.L == 2 || p.L == 4)) {
        const bool big = m % 32 == 0 && n % 32 == 0;
        if (p.L == 4) return big ? launch_blocks<TA, TB, 4, 32>(p, A, B, C, D, m, n, k, batch, s) : launch_blocks<TA, TB, 4, 16>(p, A, B, C, D, m, n, k, batch, s);
        return big ? launch_blocks<TA, TB, 2, 32>(p, A, B, C, D, m, n, k, batch, s) : launch_blocks<TA, TB, 2, 16>(p, A, B, C, D, m, n, k, batch, s);
    }
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
