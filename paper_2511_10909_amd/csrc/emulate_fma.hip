// The model built from the standard fused multiply-add (paper Sec. 4.1.2): Algorithm "Phi_FMA" around Algorithm
// "FMA", binary32 operands and accumulators.  One thread per output element runs the chain d <- FMA(a_k, b_k, d) in
// k order.
//
// The device's v_fma_f32 is IEEE-754's fusedMultiplyAdd (a b + d exact, one rounding to nearest-even, gradual
// underflow, the standard's signs of zero; this library is compiled with binary32 subnormals kept), which is the
// operation Algorithm "FMA" states, so each step is one instruction.  What the instruction leaves open is the NaN it
// returns: whenever a step's result is a NaN the model's own rule replaces it (Sec. 4.2: one pattern nan_bits, or the
// payload rule of the nan_propagate variation).
//
// HBM-bound on instruction-shaped tiles: a 16x16x4 tile reads 1.5 KiB and writes 1 KiB for 1024 terms (those keep several
// blocks in flight per thread).  Mid-sized
// problems are walked in 16x16 blocks of D so that a wavefront shares 4 rows of A and 16 rows of B in the caches; large
// ones (m, n multiples of 64, k of 16 and at least 64) take the LDS-tiled kernel below.
#include "common.hpp"

namespace mmaemu {

__device__ __forceinline__ bool is_nan32(uint32_t b) { return (b & 0x7FFFFFFFu) > 0x7F800000u; }
__device__ __forceinline__ bool is_inf32(uint32_t b) { return (b & 0x7FFFFFFFu) == 0x7F800000u; }
__device__ __forceinline__ bool is_zero32(uint32_t b) { return (b & 0x7FFFFFFFu) == 0u; }

template <bool PROPAGATE>
__device__ __forceinline__ uint32_t fma_step(uint32_t x, uint32_t y, uint32_t d, uint32_t nan_bits)
{
    uint32_t r = __float_as_uint(__builtin_fmaf(__uint_as_float(x), __uint_as_float(y), __uint_as_float(d)));
    if (is_nan32(r)) {                       // a NaN operand, infinity times zero, or infinities of both signs
        r = nan_bits;
        if (PROPAGATE) {
            if (is_nan32(x)) r = x | 0x00400000u;
            else if (is_nan32(y)) r = y | 0x00400000u;
            else if ((is_inf32(x) && is_zero32(y)) || (is_inf32(y) && is_zero32(x))) r = nan_bits;
            else if (is_nan32(d)) r = d | 0x00400000u;
        }
    }
    return r;
}

// BLOCKED: m and n are multiples of 16 and a workgroup owns one 16x16 block of D; otherwise outputs are taken in
// row-major order, 256 per workgroup.  VEC = 4 (2): k is a multiple of 4 (2) and the rows of A and B are 16-byte (8-byte)
// aligned, so that four (two) consecutive k come with one load.
template <bool PROPAGATE, bool BLOCKED, int VEC>
__global__ void __launch_bounds__(256)
emulate_fma_kernel(const uint32_t *__restrict__ A, const uint32_t *__restrict__ B, const uint32_t *C, uint32_t *D, uint32_t m,
                   uint32_t n, uint32_t k, uint64_t total, uint64_t nblocks, uint32_t nan_bits)
{
    const uint64_t mn = (uint64_t)m * n;
    for (uint64_t w = blockIdx.x; w < nblocks; w += gridDim.x) {
        uint64_t t;
        uint32_t i, j;
        if (BLOCKED) {
            const uint32_t bpr = n / 16u;
            const uint64_t bpt = (uint64_t)(m / 16u) * bpr;
            t = w / bpt;
            const uint32_t r = (uint32_t)(w - t * bpt);
            i = 16u * (r / bpr) + threadIdx.x / 16u;
            j = 16u * (r % bpr) + threadIdx.x % 16u;
        } else {
            const uint64_t o = w * 256u + threadIdx.x;
            if (o >= total) continue;
            t = o / mn;
            const uint32_t r = (uint32_t)(o - t * mn);
            i = r / n;
            j = r - i * n;
        }
        const uint64_t o = t * mn + (uint64_t)i * n + j;
        const uint32_t *a = A + (t * m + i) * (uint64_t)k;
        const uint32_t *b = B + (t * n + j) * (uint64_t)k;
        uint32_t d = C[o];
        if (VEC == 4) {
            for (uint32_t k0 = 0; k0 < k; k0 += 4) {
                const uint4 x = *reinterpret_cast<const uint4 *>(a + k0), y = *reinterpret_cast<const uint4 *>(b + k0);
                d = fma_step<PROPAGATE>(x.x, y.x, d, nan_bits);
                d = fma_step<PROPAGATE>(x.y, y.y, d, nan_bits);
                d = fma_step<PROPAGATE>(x.z, y.z, d, nan_bits);
                d = fma_step<PROPAGATE>(x.w, y.w, d, nan_bits);
            }
        } else if (VEC == 2) {
            for (uint32_t k0 = 0; k0 < k; k0 += 2) {
                const uint2 x = *reinterpret_cast<const uint2 *>(a + k0), y = *reinterpret_cast<const uint2 *>(b + k0);
                d = fma_step<PROPAGATE>(x.x, y.x, d, nan_bits);
                d = fma_step<PROPAGATE>(x.y, y.y, d, nan_bits);
            }
        } else {
            for (uint32_t kk = 0; kk < k; ++kk) d = fma_step<PROPAGATE>(a[kk], b[kk], d, nan_bits);
        }
        D[o] = d;
    }
}

// Instruction-shaped tiles (k of 2 or 4, a row one 8- or 16-byte load): the same walk in 16x16 blocks with U blocks in
// flight per thread, their loads issued together.  The kernel is bound by memory latency, not by arithmetic: one block at a
// time left it at 0.45 of the HBM peak.
template <bool PROPAGATE, int VEC, int U>
__global__ void __launch_bounds__(256)
emulate_fma_short_kernel(const uint32_t *__restrict__ A, const uint32_t *__restrict__ B, const uint32_t *C, uint32_t *D, uint32_t m,
                         uint32_t n, uint64_t nblocks, uint32_t nan_bits)
{
    typedef typename std::conditional<VEC == 4, uint4, uint2>::type Row;          // (k = VEC)
    const uint64_t mn = (uint64_t)m * n;
    const uint32_t bpr = n / 16u;
    const uint64_t bpt = (uint64_t)(m / 16u) * bpr;
    for (uint64_t w0 = (uint64_t)blockIdx.x * U; w0 < nblocks; w0 += (uint64_t)gridDim.x * U) {
        uint64_t o[U];
        Row x[U], y[U];
        uint32_t d[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint64_t w = w0 + u;
            w = w < nblocks ? w : nblocks - 1;                                    // (surplus slots repeat the last block and store nothing)
            const uint64_t t = w / bpt;
            const uint32_t r = (uint32_t)(w - t * bpt);
            const uint32_t i = 16u * (r / bpr) + threadIdx.x / 16u, j = 16u * (r % bpr) + threadIdx.x % 16u;
            o[u] = t * mn + (uint64_t)i * n + j;
            x[u] = *reinterpret_cast<const Row *>(A + (t * m + i) * (uint64_t)VEC);
            y[u] = *reinterpret_cast<const Row *>(B + (t * n + j) * (uint64_t)VEC);
            d[u] = C[o[u]];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            d[u] = fma_step<PROPAGATE>(x[u].x, y[u].x, d[u], nan_bits);
            d[u] = fma_step<PROPAGATE>(x[u].y, y[u].y, d[u], nan_bits);
            if constexpr (VEC == 4) {
                d[u] = fma_step<PROPAGATE>(x[u].z, y[u].z, d[u], nan_bits);
                d[u] = fma_step<PROPAGATE>(x[u].w, y[u].w, d[u], nan_bits);
            }
            if (w0 + u < nblocks) D[o[u]] = d[u];
        }
    }
}

// Large problems: a workgroup owns a 64 x 64 (NT = 1) or 128 x 128 (NT = 2) block of D, a thread NT x NT sub-blocks of
// 4 x 4 outputs, 64 apart; A and B go through LDS sixteen k at a time, transposed so that a thread reads four rows
// (columns) with one 128-bit load.  Every output still runs its own chain d <- fma(a_k, b_k, d) in k order.  A NaN is
// sticky in such a chain, so the loop carries no test: an output that ends as a NaN is the model's one pattern, or, under
// the payload rule (where the step that produced it matters), is run again step by step from global memory.  m and n
// multiples of the block, k of 16, rows 16-byte aligned.
constexpr int FK = 16, FPAD = 4;

template <bool PROPAGATE, int NT>
__global__ void __launch_bounds__(256)
emulate_fma_tiled_kernel(const uint32_t *__restrict__ A, const uint32_t *__restrict__ B, const uint32_t *C, uint32_t *D, uint32_t m,
                         uint32_t n, uint32_t k, uint32_t nan_bits)
{
    constexpr int FT = 64 * NT;
    __shared__ __attribute__((aligned(16))) float As[FK][FT + FPAD];
    __shared__ __attribute__((aligned(16))) float Bs[FK][FT + FPAD];
    const uint32_t bn = n / FT, bpt = (m / FT) * bn;
    const uint32_t t = blockIdx.x / bpt, r0 = blockIdx.x % bpt;
    const uint32_t i0 = FT * (r0 / bn), j0 = FT * (r0 % bn);
    const uint32_t tid = threadIdx.x, ty = tid / 16u, tx = tid % 16u;
    const uint32_t lrow = tid / 4u, lk = 4u * (tid % 4u);                    // this thread's part of a staged panel (+ 64 q)
    const uint32_t *a_src = A + ((uint64_t)t * m + i0 + lrow) * k + lk;
    const uint32_t *b_src = B + ((uint64_t)t * n + j0 + lrow) * k + lk;
    // output (hr, r, hc, c): row i0 + 64 hr + 4 ty + r, column j0 + 64 hc + 4 tx + c
    const uint64_t d0 = ((uint64_t)t * m + i0 + 4u * ty) * n + j0 + 4u * tx;

    float acc[NT][4][NT][4];
#pragma unroll
    for (int hr = 0; hr < NT; ++hr)
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int hc = 0; hc < NT; ++hc) {
                const uint4 c4 = *reinterpret_cast<const uint4 *>(C + d0 + (uint64_t)(64 * hr + r) * n + 64 * hc);
                acc[hr][r][hc][0] = __uint_as_float(c4.x); acc[hr][r][hc][1] = __uint_as_float(c4.y);
                acc[hr][r][hc][2] = __uint_as_float(c4.z); acc[hr][r][hc][3] = __uint_as_float(c4.w);
            }
    uint4 pa[NT], pb[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        pa[q] = *reinterpret_cast<const uint4 *>(a_src + (uint64_t)(64 * q) * k);
        pb[q] = *reinterpret_cast<const uint4 *>(b_src + (uint64_t)(64 * q) * k);
    }
    for (uint32_t k0 = 0; k0 < k; k0 += FK) {
        __syncthreads();                                                     // the previous panel's readers are done
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            const uint32_t row = lrow + 64u * q;
            As[lk + 0][row] = __uint_as_float(pa[q].x); As[lk + 1][row] = __uint_as_float(pa[q].y);
            As[lk + 2][row] = __uint_as_float(pa[q].z); As[lk + 3][row] = __uint_as_float(pa[q].w);
            Bs[lk + 0][row] = __uint_as_float(pb[q].x); Bs[lk + 1][row] = __uint_as_float(pb[q].y);
            Bs[lk + 2][row] = __uint_as_float(pb[q].z); Bs[lk + 3][row] = __uint_as_float(pb[q].w);
        }
        __syncthreads();
        if (k0 + FK < k) {                                                   // next panel in flight during the arithmetic
#pragma unroll
            for (int q = 0; q < NT; ++q) {
                pa[q] = *reinterpret_cast<const uint4 *>(a_src + (uint64_t)(64 * q) * k + k0 + FK);
                pb[q] = *reinterpret_cast<const uint4 *>(b_src + (uint64_t)(64 * q) * k + k0 + FK);
            }
        }
#pragma unroll
        for (int kk = 0; kk < FK; ++kk) {
            float a[NT][4], b[NT][4];
#pragma unroll
            for (int h = 0; h < NT; ++h) {
                const float4 av = *reinterpret_cast<const float4 *>(&As[kk][64 * h + 4u * ty]);
                const float4 bv = *reinterpret_cast<const float4 *>(&Bs[kk][64 * h + 4u * tx]);
                a[h][0] = av.x; a[h][1] = av.y; a[h][2] = av.z; a[h][3] = av.w;
                b[h][0] = bv.x; b[h][1] = bv.y; b[h][2] = bv.z; b[h][3] = bv.w;
            }
#pragma unroll
            for (int hr = 0; hr < NT; ++hr)
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int hc = 0; hc < NT; ++hc)
#pragma unroll
                        for (int c = 0; c < 4; ++c) acc[hr][r][hc][c] = __builtin_fmaf(a[hr][r], b[hc][c], acc[hr][r][hc][c]);
        }
    }
#pragma unroll
    for (int hr = 0; hr < NT; ++hr)
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int hc = 0; hc < NT; ++hc) {
                const uint64_t o = d0 + (uint64_t)(64 * hr + r) * n + 64 * hc;
                uint32_t out[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    out[c] = __float_as_uint(acc[hr][r][hc][c]);
                    if (is_nan32(out[c])) {
                        out[c] = nan_bits;
                        if (PROPAGATE) {
                            const uint32_t *a = A + ((uint64_t)t * m + i0 + 64u * hr + 4u * ty + r) * k;
                            const uint32_t *b = B + ((uint64_t)t * n + j0 + 64u * hc + 4u * tx + c) * k;
                            uint32_t d = C[o + c];
                            for (uint32_t kk = 0; kk < k; ++kk) d = fma_step<true>(a[kk], b[kk], d, nan_bits);
                            out[c] = d;
                        }
                    }
                }
                *reinterpret_cast<uint4 *>(D + o) = make_uint4(out[0], out[1], out[2], out[3]);
            }
}

template <bool PROPAGATE, bool BLOCKED, int VEC>
static mmaemu_status launch_v(const void *A, const void *B, const void *C, void *D, uint32_t m, uint32_t n, uint32_t k,
                              uint64_t batch, uint32_t nan_bits, hipStream_t s)
{
    const uint64_t total = batch * m * n;
    const uint64_t nblocks = (total + 255) / 256;         // (blocked: total is a multiple of 256)
    const uint64_t grid = nblocks < 16384 ? nblocks : 16384;             // (grid-stride beyond that)
    hipLaunchKernelGGL((emulate_fma_kernel<PROPAGATE, BLOCKED, VEC>), dim3((uint32_t)grid), dim3(256), 0, s, (const uint32_t *)A,
                       (const uint32_t *)B, (const uint32_t *)C, (uint32_t *)D, m, n, k, total, nblocks, nan_bits);
    MMAEMU_HIP(hipGetLastError());
    set_last_kernel("fma chain%s%s%s", PROPAGATE ? ", payloads" : "", BLOCKED ? ", 16x16 blocks" : "",
                    VEC == 4 ? ", 128-bit loads" : (VEC == 2 ? ", 64-bit loads" : ""));
    return MMAEMU_OK;
}

template <bool PROPAGATE>
static mmaemu_status launch_p(const void *A, const void *B, const void *C, void *D, uint32_t m, uint32_t n, uint32_t k,
                              uint64_t batch, uint32_t nan_bits, hipStream_t s)
{
    const bool blocked = m % 16 == 0 && n % 16 == 0;
    const uintptr_t addr = reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B);
    const uintptr_t addr_cd = reinterpret_cast<uintptr_t>(C) | reinterpret_cast<uintptr_t>(D);
    if (m % 64 == 0 && n % 64 == 0 && k % FK == 0 && k >= 4 * FK && ((addr | addr_cd) & 15) == 0) {
        // (D may alias C: a thread reads exactly the elements of C it later writes)
        const uint64_t tiles64 = batch * (m / 64) * (n / 64), tiles128 = batch * (m / 128) * (n / 128);
        if (m % 128 == 0 && n % 128 == 0 && tiles128 >= 512 && tiles128 <= 0x7FFFFFFFull) {      // two workgroups per CU and more
            hipLaunchKernelGGL((emulate_fma_tiled_kernel<PROPAGATE, 2>), dim3((uint32_t)tiles128), dim3(256), 0, s, (const uint32_t *)A,
                               (const uint32_t *)B, (const uint32_t *)C, (uint32_t *)D, m, n, k, nan_bits);
            MMAEMU_HIP(hipGetLastError());
            set_last_kernel("fma chain%s, 128x128 blocks through LDS", PROPAGATE ? ", payloads" : "");
            return MMAEMU_OK;
        }
        if (tiles64 <= 0x7FFFFFFFull) {
            hipLaunchKernelGGL((emulate_fma_tiled_kernel<PROPAGATE, 1>), dim3((uint32_t)tiles64), dim3(256), 0, s, (const uint32_t *)A,
                               (const uint32_t *)B, (const uint32_t *)C, (uint32_t *)D, m, n, k, nan_bits);
            MMAEMU_HIP(hipGetLastError());
            set_last_kernel("fma chain%s, 64x64 blocks through LDS", PROPAGATE ? ", payloads" : "");
            return MMAEMU_OK;
        }
    }
    const int vec = (k % 4 == 0 && (addr & 15) == 0) ? 4 : ((k % 2 == 0 && (addr & 7) == 0) ? 2 : 1);
    if (blocked && (int)k == vec && vec >= 2) {
        // (D may alias C here too: a thread reads exactly the elements of C it later writes)
        constexpr int U = 4;
        const uint64_t nblocks = batch * (m / 16) * (n / 16), groups = (nblocks + U - 1) / U;
        const uint32_t grid = (uint32_t)(groups < 16384 ? groups : 16384);
        if (vec == 4)
            hipLaunchKernelGGL((emulate_fma_short_kernel<PROPAGATE, 4, U>), dim3(grid), dim3(256), 0, s, (const uint32_t *)A, (const uint32_t *)B,
                               (const uint32_t *)C, (uint32_t *)D, m, n, nblocks, nan_bits);
        else
            hipLaunchKernelGGL((emulate_fma_short_kernel<PROPAGATE, 2, U>), dim3(grid), dim3(256), 0, s, (const uint32_t *)A, (const uint32_t *)B,
                               (const uint32_t *)C, (uint32_t *)D, m, n, nblocks, nan_bits);
        MMAEMU_HIP(hipGetLastError());
        set_last_kernel("fma chain%s, 16x16 blocks, %d-bit loads, %d blocks in flight", PROPAGATE ? ", payloads" : "", vec * 32, U);
        return MMAEMU_OK;
    }
    if (blocked) {
        if (vec == 4) return launch_v<PROPAGATE, true, 4>(A, B, C, D, m, n, k, batch, nan_bits, s);
        if (vec == 2) return launch_v<PROPAGATE, true, 2>(A, B, C, D, m, n, k, batch, nan_bits, s);
        return launch_v<PROPAGATE, true, 1>(A, B, C, D, m, n, k, batch, nan_bits, s);
    }
    if (vec == 4) return launch_v<PROPAGATE, false, 4>(A, B, C, D, m, n, k, batch, nan_bits, s);
    if (vec == 2) return launch_v<PROPAGATE, false, 2>(A, B, C, D, m, n, k, batch, nan_bits, s);
    return launch_v<PROPAGATE, false, 1>(A, B, C, D, m, n, k, batch, nan_bits, s);
}

// ---- binary64 (Algorithms "FMA" / "Phi_FMA" with F = FP64) ----------------------------------------------------------------
// v_fma_f64 is the standard's operation on binary64 (subnormals always kept), so a step is again one instruction plus the
// model's NaN rule.  The model's NaN pattern is a binary32 word; here it is widened the way a conversion between the
// formats widens a NaN: sign, exponent field all ones, the 23 mantissa bits at the top of the 52.
__device__ __forceinline__ bool is_nan64(uint64_t b) { return (b & 0x7FFFFFFFFFFFFFFFull) > 0x7FF0000000000000ull; }
__device__ __forceinline__ bool is_inf64(uint64_t b) { return (b & 0x7FFFFFFFFFFFFFFFull) == 0x7FF0000000000000ull; }
__device__ __forceinline__ bool is_zero64(uint64_t b) { return (b & 0x7FFFFFFFFFFFFFFFull) == 0ull; }

template <bool PROPAGATE>
__device__ __forceinline__ uint64_t fma_step64(uint64_t x, uint64_t y, uint64_t d, uint64_t nan64)
{
    uint64_t r = (uint64_t)__double_as_longlong(__builtin_fma(__longlong_as_double((long long)x), __longlong_as_double((long long)y),
                                                              __longlong_as_double((long long)d)));
    if (is_nan64(r)) {
        r = nan64;
        if (PROPAGATE) {
            constexpr uint64_t QUIET = 1ull << 51;
            if (is_nan64(x)) r = x | QUIET;
            else if (is_nan64(y)) r = y | QUIET;
            else if ((is_inf64(x) && is_zero64(y)) || (is_inf64(y) && is_zero64(x))) r = nan64;
            else if (is_nan64(d)) r = d | QUIET;
        }
    }
    return r;
}

// One thread per output; a workgroup owns a 16x16 block of D when m and n allow (a wavefront then shares 4 rows of A and
// 16 of B), else 256 outputs in row-major order.  VEC2: k even and 16-byte aligned rows: two k per load.
template <bool PROPAGATE, bool BLOCKED, bool VEC2>
__global__ void __launch_bounds__(256)
emulate_fma64_kernel(const uint64_t *__restrict__ A, const uint64_t *__restrict__ B, const uint64_t *C, uint64_t *D, uint32_t m,
                     uint32_t n, uint32_t k, uint64_t total, uint64_t nblocks, uint64_t nan64)
{
    const uint64_t mn = (uint64_t)m * n;
    for (uint64_t w = blockIdx.x; w < nblocks; w += gridDim.x) {
        uint64_t t;
        uint32_t i, j;
        if (BLOCKED) {
            const uint32_t bpr = n / 16u;
            const uint64_t bpt = (uint64_t)(m / 16u) * bpr;
            t = w / bpt;
            const uint32_t r = (uint32_t)(w - t * bpt);
            i = 16u * (r / bpr) + threadIdx.x / 16u;
            j = 16u * (r % bpr) + threadIdx.x % 16u;
        } else {
            const uint64_t o = w * 256u + threadIdx.x;
            if (o >= total) continue;
            t = o / mn;
            const uint32_t r = (uint32_t)(o - t * mn);
            i = r / n;
            j = r - i * n;
        }
        const uint64_t o = t * mn + (uint64_t)i * n + j;
        const uint64_t *a = A + (t * m + i) * (uint64_t)k;
        const uint64_t *b = B + (t * n + j) * (uint64_t)k;
        uint64_t d = C[o];
        if (VEC2) {
            for (uint32_t k0 = 0; k0 < k; k0 += 2) {
                const ulonglong2 x = *reinterpret_cast<const ulonglong2 *>(a + k0), y = *reinterpret_cast<const ulonglong2 *>(b + k0);
                d = fma_step64<PROPAGATE>(x.x, y.x, d, nan64);
                d = fma_step64<PROPAGATE>(x.y, y.y, d, nan64);
            }
        } else {
            for (uint32_t kk = 0; kk < k; ++kk) d = fma_step64<PROPAGATE>(a[kk], b[kk], d, nan64);
        }
        D[o] = d;
    }
}

// k = 4 in 16x16 blocks (the shape of the binary64 instruction): U blocks in flight per thread, their loads issued together
template <bool PROPAGATE, int U>
__global__ void __launch_bounds__(256)
emulate_fma64_short_kernel(const uint64_t *__restrict__ A, const uint64_t *__restrict__ B, const uint64_t *C, uint64_t *D, uint32_t m,
                           uint32_t n, uint64_t nblocks, uint64_t nan64)
{
    const uint64_t mn = (uint64_t)m * n;
    const uint32_t bpr = n / 16u;
    const uint64_t bpt = (uint64_t)(m / 16u) * bpr;
    for (uint64_t w0 = (uint64_t)blockIdx.x * U; w0 < nblocks; w0 += (uint64_t)gridDim.x * U) {
        uint64_t o[U], d[U];
        ulonglong2 x0[U], x1[U], y0[U], y1[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint64_t w = w0 + u;
            w = w < nblocks ? w : nblocks - 1;                                    // (surplus slots repeat the last block and store nothing)
            const uint64_t t = w / bpt;
            const uint32_t r = (uint32_t)(w - t * bpt);
            const uint32_t i = 16u * (r / bpr) + threadIdx.x / 16u, j = 16u * (r % bpr) + threadIdx.x % 16u;
            o[u] = t * mn + (uint64_t)i * n + j;
            const ulonglong2 *a = reinterpret_cast<const ulonglong2 *>(A + (t * m + i) * 4ull);
            const ulonglong2 *b = reinterpret_cast<const ulonglong2 *>(B + (t * n + j) * 4ull);
            x0[u] = a[0]; x1[u] = a[1];
            y0[u] = b[0]; y1[u] = b[1];
            d[u] = C[o[u]];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            d[u] = fma_step64<PROPAGATE>(x0[u].x, y0[u].x, d[u], nan64);
            d[u] = fma_step64<PROPAGATE>(x0[u].y, y0[u].y, d[u], nan64);
            d[u] = fma_step64<PROPAGATE>(x1[u].x, y1[u].x, d[u], nan64);
            d[u] = fma_step64<PROPAGATE>(x1[u].y, y1[u].y, d[u], nan64);
            if (w0 + u < nblocks) D[o[u]] = d[u];
        }
    }
}

template <bool PROPAGATE, bool BLOCKED, bool VEC2>
static mmaemu_status launch64_v(const void *A, const void *B, const void *C, void *D, uint32_t m, uint32_t n, uint32_t k,
                                uint64_t batch, uint64_t nan64, hipStream_t s)
{
    const uint64_t total = batch * m * n;
    const uint64_t nblocks = (total + 255) / 256;
    const uint64_t grid = nblocks < 16384 ? nblocks : 16384;
    hipLaunchKernelGGL((emulate_fma64_kernel<PROPAGATE, BLOCKED, VEC2>), dim3((uint32_t)grid), dim3(256), 0, s, (const uint64_t *)A,
                       (const uint64_t *)B, (const uint64_t *)C, (uint64_t *)D, m, n, k, total, nblocks, nan64);
    MMAEMU_HIP(hipGetLastError());
    set_last_kernel("fma chain fp64%s%s%s", PROPAGATE ? ", payloads" : "", BLOCKED ? ", 16x16 blocks" : "", VEC2 ? ", 128-bit loads" : "");
    return MMAEMU_OK;
}

mmaemu_status launch_emulate_fma64(const void *A, const void *B, const void *C, void *D, uint32_t m, uint32_t n, uint32_t k,
                                   uint64_t batch, uint32_t nan_bits, bool nan_propagate, hipStream_t s)
{
    const uint64_t nan64 = ((uint64_t)(nan_bits >> 31) << 63) | 0x7FF0000000000000ull | ((uint64_t)(nan_bits & 0x7FFFFFu) << 29);
    const bool blocked = m % 16 == 0 && n % 16 == 0;
    const bool vec2 = k % 2 == 0 && ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 15) == 0;
    if (blocked && vec2 && k == 4) {
        constexpr int U = 4;
        const uint64_t nblocks = batch * (m / 16) * (n / 16), groups = (nblocks + U - 1) / U;
        const uint32_t grid = (uint32_t)(groups < 16384 ? groups : 16384);
        if (nan_propagate)
            hipLaunchKernelGGL((emulate_fma64_short_kernel<true, U>), dim3(grid), dim3(256), 0, s, (const uint64_t *)A, (const uint64_t *)B,
                               (const uint64_t *)C, (uint64_t *)D, m, n, nblocks, nan64);
        else
            hipLaunchKernelGGL((emulate_fma64_short_kernel<false, U>), dim3(grid), dim3(256), 0, s, (const uint64_t *)A, (const uint64_t *)B,
                               (const uint64_t *)C, (uint64_t *)D, m, n, nblocks, nan64);
        MMAEMU_HIP(hipGetLastError());
        set_last_kernel("fma chain fp64%s, 16x16 blocks, 128-bit loads, %d blocks in flight", nan_propagate ? ", payloads" : "", U);
        return MMAEMU_OK;
    }
#define GO(P, BL, V) return launch64_v<P, BL, V>(A, B, C, D, m, n, k, batch, nan64, s)
    if (nan_propagate) {
        if (blocked) { if (vec2) GO(true, true, true); GO(true, true, false); }
        if (vec2) GO(true, false, true);
        GO(true, false, false);
    }
    if (blocked) { if (vec2) GO(false, true, true); GO(false, true, false); }
    if (vec2) GO(false, false, true);
    GO(false, false, false);
#undef GO
}

mmaemu_status launch_emulate_fma(const void *A, const void *B, const void *C, void *D, uint32_t m, uint32_t n, uint32_t k,
                                 uint64_t batch, uint32_t nan_bits, bool nan_propagate, hipStream_t s)
{
    if (nan_propagate) return launch_p<true>(A, B, C, D, m, n, k, batch, nan_bits, s);
    return launch_p<false>(A, B, C, D, m, n, k, batch, nan_bits, s);
}

} // namespace mmaemu
