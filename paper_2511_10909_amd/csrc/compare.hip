// Bitwise comparison of two FP32 (or two FP16) outputs with mismatch statistics (paper Eq. 2 and
// Sec. 3.1 Step 4: the model must reproduce the interface bit by bit).
//
// HBM-bound: 8 (4) bytes read per compared pair.  Each lane handles four (eight) consecutive
// elements (one 128-bit load per input).  The histogram is kept in LDS in 32 copies per
// bucket (copy = lane mod 32), so that lanes counting the same bucket do not serialise
// on one address; counters are flushed with one global atomic per non-zero counter per
// workgroup.
#include "common.hpp"

namespace mmaemu {

__global__ void stats_reset_kernel(mmaemu_stats *st)
{
    uint64_t *w = reinterpret_cast<uint64_t *>(st);
    const uint32_t i = threadIdx.x;
    if (i < sizeof(mmaemu_stats) / 8) w[i] = (i == 3) ? ~0ull : 0ull;   // word 3: first_mismatch_index
}

// W = 32: binary32 patterns; W = 16: binary16 patterns (widened to 32 bits by the caller of one_pair)
template <int W> __device__ __forceinline__ int64_t ordered_key(uint32_t b)
{
    constexpr uint32_t SIGN = 1u << (W - 1);
    return (b & SIGN) ? -(int64_t)(b & (SIGN - 1u)) : (int64_t)b;
}

struct Local {
    uint32_t mism, nan_equiv;
    uint64_t first, maxd;
};

template <int W>
__device__ __forceinline__ void one_pair(uint32_t x, uint32_t y, uint64_t idx, Local &lc, uint32_t *hist)
{
    constexpr uint32_t MAG = (1u << (W - 1)) - 1u, INF = W == 32 ? 0x7F800000u : 0x7C00u;
    const bool nx = (x & MAG) > INF, ny = (y & MAG) > INF;
    uint32_t bucket;
    if (x != y) {
        lc.mism += 1;
        lc.first = idx < lc.first ? idx : lc.first;
    }
    if (nx || ny) {
        bucket = (nx && ny) ? 0u : 33u;
        if (nx && ny && x != y) lc.nan_equiv += 1;
    } else {
        const int64_t kx = ordered_key<W>(x), ky = ordered_key<W>(y);
        const uint64_t dist = (uint64_t)(kx > ky ? kx - ky : ky - kx);
        lc.maxd = dist > lc.maxd ? dist : lc.maxd;
        bucket = dist ? 64u - (uint32_t)__builtin_clzll(dist) : 0u;
    }
    if (bucket) atomicAdd(&hist[bucket * 32u + (threadIdx.x & 31u)], 1u);   // bucket 0 is derived from the total
}

// the 128 / W elements of one 128-bit load from each input, first element index i0
template <int W>
__device__ __forceinline__ void one_vector(const uint4 &x, const uint4 &y, uint64_t i0, Local &lc, uint32_t *hist)
{
    const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        if (W == 32) {
            one_pair<W>(xs[w], ys[w], i0 + w, lc, hist);
        } else {
            one_pair<W>(xs[w] & 0xFFFFu, ys[w] & 0xFFFFu, i0 + 2 * w, lc, hist);
            one_pair<W>(xs[w] >> 16, ys[w] >> 16, i0 + 2 * w + 1, lc, hist);
        }
    }
}

// per-workgroup state in LDS
struct WgStats {
    uint32_t hist[34 * 32];
    uint32_t mism, nan_equiv;
    unsigned long long first, maxd;
    uint32_t tot[34];
};

__device__ __forceinline__ void wg_init(WgStats &ws)
{
    for (uint32_t i = threadIdx.x; i < 34 * 32; i += blockDim.x) ws.hist[i] = 0;
    if (threadIdx.x == 0) { ws.mism = 0; ws.nan_equiv = 0; ws.first = ~0ull; ws.maxd = 0; }
    __syncthreads();
}

// lanes -> wavefront -> workgroup -> the caller's struct
__device__ __forceinline__ void wg_flush(WgStats &ws, Local lc, uint64_t count, mmaemu_stats *st)
{
    // one set of LDS atomics per wavefront, not per lane: 64 lanes on one address take 64 turns
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        lc.mism += __shfl_xor(lc.mism, o);
        lc.nan_equiv += __shfl_xor(lc.nan_equiv, o);
        const unsigned long long f = __shfl_xor((unsigned long long)lc.first, o), d = __shfl_xor((unsigned long long)lc.maxd, o);
        lc.first = f < lc.first ? f : lc.first;
        lc.maxd = d > lc.maxd ? d : lc.maxd;
    }
    if ((threadIdx.x & 63u) == 0) {
        if (lc.mism) {
            atomicAdd(&ws.mism, lc.mism);
            atomicMin(&ws.first, (unsigned long long)lc.first);
        }
        if (lc.nan_equiv) atomicAdd(&ws.nan_equiv, lc.nan_equiv);
        if (lc.maxd) atomicMax(&ws.maxd, (unsigned long long)lc.maxd);
    }
    __syncthreads();

    unsigned long long *g = reinterpret_cast<unsigned long long *>(st);
    if (threadIdx.x < 34) {
        uint32_t t = 0;
        for (int cpy = 0; cpy < 32; ++cpy) t += ws.hist[threadIdx.x * 32 + cpy];
        ws.tot[threadIdx.x] = t;
        if (threadIdx.x >= 1 && t) atomicAdd(&g[5 + threadIdx.x], (unsigned long long)t);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t nonzero = 0;
        for (int b = 1; b < 34; ++b) nonzero += ws.tot[b];
        // n_compared and bucket 0 are known up front: workgroup 0 adds the whole count once,
        // every workgroup takes its non-zero buckets back out of bucket 0 (sums are modular,
        // so the order does not matter); equal inputs then cost no further atomics at all
        if (blockIdx.x == 0) {
            atomicAdd(&g[0], (unsigned long long)count);
            atomicAdd(&g[5 + 0], (unsigned long long)count);
        }
        if (nonzero) atomicAdd(&g[5 + 0], 0ull - (unsigned long long)nonzero);
        if (ws.mism) {
            atomicAdd(&g[1], (unsigned long long)ws.mism);
            atomicMin(&g[3], ws.first);
        }
        if (ws.nan_equiv) atomicAdd(&g[2], (unsigned long long)ws.nan_equiv);
        if (ws.maxd) atomicMax(&g[4], ws.maxd);
    }
}

template <int W, typename T>
__global__ void __launch_bounds__(1024)
compare_kernel(const T *__restrict__ d0, const T *__restrict__ d1, uint64_t count, uint64_t base, mmaemu_stats *st)
{
    constexpr uint32_t EPV = 128 / W;                    // elements per 128-bit load
    __shared__ WgStats ws;
    wg_init(ws);
    uint32_t *hist = ws.hist;

    Local lc = {0, 0, ~0ull, 0};
    const uint64_t nvec = count / EPV;
    const bool aligned = ((reinterpret_cast<uintptr_t>(d0) | reinterpret_cast<uintptr_t>(d1)) & 15) == 0;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    if (aligned) {
        const uint4 *v0 = reinterpret_cast<const uint4 *>(d0), *v1 = reinterpret_cast<const uint4 *>(d1);
        uint64_t v = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
        for (; v + stride < nvec; v += 2 * stride) {               // two independent 128-bit loads per input in flight
            const uint4 x0 = v0[v], y0 = v1[v], x1 = v0[v + stride], y1 = v1[v + stride];
            one_vector<W>(x0, y0, base + EPV * v, lc, hist);
            one_vector<W>(x1, y1, base + EPV * (v + stride), lc, hist);
        }
        for (; v < nvec; v += stride) one_vector<W>(v0[v], v1[v], base + EPV * v, lc, hist);
        for (uint64_t i = EPV * nvec + (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride)
            one_pair<W>(d0[i], d1[i], base + i, lc, hist);
    } else {
        for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride)
            one_pair<W>(d0[i], d1[i], base + i, lc, hist);
    }
    wg_flush(ws, lc, count, st);
}

// binary64 patterns: the same statistics; the ordered distance can take 64 bits, and the last distance bucket (32) also
// holds everything from 2^32 upward
__device__ __forceinline__ void one_pair64(uint64_t x, uint64_t y, uint64_t idx, Local &lc, uint32_t *hist)
{
    constexpr uint64_t MAG = 0x7FFFFFFFFFFFFFFFull, INF = 0x7FF0000000000000ull;
    const bool nx = (x & MAG) > INF, ny = (y & MAG) > INF;
    uint32_t bucket;
    if (x != y) {
        lc.mism += 1;
        lc.first = idx < lc.first ? idx : lc.first;
    }
    if (nx || ny) {
        bucket = (nx && ny) ? 0u : 33u;
        if (nx && ny && x != y) lc.nan_equiv += 1;
    } else {
        // |key(x) - key(y)| without leaving 64 bits: same sign: difference of the magnitudes; else their sum (< 2^64)
        const uint64_t ax = x & MAG, ay = y & MAG;
        const uint64_t dist = ((x ^ y) >> 63) ? ax + ay : (ax > ay ? ax - ay : ay - ax);
        lc.maxd = dist > lc.maxd ? dist : lc.maxd;
        const uint32_t bl = dist ? 64u - (uint32_t)__builtin_clzll(dist) : 0u;
        bucket = bl > 32u ? 32u : bl;
    }
    if (bucket) atomicAdd(&hist[bucket * 32u + (threadIdx.x & 31u)], 1u);
}

__global__ void __launch_bounds__(1024)
compare64_kernel(const uint64_t *__restrict__ d0, const uint64_t *__restrict__ d1, uint64_t count, uint64_t base, mmaemu_stats *st)
{
    __shared__ WgStats ws;
    wg_init(ws);
    Local lc = {0, 0, ~0ull, 0};
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    const uint64_t nvec = count / 2;
    if (((reinterpret_cast<uintptr_t>(d0) | reinterpret_cast<uintptr_t>(d1)) & 15) == 0) {
        const ulonglong2 *v0 = reinterpret_cast<const ulonglong2 *>(d0), *v1 = reinterpret_cast<const ulonglong2 *>(d1);
        for (uint64_t v = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; v < nvec; v += stride) {
            const ulonglong2 x = v0[v], y = v1[v];
            one_pair64(x.x, y.x, base + 2 * v, lc, ws.hist);
            one_pair64(x.y, y.y, base + 2 * v + 1, lc, ws.hist);
        }
        if ((count & 1) && blockIdx.x == 0 && threadIdx.x == 0) one_pair64(d0[count - 1], d1[count - 1], base + count - 1, lc, ws.hist);
    } else {
        for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) one_pair64(d0[i], d1[i], base + i, lc, ws.hist);
    }
    wg_flush(ws, lc, count, st);
}

mmaemu_status launch_stats_reset(mmaemu_stats *st, hipStream_t s)
{
    hipLaunchKernelGGL(stats_reset_kernel, dim3(1), dim3(64), 0, s, st);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

mmaemu_status launch_compare64(const void *d0, const void *d1, uint64_t count, uint64_t base, mmaemu_stats *st, hipStream_t s)
{
    uint64_t blocks = (count + 16383) / 16384;
    blocks = blocks < 1 ? 1 : (blocks > 256 ? 256 : blocks);
    hipLaunchKernelGGL(compare64_kernel, dim3((uint32_t)blocks), dim3(1024), 0, s, (const uint64_t *)d0, (const uint64_t *)d1, count, base, st);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

mmaemu_status launch_compare(const void *d0, const void *d1, uint64_t count, uint64_t base, bool half,
                             mmaemu_stats *st, hipStream_t s)
{
    // Few, fat workgroups: every workgroup ends with up to ~40 global atomics on the same
    // few addresses, and those serialise across the chip (measured: ~40-80 ns per workgroup), so a
    // workgroup covers at least 16K pairs before it pays for them; 1024 threads each, so that a
    // workgroup has 16 waves' worth of loads in flight (a small comparison is latency-bound).  One workgroup per CU at
    // most: with two, equal inputs stream 4 % faster, but inputs that differ pay twice the atomics (2^24 pairs: 40 us
    // against 46 us), and the closed-loop workloads compare mostly differing outputs.
    uint64_t blocks = (count + 16383) / 16384;
    if (blocks < 1) blocks = 1;
    if (blocks > 256) blocks = 256;
    if (half)
        hipLaunchKernelGGL((compare_kernel<16, uint16_t>), dim3((uint32_t)blocks), dim3(1024), 0, s, (const uint16_t *)d0,
                           (const uint16_t *)d1, count, base, st);
    else
        hipLaunchKernelGGL((compare_kernel<32, uint32_t>), dim3((uint32_t)blocks), dim3(1024), 0, s, (const uint32_t *)d0,
                           (const uint32_t *)d1, count, base, st);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

} // namespace mmaemu
