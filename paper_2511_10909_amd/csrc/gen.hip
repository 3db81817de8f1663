// On-device operand generators (the input families of the paper's randomized validation,
// Sec. 3.1 Step 4).  Counter-based: every element's random words are a pure function of
// (seed, operand, global element index), so any range of tiles can be produced in place,
// in any order, on any number of devices.
//
// Random words: Philox-4x32-10 (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as
// easy as 1, 2, 3", SC'11), written from its published definition.
//
// This file must be compiled with floating-point contraction off: the NORMAL family is
// defined as a fixed sequence of IEEE-754 binary64 +, *, / operations, and a fused
// multiply-add anywhere would change the bits.
#include "common.hpp"

#include <mutex>

namespace mmaemu {

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4])
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        // (one 32 x 32 -> 64-bit multiply per product: both halves from one instruction)
        const uint64_t p0 = (uint64_t)M0 * c0, p1 = (uint64_t)M1 * c2;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        // (a ^ b ^ c in one instruction: v_bitop3_b32 with the truth table of the three-input exclusive or)
        c0 = __builtin_amdgcn_bitop3_b32(hi1, c1, k0, 0x96);
        c1 = lo1;
        c2 = __builtin_amdgcn_bitop3_b32(hi0, c3, k1, 0x96);
        c3 = lo0;
        k0 += W0;
        k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

struct GenArgs {
    uint32_t family, operand, k0, k1;
    uint32_t width, mbits, nmag;          // output format (width: bits of a code, sign on top); nmag = number of finite magnitudes
    uint32_t exp_lo, nchoices, exp_zero;  // UNIFORM_EXP
    uint32_t fp32_two_words;              // UNIFORM_EXP with FP32 output
    uint32_t bias, max_code;              // NORMAL: target format
    uint32_t dtype;
    uint32_t scale_scope;
    double scale_target;
};

__device__ __forceinline__ void block_words(const GenArgs &g, uint64_t blk, uint32_t w[4])
{
    philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), g.operand, 0u, g.k0, g.k1, w);
}

// ---- bit-pattern families ------------------------------------------------------------

__device__ __forceinline__ uint32_t bits_from_word(const GenArgs &g, uint32_t r, uint32_t r1)
{
    // (CANCELLING draws like UNIFORM_EXP; the pairing of even and odd elements is applied by the caller)
    if (g.family == MMAEMU_GEN_RANDOM_BITS) return g.width == 32 ? r : (r & ((1u << g.width) - 1u));
    if (g.family == MMAEMU_GEN_FINITE_BITS) {
        const uint32_t v = __umulhi(r, 2u * g.nmag);
        const uint32_t sign = v >= g.nmag;
        return (sign << (g.width - 1)) | (v - sign * g.nmag);
    }
    if (g.family == MMAEMU_GEN_SIGNED_ZEROS) {
        const uint32_t kind = r >> 30, sign = (r >> 29) & 1u;
        const uint32_t mag = kind == 2u ? (g.bias << g.mbits) : (kind == 3u ? 1u : 0u);
        return (sign << (g.width - 1)) | mag;
    }
    // UNIFORM_EXP (scale codes have no sign bit)
    const uint32_t sign = g.dtype == MMAEMU_E8M0 ? 0u : (r >> 31);
    uint32_t idx, mant;
    if (g.fp32_two_words) {
        idx = (uint32_t)(((uint64_t)(r & 0x7FFFFFFFu) * g.nchoices) >> 31);
        mant = r1 & 0x7FFFFFu;
    } else {
        const uint32_t nsel = 31u - g.mbits;
        const uint32_t sel = (r >> g.mbits) & ((1u << nsel) - 1u);
        idx = (uint32_t)(((uint64_t)sel * g.nchoices) >> nsel);
        mant = r & ((1u << g.mbits) - 1u);
    }
    const uint32_t E = g.exp_zero ? (idx == 0 ? 0u : g.exp_lo + idx - 1u) : g.exp_lo + idx;
    return (sign << (g.width - 1)) | (E << g.mbits) | mant;
}

template <typename T> __device__ __forceinline__ void store4(T *p, const uint32_t v[4]);
template <> __device__ __forceinline__ void store4<uint8_t>(uint8_t *p, const uint32_t v[4])
{
    *reinterpret_cast<uint32_t *>(p) = v[0] | (v[1] << 8) | (v[2] << 16) | (v[3] << 24);
}
template <> __device__ __forceinline__ void store4<uint16_t>(uint16_t *p, const uint32_t v[4])
{
    *reinterpret_cast<uint2 *>(p) = make_uint2(v[0] | (v[1] << 16), v[2] | (v[3] << 16));
}
template <> __device__ __forceinline__ void store4<uint32_t>(uint32_t *p, const uint32_t v[4])
{
    *reinterpret_cast<uint4 *>(p) = make_uint4(v[0], v[1], v[2], v[3]);
}

// elements [g0, g0 + total) of the operand; thread t owns Philox block blk0 + t
template <typename T>
__global__ void __launch_bounds__(256)
gen_bits_kernel(GenArgs g, T *out, uint64_t g0, uint64_t total, uint64_t blk0, uint64_t nblk)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nblk) return;
    const uint64_t blk = blk0 + t;
    uint32_t w[4];
    block_words(g, blk, w);
    if (g.fp32_two_words) {
#pragma unroll
        for (int j = 0; j < 4; j += 2) {
            const uint64_t e = (4 * blk + j) >> 1;
            if (e >= g0 && e - g0 < total) out[e - g0] = (T)bits_from_word(g, w[j], w[j + 1]);
        }
        return;
    }
    uint32_t v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = bits_from_word(g, w[j], 0u);
    if (g.family == MMAEMU_GEN_CANCELLING) {
        // element 2q+1 repeats element 2q (both live in this block): sign flipped for operand 0; for the other
        // operands the last mantissa bit is flipped where the odd element's own word ends in four zero bits
#pragma unroll
        for (int j = 1; j < 4; j += 2)
            v[j] = g.operand == 0 ? (v[j - 1] ^ (1u << (g.width - 1))) : (v[j - 1] ^ ((w[j] & 0xFu) == 0 ? 1u : 0u));
    }
    const uint64_t e0 = 4 * blk;
    if (e0 >= g0 && e0 + 4 <= g0 + total && ((reinterpret_cast<uintptr_t>(out + (e0 - g0)) & (4 * sizeof(T) - 1)) == 0)) {
        store4<T>(out + (e0 - g0), v);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint64_t e = e0 + j;
            if (e >= g0 && e - g0 < total) out[e - g0] = (T)v[j];
        }
    }
}

__global__ void zero_kernel(uint32_t *out, uint64_t nwords, uint8_t *tail, uint32_t ntail)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nwords; i += stride) out[i] = 0u;
    if (blockIdx.x == 0 && threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

// ---- NORMAL family --------------------------------------------------------------------
// binary64 elementary functions from +, *, / only, in a fixed order (the square root is IEEE-754's own operation)

__device__ __forceinline__ double ln_unit(uint32_t r)       // ln((r + 0.5) / 2^32)
{
    const double t = 2.0 * (double)r + 1.0;                 // odd integer < 2^33, exact
    const long long tb = __double_as_longlong(t);
    const int ex = (int)((tb >> 52) & 0x7FF) - 1023;        // t = m * 2^ex, m in [1, 2)
    const double m = __longlong_as_double((tb & 0x000FFFFFFFFFFFFFll) | 0x3FF0000000000000ll);
    const double s = (m - 1.0) / (m + 1.0);
    const double s2 = s * s;
    double poly = 1.0 / 25.0;
    poly = poly * s2 + 1.0 / 23.0;
    poly = poly * s2 + 1.0 / 21.0;
    poly = poly * s2 + 1.0 / 19.0;
    poly = poly * s2 + 1.0 / 17.0;
    poly = poly * s2 + 1.0 / 15.0;
    poly = poly * s2 + 1.0 / 13.0;
    poly = poly * s2 + 1.0 / 11.0;
    poly = poly * s2 + 1.0 / 9.0;
    poly = poly * s2 + 1.0 / 7.0;
    poly = poly * s2 + 1.0 / 5.0;
    poly = poly * s2 + 1.0 / 3.0;
    poly = poly * s2 + 1.0;
    const double lnm = (2.0 * s) * poly;
    return lnm + (double)(ex - 33) * 0x1.62e42fefa39efp-1;
}

__device__ __forceinline__ void sincos_quarter(double th, double &sn, double &cs)
{
    const double t2 = th * th;
    double ps = -1.0 / 121645100408832000.0;     // -1/19!
    ps = ps * t2 + 1.0 / 355687428096000.0;      // 17!
    ps = ps * t2 + -1.0 / 1307674368000.0;       // 15!
    ps = ps * t2 + 1.0 / 6227020800.0;           // 13!
    ps = ps * t2 + -1.0 / 39916800.0;            // 11!
    ps = ps * t2 + 1.0 / 362880.0;               // 9!
    ps = ps * t2 + -1.0 / 5040.0;                // 7!
    ps = ps * t2 + 1.0 / 120.0;                  // 5!
    ps = ps * t2 + -1.0 / 6.0;                   // 3!
    ps = ps * t2 + 1.0;
    double pc = 1.0 / 2432902008176640000.0;     // 20!
    pc = pc * t2 + -1.0 / 6402373705728000.0;    // 18!
    pc = pc * t2 + 1.0 / 20922789888000.0;       // 16!
    pc = pc * t2 + -1.0 / 87178291200.0;         // 14!
    pc = pc * t2 + 1.0 / 479001600.0;            // 12!
    pc = pc * t2 + -1.0 / 3628800.0;             // 10!
    pc = pc * t2 + 1.0 / 40320.0;                // 8!
    pc = pc * t2 + -1.0 / 720.0;                 // 6!
    pc = pc * t2 + 1.0 / 24.0;                   // 4!
    pc = pc * t2 + -1.0 / 2.0;                   // 2!
    pc = pc * t2 + 1.0;
    sn = th * ps;
    cs = pc;
}

// Box-Muller on one word pair
__device__ __forceinline__ void normal_pair(uint32_t r_even, uint32_t r_odd, double &z_even, double &z_odd)
{
    const double radius = __builtin_sqrt(-2.0 * ln_unit(r_even));   // IEEE-754 squareRoot: correctly rounded
    const uint32_t quad = r_odd >> 30;
    const double frac = ((double)(r_odd & 0x3FFFFFFFu) + 0.5) * (1.0 / 1073741824.0);
    double s, c;
    sincos_quarter(frac * 0x1.921fb54442d18p+0, s, c);
    const double cosphi = quad == 0 ? c : quad == 1 ? -s : quad == 2 ? -c : s;
    const double sinphi = quad == 0 ? s : quad == 1 ? c : quad == 2 ? -s : -c;
    z_even = radius * cosphi;
    z_odd = radius * sinphi;
}

// the four binary64 values of one Philox block, by family
__device__ __forceinline__ void block_normals(const GenArgs &g, uint64_t blk, double z[4])
{
    uint32_t w[4];
    block_words(g, blk, w);
    if (g.family == MMAEMU_GEN_UNIFORM) {
#pragma unroll
        for (int j = 0; j < 4; ++j) z[j] = ((double)w[j] + 0.5) * (1.0 / 2147483648.0) - 1.0;      // exact
        return;
    }
    normal_pair(w[0], w[1], z[0], z[1]);
    normal_pair(w[2], w[3], z[2], z[3]);
    if (g.family == MMAEMU_GEN_NORMAL_OUTLIERS) {
        uint32_t w2[4], wh[4];
        double z2[4];
        philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), g.operand + 256u, 0u, g.k0, g.k1, w2);
        philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), g.operand + 512u, 0u, g.k0, g.k1, wh);
        normal_pair(w2[0], w2[1], z2[0], z2[1]);
        normal_pair(w2[2], w2[3], z2[2], z2[3]);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (wh[j] < 4294967u) z[j] = z[j] + 10.0 * z2[j];                                       // floor(0.001 * 2^32)
    }
}

// binary64 -> binary32 (RNE, hardware conversion) -> output format (RNE on the integer
// significand, saturating at the largest finite magnitude)
__device__ __forceinline__ uint32_t cast_out(const GenArgs &g, double v)
{
    const uint32_t b = __float_as_uint((float)v);
    if (g.dtype == MMAEMU_FP32) return b;
    const uint32_t sign = b >> 31, E32 = (b >> 23) & 0xFFu;
    const uint32_t sig = (b & 0x7FFFFFu) | (E32 ? 0x800000u : 0u);
    const int exp = (int)(E32 ? E32 : 1u) - 127;
    const int minexp = 1 - (int)g.bias;
    const int q = (exp > minexp ? exp : minexp) - (int)g.mbits;
    int shift = q - (exp - 23);                     // >= 23 - mbits > 0
    shift = shift > 31 ? 31 : shift;                // sig < 2^24: everything beyond 25 gives 0
    uint32_t n = sig >> shift;
    const uint32_t rem = sig & ((1u << shift) - 1u), half = 1u << (shift - 1);
    n += (rem > half) || (rem == half && (n & 1u));
    const int Et = exp + (int)g.bias;
    uint32_t code = ((uint32_t)((Et > 1 ? Et : 1) - 1) << g.mbits) + n;
    code = code > g.max_code ? g.max_code : code;
    return (sign << (g.width - 1)) | code;
}

template <typename T>
__device__ __forceinline__ void write_block(const GenArgs &g, T *out, uint64_t blk, const double z[4], double scale,
                                            bool scaled, uint64_t g0, uint64_t total)
{
    uint32_t v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = cast_out(g, scaled ? z[j] * scale : z[j]);
    const uint64_t e0 = 4 * blk;
    if (e0 >= g0 && e0 + 4 <= g0 + total && ((reinterpret_cast<uintptr_t>(out + (e0 - g0)) & (4 * sizeof(T) - 1)) == 0)) {
        store4<T>(out + (e0 - g0), v);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint64_t e = e0 + j;
            if (e >= g0 && e - g0 < total) out[e - g0] = (T)v[j];
        }
    }
}

__device__ __forceinline__ double block_absmax(const double z[4], uint64_t blk, uint64_t lo, uint64_t hi)
{
    double mx = 0.0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint64_t e = 4 * blk + j;
        const double a = z[j] < 0.0 ? -z[j] : z[j];
        if (e >= lo && e < hi && a > mx) mx = a;
    }
    return mx;
}

// no scaling, or scaling by a maximum already sitting in *absmax (SCALE_TENSOR, second step)
template <typename T>
__global__ void __launch_bounds__(256)
gen_normal_kernel(GenArgs g, T *out, uint64_t g0, uint64_t total, uint64_t blk0, uint64_t nblk, const double *absmax)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nblk) return;
    double z[4];
    block_normals(g, blk0 + t, z);
    const bool by_factor = g.scale_scope == MMAEMU_SCALE_FACTOR;          // every value times scale_target itself
    const bool scaled = by_factor || absmax != nullptr;
    const double scale = by_factor ? g.scale_target : (absmax != nullptr ? g.scale_target / *absmax : 1.0);
    write_block<T>(g, out, blk0 + t, z, scale, scaled, g0, total);
}

// SCALE_TENSOR, first step: max |z| over the call's elements into *absmax (zeroed before).
// Non-negative doubles order like their bit patterns, so an integer atomic max serves.
__global__ void __launch_bounds__(256)
gen_absmax_kernel(GenArgs g, uint64_t g0, uint64_t total, uint64_t blk0, uint64_t nblk, unsigned long long *absmax)
{
    __shared__ unsigned long long smax;
    if (threadIdx.x == 0) smax = 0ull;
    __syncthreads();
    double mx = 0.0;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; t < nblk; t += stride) {
        double z[4];
        block_normals(g, blk0 + t, z);
        const double a = block_absmax(z, blk0 + t, g0, g0 + total);
        mx = a > mx ? a : mx;
    }
    if (mx > 0.0) atomicMax(&smax, (unsigned long long)__double_as_longlong(mx));
    __syncthreads();
    if (threadIdx.x == 0 && smax) atomicMax(absmax, smax);
}

__global__ void zero_u64_kernel(unsigned long long *p) { *p = 0ull; }

// SCALE_TILE: one workgroup per tile; max |z| over the tile, then scale and write.
template <typename T>
__global__ void __launch_bounds__(256)
gen_normal_tile_kernel(GenArgs g, T *out, uint64_t ept, uint64_t first_tile, uint64_t n_tiles)
{
    __shared__ unsigned long long smax;
    const uint64_t g_call0 = first_tile * ept;
    for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint64_t lo = (first_tile + tile) * ept, hi = lo + ept;
        const uint64_t blk_lo = lo >> 2, nblk = ((hi - 1) >> 2) - blk_lo + 1;
        __syncthreads();                       // previous tile's readers are done with smax
        if (threadIdx.x == 0) smax = 0ull;
        __syncthreads();
        double mx = 0.0, zc[4] = {0.0, 0.0, 0.0, 0.0};
        uint64_t cached = ~0ull;
        for (uint64_t t = threadIdx.x; t < nblk; t += blockDim.x) {
            block_normals(g, blk_lo + t, zc);
            cached = blk_lo + t;
            const double a = block_absmax(zc, cached, lo, hi);
            mx = a > mx ? a : mx;
        }
        if (mx > 0.0) atomicMax(&smax, (unsigned long long)__double_as_longlong(mx));
        __syncthreads();
        const double scale = g.scale_target / __longlong_as_double((long long)smax);
        for (uint64_t t = threadIdx.x; t < nblk; t += blockDim.x) {
            double z[4];
            if (blk_lo + t == cached) { z[0] = zc[0]; z[1] = zc[1]; z[2] = zc[2]; z[3] = zc[3]; }
            else block_normals(g, blk_lo + t, z);
            // only this tile's elements: clip the writable range to [lo, hi)
            write_block<T>(g, out + (lo - g_call0), blk_lo + t, z, scale, true, lo, ept);
        }
    }
}

// SCALE_TILE for tiles of at most 256 elements that start on a Philox block (elements per tile a multiple of 4): one
// wavefront per tile, the maximum by lane shuffles, no LDS and no barrier.  Same values, same scale, same casts.
template <typename T>
__global__ void __launch_bounds__(256)
gen_normal_tile_wave_kernel(GenArgs g, T *out, uint64_t ept, uint64_t first_tile, uint64_t n_tiles)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const uint64_t nwaves = ((uint64_t)gridDim.x * blockDim.x) >> 6;
    const uint64_t g_call0 = first_tile * ept;
    const uint32_t nblk = (uint32_t)(ept / 4);
    for (uint64_t tile = wave; tile < n_tiles; tile += nwaves) {
        const uint64_t lo = (first_tile + tile) * ept, hi = lo + ept, blk_lo = lo >> 2;
        double z[4] = {0.0, 0.0, 0.0, 0.0}, mx = 0.0;
        if (lane < nblk) {
            block_normals(g, blk_lo + lane, z);
            mx = block_absmax(z, blk_lo + lane, lo, hi);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const double other = __shfl_xor(mx, o);
            mx = other > mx ? other : mx;
        }
        const double scale = g.scale_target / mx;
        if (lane < nblk) write_block<T>(g, out + (lo - g_call0), blk_lo + lane, z, scale, true, lo, ept);
    }
}

// ---- host side ------------------------------------------------------------------------

template <typename T>
static mmaemu_status launch_typed(const GenArgs &ga, void *out, uint64_t ept, uint64_t first_tile,
                                  uint64_t n_tiles, void *workspace, hipStream_t s)
{
    const uint64_t g0 = first_tile * ept, total = n_tiles * ept;
    const uint64_t wpe = ga.fp32_two_words ? 2 : 1;
    const uint64_t blk0 = (g0 * wpe) >> 2, nblk = (((g0 + total) * wpe - 1) >> 2) - blk0 + 1;
    const uint64_t grid = (nblk + 255) / 256;
    if (grid > 0x7FFFFFFFull) { set_error("generate: too many elements for one call"); return MMAEMU_ERR_SHAPE; }
    const bool value_family = ga.family == MMAEMU_GEN_NORMAL || ga.family == MMAEMU_GEN_UNIFORM || ga.family == MMAEMU_GEN_NORMAL_OUTLIERS;
    if (!value_family) {
        hipLaunchKernelGGL((gen_bits_kernel<T>), dim3((uint32_t)grid), dim3(256), 0, s, ga, (T *)out, g0, total, blk0, nblk);
    } else if (ga.scale_scope == MMAEMU_SCALE_NONE || ga.scale_scope == MMAEMU_SCALE_FACTOR) {
        hipLaunchKernelGGL((gen_normal_kernel<T>), dim3((uint32_t)grid), dim3(256), 0, s, ga, (T *)out, g0, total, blk0, nblk,
                           (const double *)nullptr);
    } else if (ga.scale_scope == MMAEMU_SCALE_TENSOR) {
        hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, s, (unsigned long long *)workspace);
        const uint64_t rgrid = grid > 2048 ? 2048 : grid;
        hipLaunchKernelGGL(gen_absmax_kernel, dim3((uint32_t)rgrid), dim3(256), 0, s, ga, g0, total, blk0, nblk,
                           (unsigned long long *)workspace);
        hipLaunchKernelGGL((gen_normal_kernel<T>), dim3((uint32_t)grid), dim3(256), 0, s, ga, (T *)out, g0, total, blk0, nblk,
                           (const double *)workspace);
    } else if (ept % 4 == 0 && ept <= 256) {
        const uint64_t wgrid = (n_tiles + 3) / 4 > (1ull << 20) ? (1ull << 20) : (n_tiles + 3) / 4;
        hipLaunchKernelGGL((gen_normal_tile_wave_kernel<T>), dim3((uint32_t)wgrid), dim3(256), 0, s, ga, (T *)out, ept, first_tile,
                           n_tiles);
    } else {
        const uint64_t per_tile_blocks = (ept + 3) / 4 + 1;
        uint32_t threads = per_tile_blocks <= 64 ? 64 : per_tile_blocks <= 128 ? 128 : 256;
        const uint64_t tgrid = n_tiles > (1ull << 20) ? (1ull << 20) : n_tiles;
        hipLaunchKernelGGL((gen_normal_tile_kernel<T>), dim3((uint32_t)tgrid), dim3(threads), 0, s, ga, (T *)out, ept,
                           first_tile, n_tiles);
    }
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

// ---- binary64 output ------------------------------------------------------------------------
// Value families: the binary64 value itself (times scale_target under SCALE_FACTOR), one word per element as for every
// other format.  Bit families: element g owns the words 2g (low half) and 2g + 1 (high half), so a Philox block holds
// two elements:
//   RANDOM_BITS   hi:lo
//   FINITE_BITS   v = floor(hi:lo * 2 nmag / 2^64), nmag = 2047 * 2^52 finite magnitudes; sign = v >= nmag
//   UNIFORM_EXP   sign = hi bit 31; exponent field from hi's low 31 bits as for FP32; mantissa = (hi's low 20 bits):lo
//   SIGNED_ZEROS  decided by hi as for the other formats
__global__ void __launch_bounds__(256)
gen_bits64_kernel(GenArgs g, uint64_t *out, uint64_t g0, uint64_t total, uint64_t blk0, uint64_t nblk)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nblk) return;
    const uint64_t blk = blk0 + t;
    uint32_t w[4];
    block_words(g, blk, w);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint64_t e = 2 * blk + j;
        if (e < g0 || e - g0 >= total) continue;
        const uint32_t lo = w[2 * j], hi = w[2 * j + 1];
        uint64_t v;
        if (g.family == MMAEMU_GEN_RANDOM_BITS) v = ((uint64_t)hi << 32) | lo;
        else if (g.family == MMAEMU_GEN_FINITE_BITS) {
            constexpr uint64_t NMAG = 2047ull << 52;
            const uint64_t u = __umul64hi(((uint64_t)hi << 32) | lo, 2ull * NMAG);
            const uint64_t sign = u >= NMAG;
            v = (sign << 63) | (u - sign * NMAG);
        } else if (g.family == MMAEMU_GEN_SIGNED_ZEROS) {
            const uint32_t kind = hi >> 30;
            const uint64_t mag = kind == 2u ? (1023ull << 52) : (kind == 3u ? 1ull : 0ull);
            v = ((uint64_t)((hi >> 29) & 1u) << 63) | mag;
        } else {                                                     // UNIFORM_EXP
            const uint32_t idx = (uint32_t)(((uint64_t)(hi & 0x7FFFFFFFu) * g.nchoices) >> 31);
            const uint64_t E = g.exp_zero ? (idx == 0 ? 0u : g.exp_lo + idx - 1u) : g.exp_lo + idx;
            v = ((uint64_t)(hi >> 31) << 63) | (E << 52) | ((uint64_t)(hi & 0xFFFFFu) << 32) | lo;
        }
        out[e - g0] = v;
    }
}

__global__ void __launch_bounds__(256)
gen_normal64_kernel(GenArgs g, uint64_t *out, uint64_t g0, uint64_t total, uint64_t blk0, uint64_t nblk)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nblk) return;
    double z[4];
    block_normals(g, blk0 + t, z);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint64_t e = 4 * (blk0 + t) + j;
        if (e < g0 || e - g0 >= total) continue;
        const double v = g.scale_scope == MMAEMU_SCALE_FACTOR ? z[j] * g.scale_target : z[j];
        out[e - g0] = (uint64_t)__double_as_longlong(v);
    }
}

static mmaemu_status launch_generate64(const GenArgs &ga, void *out, uint64_t ept, uint64_t first_tile, uint64_t n_tiles, hipStream_t s)
{
    const uint64_t g0 = first_tile * ept, total = n_tiles * ept;
    const bool value_family = ga.family == MMAEMU_GEN_NORMAL || ga.family == MMAEMU_GEN_UNIFORM || ga.family == MMAEMU_GEN_NORMAL_OUTLIERS;
    const uint64_t wpe = value_family ? 1 : 2;
    const uint64_t blk0 = (g0 * wpe) >> 2, nblk = (((g0 + total) * wpe - 1) >> 2) - blk0 + 1;
    const uint64_t grid = (nblk + 255) / 256;
    if (grid > 0x7FFFFFFFull) { set_error("generate: too many elements for one call"); return MMAEMU_ERR_SHAPE; }
    if (value_family) hipLaunchKernelGGL(gen_normal64_kernel, dim3((uint32_t)grid), dim3(256), 0, s, ga, (uint64_t *)out, g0, total, blk0, nblk);
    else hipLaunchKernelGGL(gen_bits64_kernel, dim3((uint32_t)grid), dim3(256), 0, s, ga, (uint64_t *)out, g0, total, blk0, nblk);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

mmaemu_status launch_generate(const mmaemu_gen_params &gp, void *out, uint32_t dtype, uint64_t ept,
                              uint64_t first_tile, uint64_t n_tiles, void *workspace, hipStream_t s)
{
    if (dtype == MMAEMU_FP64) {
        const uint64_t total64 = n_tiles * ept;
        if (gp.family == MMAEMU_GEN_ZERO) {
            uint64_t grid = (2 * total64 + 255) / 256;
            grid = grid < 1 ? 1 : (grid > 4096 ? 4096 : grid);
            hipLaunchKernelGGL(zero_kernel, dim3((uint32_t)grid), dim3(256), 0, s, (uint32_t *)out, 2 * total64, (uint8_t *)out, 0u);
            MMAEMU_HIP(hipGetLastError());
            return MMAEMU_OK;
        }
        GenArgs g64 = {};
        g64.family = gp.family;
        g64.operand = gp.operand;
        g64.k0 = (uint32_t)gp.seed;
        g64.k1 = (uint32_t)(gp.seed >> 32);
        g64.exp_lo = gp.exp_lo;
        g64.exp_zero = gp.exp_zero ? 1u : 0u;
        g64.nchoices = gp.exp_hi - gp.exp_lo + 1u + g64.exp_zero;
        g64.dtype = dtype;
        g64.scale_scope = gp.scale_scope;
        g64.scale_target = gp.scale_target;
        return launch_generate64(g64, out, ept, first_tile, n_tiles, s);
    }
    const FmtInfo f = fmt_info(dtype);
    const uint64_t total = n_tiles * ept;
    if (gp.family == MMAEMU_GEN_ZERO) {
        const uint64_t bytes = total * (uint64_t)(f.width / 8), nwords = bytes / 4;
        uint64_t grid = (nwords + 255) / 256;
        grid = grid < 1 ? 1 : (grid > 4096 ? 4096 : grid);
        hipLaunchKernelGGL(zero_kernel, dim3((uint32_t)grid), dim3(256), 0, s, (uint32_t *)out, nwords,
                           (uint8_t *)out + 4 * nwords, (uint32_t)(bytes - 4 * nwords));
        MMAEMU_HIP(hipGetLastError());
        return MMAEMU_OK;
    }
    GenArgs ga = {};
    ga.family = gp.family;
    ga.operand = gp.operand;
    ga.k0 = (uint32_t)gp.seed;
    ga.k1 = (uint32_t)(gp.seed >> 32);
    ga.width = dtype == MMAEMU_E8M0 ? 8u : (uint32_t)(1 + f.ebits + f.mbits);
    ga.mbits = (uint32_t)f.mbits;
    const uint32_t emax_field = (1u << f.ebits) - 1u;
    ga.nmag = f.ieee ? (emax_field << f.mbits) : (((emax_field + 1u) << f.mbits) - (f.nospec ? 0u : 1u));
    ga.exp_lo = gp.exp_lo;
    ga.exp_zero = gp.exp_zero ? 1u : 0u;
    ga.nchoices = gp.exp_hi - gp.exp_lo + 1u + ga.exp_zero;
    ga.fp32_two_words = (gp.family == MMAEMU_GEN_UNIFORM_EXP && dtype == MMAEMU_FP32) ? 1u : 0u;
    ga.bias = (uint32_t)f.bias;
    ga.max_code = ga.nmag - 1u;
    ga.dtype = dtype;
    ga.scale_scope = gp.scale_scope;
    ga.scale_target = gp.scale_target;
    switch (f.width) {
    case 8: return launch_typed<uint8_t>(ga, out, ept, first_tile, n_tiles, workspace, s);
    case 16: return launch_typed<uint16_t>(ga, out, ept, first_tile, n_tiles, workspace, s);
    default: return launch_typed<uint32_t>(ga, out, ept, first_tile, n_tiles, workspace, s);
    }
}

// ---- the variant for callers that cannot allocate -----------------------------------------
// The per-tensor scaling needs eight bytes of device memory for the running maximum.  Here they come out of an
// array that is part of the library's image: every GPU the library runs on holds its own copy at its own address
// until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the address it
// returns (looked up once per device, with that device current) is what kernels and fills get.
static __device__ __align__(256) unsigned char scratch[256];

static constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[MAX_DEVICES];          // per device, null until the first call on it

static mmaemu_status scratch_for_current_device(void **out)
{
    int dev = -1;
    MMAEMU_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) { set_error("generate_noalloc: device ordinal %d outside 0..%d", dev, MAX_DEVICES - 1); return MMAEMU_ERR_UNSUPPORTED; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        MMAEMU_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) { set_error("generate_noalloc: the scratch array has no device address"); return MMAEMU_ERR_HIP; }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MMAEMU_OK;
}

mmaemu_status launch_generate_noalloc(const mmaemu_gen_params &gp, void *out, uint32_t dtype, uint64_t ept,
                                      uint64_t first_tile, uint64_t n_tiles, hipStream_t s)
{
    void *ws = nullptr;
    const mmaemu_status st = scratch_for_current_device(&ws);
    if (st != MMAEMU_OK) return st;
    return launch_generate(gp, out, dtype, ept, first_tile, n_tiles, ws, s);      // (its first kernel clears the maximum)
}

} // namespace mmaemu
