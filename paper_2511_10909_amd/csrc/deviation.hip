// Distribution of the deviation delta = D - D_real of a model's (or an instruction's) outputs from the real result
// (Sec. 6.2.4: the bias of the round-down modes shows as a distribution of delta shifted toward the negative side,
// against a symmetric one for the variant that truncates toward zero).  D_real = c + sum_k a_k b_k is taken exactly:
// per sampled output one thread adds D and subtracts every product and the accumulator, in an unevaluated pair of
// binary64 numbers while that is exact and in a wide fixed-point number otherwise, so delta itself is exact; only its
// binary64 image (for the three sums) is rounded.  Linear bins of width 2^bin_exp
// around zero: bin i holds delta in [(i - 32) w, (i - 31) w), the outermost bins everything beyond.
#include "efdpa_pair.hpp"

namespace mmaemu {

constexpr int DEV_WORDS = sizeof(mmaemu_deviation_hist) / 8;
static_assert(DEV_WORDS == 5 + MMAEMU_DEVIATION_BINS + 3, "layout of mmaemu_deviation_hist");

__global__ void deviation_reset_kernel(mmaemu_deviation_hist *h)
{
    uint64_t *w = reinterpret_cast<uint64_t *>(h);
    if (threadIdx.x < DEV_WORDS) w[threadIdx.x] = 0ull;             // +0.0 is all-zero bits
}

// Elements kk .. kk + 7 of a row (bits as elem_bits gives them): `vec` says that the row's bytes from kk on are 16-byte
// aligned (8-byte for one-byte elements), so one or two wide loads bring them; per-element loads of 64 lanes, each in a
// row of its own, keep the address unit busy for longer than all the arithmetic of a sample takes.
__device__ __forceinline__ void load8(uint32_t t, uint32_t esize, const uint8_t *row, uint32_t kk, bool vec, uint32_t (&r)[8])
{
    if (!vec) {
#pragma unroll
        for (int q = 0; q < 8; ++q) r[q] = elem_bits(t, esize, row, kk + q);
    } else if (esize == 2) {
        const uint4 v = *reinterpret_cast<const uint4 *>(row + 2u * kk);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) { r[2 * q] = w[q] & 0xFFFFu; r[2 * q + 1] = w[q] >> 16; }
    } else if (esize == 1) {
        const uint2 v = *reinterpret_cast<const uint2 *>(row + kk);
#pragma unroll
        for (int q = 0; q < 4; ++q) { r[q] = (v.x >> (8 * q)) & 0xFFu; r[4 + q] = (v.y >> (8 * q)) & 0xFFu; }
    } else {
        const uint4 v0 = *reinterpret_cast<const uint4 *>(row + 4u * kk), v1 = *reinterpret_cast<const uint4 *>(row + 4u * kk + 16u);
        const uint32_t w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
        for (int q = 0; q < 8; ++q) r[q] = t == MMAEMU_TF32 ? w[q] >> 13 : w[q];
    }
}

// The same through the wide fixed-point number (exact for any finite operands): sign, whether delta is zero,
// floor(delta / 2^bin_exp) clamped to +-NB, and |delta|'s binary64 image (its 64 bits from the leading one downward,
// converted once).
__device__ __noinline__ void delta_wide(DynFmt fa, DynFmt fb, const uint8_t *a, const uint8_t *b, uint32_t k, uint32_t cb, uint32_t db,
                                        int unit_bit, uint32_t &neg, bool &zero, int &fi, double &ad)
{
    constexpr int NB = MMAEMU_DEVIATION_BINS;
    uint32_t w[XL];
    for (int q = 0; q < XL; ++q) w[q] = 0u;
    for (uint32_t kk = 0; kk < k; ++kk) {
        const Dec x = decode_as(fa, fa.load(a, kk), 0u), y = decode_as(fb, fb.load(b, kk), 0u);
        wide_add(w, sig_product(fa, fb, x, y), x.exp + y.exp - fa.mb() - fb.mb(), (x.sign ^ y.sign) ^ 1u);   // - a b
    }
    {
        const uint32_t Ec = (cb >> 23) & 0xFFu, Ed = (db >> 23) & 0xFFu;
        wide_add(w, (cb & 0x7FFFFFu) | (Ec ? 0x800000u : 0u), (int)(Ec ? Ec : 1u) - 150, (cb >> 31) ^ 1u);        // - c
        wide_add(w, (db & 0x7FFFFFu) | (Ed ? 0x800000u : 0u), (int)(Ed ? Ed : 1u) - 150, db >> 31);               // + D
    }
    neg = w[XL - 1] >> 31;
    if (neg) {
        uint32_t carry = 1;
        for (int q = 0; q < XL; ++q) {
            const uint64_t t = (uint64_t)(~w[q]) + carry;
            w[q] = (uint32_t)t;
            carry = (uint32_t)(t >> 32);
        }
    }
    int top = XL - 1;
    while (top >= 0 && w[top] == 0u) --top;
    zero = top < 0;
    fi = 0;
    ad = 0.0;
    if (zero) return;
    const int hi_bit = 32 * top + (31 - __builtin_clz(w[top]));
    // floor(delta / 2^bin_exp) from the magnitude: its bits from unit_bit upward, and whether anything lies below
    if (hi_bit < unit_bit) fi = neg ? -1 : 0;
    else if (hi_bit - unit_bit >= 6) fi = neg ? -NB : NB;
    else {
        const int limb = unit_bit >> 5, off = unit_bit & 31;
        uint32_t v = w[limb] >> off;
        if (off && limb + 1 < XL) v |= w[limb + 1] << (32 - off);
        const int q = (int)(v & 63u);
        bool below = (off != 0) && (w[limb] & ((1u << off) - 1u)) != 0u;
        for (int t = 0; t < limb; ++t) below |= w[t] != 0u;
        fi = neg ? (below ? -q - 1 : -q) : q;
    }
    const int low_bit = hi_bit - 63;
    uint64_t mag;
    int lsb;
    if (low_bit <= 0) { mag = ((uint64_t)w[1] << 32) | w[0]; lsb = XBASE; }
    else {
        const int l0 = low_bit >> 5, sh = low_bit & 31;
        const uint32_t a0 = w[l0], a1 = w[l0 + 1], a2 = (l0 + 2 < XL) ? w[l0 + 2] : 0u;
        const u128 win = ((u128)a2 << 64) | ((u128)a1 << 32) | a0;
        mag = (uint64_t)(win >> sh);
        lsb = XBASE + low_bit;
    }
    ad = ldexp((double)mag, lsb);
}

__global__ void __launch_bounds__(256)
deviation_kernel(const void *__restrict__ A, const void *__restrict__ B, const uint32_t *__restrict__ C,
                 const uint32_t *__restrict__ D, uint32_t m, uint32_t n, uint32_t k, uint32_t ta, uint32_t tb, uint64_t stride,
                 uint64_t nsamples, int bin_exp, mmaemu_deviation_hist *hist)
{
    constexpr int NB = MMAEMU_DEVIATION_BINS;
    __shared__ uint32_t counts[5 + NB];
    if (threadIdx.x < 5 + NB) counts[threadIdx.x] = 0u;
    __syncthreads();
    const DynFmt fa = dyn_fmt(ta), fb = dyn_fmt(tb);
    const uint32_t esa = (uint32_t)fa.width_ / 8u, esb = (uint32_t)fb.width_ / 8u;
    const uint64_t per_tile = (uint64_t)m * n;
    const int unit_bit = bin_exp - XBASE;                            // index of the bit that weighs one bin width
    const bool vec_a = (reinterpret_cast<uintptr_t>(A) & 15u) == 0 && k % 8u == 0, vec_b = (reinterpret_cast<uintptr_t>(B) & 15u) == 0 && k % 8u == 0;
    double sum = 0.0, sum_abs = 0.0, sum_sq = 0.0;
    // (a workgroup handles at most 2^32 / 256 samples: the 32-bit LDS counters cannot overflow, see the launch)
    for (uint64_t sidx = (uint64_t)blockIdx.x * 256u + threadIdx.x; sidx < nsamples; sidx += (uint64_t)gridDim.x * 256u) {
        const uint64_t o = sidx * stride;
        const uint64_t tile = o / per_tile;
        const uint32_t rem = (uint32_t)(o - tile * per_tile), i = rem / n, j = rem - i * n;
        const uint8_t *a = static_cast<const uint8_t *>(A) + (tile * m + i) * (uint64_t)k * esa;
        const uint8_t *b = static_cast<const uint8_t *>(B) + (tile * n + j) * (uint64_t)k * esb;
        // delta first as an unevaluated pair of binary64 numbers (efdpa_pair.hpp): D, then every product and the accumulator
        // taken away; while the pair holds the sum exactly (always for FP16 / FP8 operands; BF16 or FP32 operands spread
        // over hundreds of binary places may leave it) sign, bin and binary64 image follow from the normalised pair
        const uint32_t cb = C ? C[o] : 0u, db = D[o];
        bool bad = (cb & 0x7F800000u) == 0x7F800000u || (db & 0x7F800000u) == 0x7F800000u;
        ExactPair pr;
        pr.start(db);
        const double finite_max = 0x1.fffffffffffffp+1023;
        uint32_t kk = 0;
        for (; kk + 8 <= k; kk += 8) {
            // (eight elements of each row fetched before the first is used: one wait per eight terms)
            uint32_t ra[8], rb[8];
            load8(ta, esa, a, kk, vec_a, ra);
            load8(tb, esb, b, kk, vec_b, rb);
            double xa[8], xb[8];
            elem_values(ta, ra, 0u, xa);                             // (one branch on the type per eight elements)
            elem_values(tb, rb, 0u, xb);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                bad |= !(__builtin_fabs(xa[q]) <= finite_max) || !(__builtin_fabs(xb[q]) <= finite_max);
                pr.add(-xa[q], xb[q]);
            }
        }
        for (; kk < k; ++kk) {
            const double x = elem_value(ta, elem_bits(ta, esa, a, kk), 0u), y = elem_value(tb, elem_bits(tb, esb, b, kk), 0u);
            bad |= !(__builtin_fabs(x) <= finite_max) || !(__builtin_fabs(y) <= finite_max);
            pr.add(-x, y);
        }
        if (bad) { atomicAdd(&counts[1], 1u); continue; }
        pr.add(-(double)__uint_as_float(cb), 1.0);
        uint32_t neg;
        bool zero;
        int fi;
        double ad;
        if (pr.lost == 0.0) {
            double h, l;
            two_sum(pr.hi, pr.lo, h, l);                                 // h = RN(delta), l = delta - h
            neg = h < 0.0;
            zero = h == 0.0;
            ad = __builtin_fabs(h);
            // floor(delta / 2^bin_exp): of h, and one less where h is a whole number of bins and l lies below it (a
            // fractional h / w keeps at least one of its own last places to either side, more than |l / w|)
            const double qh = ldexp(h, -bin_exp);
            if (qh >= (double)NB) fi = NB;
            else if (qh <= -(double)NB) fi = -NB;
            else if (qh == 0.0) fi = neg ? -1 : 0;                       // (h / w below the binary64 range)
            else {
                const double fl = __builtin_floor(qh);
                fi = (int)fl - ((fl == qh && l < 0.0) ? 1 : 0);
            }
        } else {
            delta_wide(fa, fb, a, b, k, cb, db, unit_bit, neg, zero, fi, ad);
        }
        atomicAdd(&counts[0], 1u);
        if (zero) {
            atomicAdd(&counts[3], 1u);
            atomicAdd(&counts[5 + NB / 2], 1u);
            continue;
        }
        atomicAdd(&counts[neg ? 2 : 4], 1u);
        int bin = fi + NB / 2;
        bin = bin < 0 ? 0 : (bin > NB - 1 ? NB - 1 : bin);
        atomicAdd(&counts[5 + bin], 1u);
        sum += neg ? -ad : ad;
        sum_abs += ad;
        sum_sq += ad * ad;
    }
    // the three sums: over the wavefront by lane exchanges, over the workgroup through LDS, then one atomic per workgroup
    // and sum (thousands of wavefronts adding to the same three words took longer than everything else in the kernel)
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        sum += __shfl_xor(sum, off, 64);
        sum_abs += __shfl_xor(sum_abs, off, 64);
        sum_sq += __shfl_xor(sum_sq, off, 64);
    }
    __shared__ double wave_sums[4][3];
    if ((threadIdx.x & 63u) == 0u) {
        wave_sums[threadIdx.x >> 6][0] = sum;
        wave_sums[threadIdx.x >> 6][1] = sum_abs;
        wave_sums[threadIdx.x >> 6][2] = sum_sq;
    }
    __syncthreads();
    double *gd = reinterpret_cast<double *>(reinterpret_cast<uint64_t *>(hist) + 5 + NB);
    if (threadIdx.x < 3) {
        const double t = (wave_sums[0][threadIdx.x] + wave_sums[1][threadIdx.x]) + (wave_sums[2][threadIdx.x] + wave_sums[3][threadIdx.x]);
        if (t != 0.0) atomicAdd(&gd[threadIdx.x], t);
    }
    __syncthreads();
    if (threadIdx.x < 5 + NB && counts[threadIdx.x])
        atomicAdd(reinterpret_cast<unsigned long long *>(hist) + threadIdx.x, (unsigned long long)counts[threadIdx.x]);
}

mmaemu_status launch_deviation_reset(mmaemu_deviation_hist *h, hipStream_t s)
{
    hipLaunchKernelGGL(deviation_reset_kernel, dim3(1), dim3(128), 0, s, h);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

mmaemu_status launch_deviation_sample(const void *A, const void *B, const uint32_t *C, const uint32_t *D, uint32_t m, uint32_t n,
                                      uint32_t k, uint64_t batch, uint32_t ta, uint32_t tb, uint64_t stride, int bin_exp,
                                      mmaemu_deviation_hist *h, hipStream_t s)
{
    const uint64_t total = batch * m * n;
    const uint64_t nsamples = (total + stride - 1) / stride;
    if (nsamples == 0) return MMAEMU_OK;
    uint64_t blocks = (nsamples + 255) / 256;
    if (blocks > 2048) blocks = 2048;                                // grid-stride beyond that: two rounds of what the chip holds
    if ((nsamples + blocks - 1) / blocks > 0xFFFFFFFFull) { set_error("deviation_sample: more than 2^43 samples in one call"); return MMAEMU_ERR_SHAPE; }
    hipLaunchKernelGGL(deviation_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, A, B, C, D, m, n, k, ta, tb, stride, nsamples,
                       bin_exp, h);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

} // namespace mmaemu
