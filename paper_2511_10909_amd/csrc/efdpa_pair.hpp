// The exact sum of Algorithm "E-FDPA" held as an unevaluated pair of binary64 numbers, for both kernels that use it.
//
// Every product of two operands of at most 24 significant bits is exact in binary64.  add() puts it into the high part
// with Knuth's TwoSum and the error term into the low part with a second TwoSum; while that second error is zero the
// pair is the exact sum (about 106 bits of it).  finish() normalises the pair (hi = RN(sum), lo = sum - hi), rounds hi
// to odd where lo is not zero, and converts once: 53 bits are more than 24 + 2, so the hardware conversion to binary32
// rounds the exact sum correctly.  NaN and infinite operands need nothing of their own: binary64 arithmetic gives NaN
// for a NaN, for infinity times zero and for infinities of both signs, and the infinity otherwise (Sec. 4.2's rule).
#pragma once
#include "emulate_tiled.hpp"

namespace mmaemu {

// a decoded element as the binary64 number it denotes (at most 24 significant bits: exact)
template <class FT>
__device__ __forceinline__ double dec_value(const FT &f, const Dec &x)
{
    if (x.cls == CLS_NAN) return __longlong_as_double(0x7FF8000000000000ll);
    const double mag = x.cls == CLS_INF ? __longlong_as_double(0x7FF0000000000000ll) : ldexp((double)x.sig, x.exp - f.mb());
    return x.sign ? -mag : mag;
}

// bytes per element as the arrays hold them
__device__ __host__ __forceinline__ uint32_t elem_bytes(uint32_t t)
{
    return (t == MMAEMU_FP32 || t == MMAEMU_TF32) ? 4u : ((t == MMAEMU_FP16 || t == MMAEMU_BF16) ? 2u : 1u);
}

// element idx of an array of `esize`-byte elements: its bits (TF32 without its 13 surplus bits)
__device__ __forceinline__ uint32_t elem_bits(uint32_t t, uint32_t esize, const void *p, uint64_t idx)
{
    if (esize == 1) return static_cast<const uint8_t *>(p)[idx];
    if (esize == 2) return static_cast<const uint16_t *>(p)[idx];
    const uint32_t w = static_cast<const uint32_t *>(p)[idx];
    return t == MMAEMU_TF32 ? w >> 13 : w;
}

// the binary64 number that an element's bits denote (NaN and infinities as themselves); FlushSubnormal on request
__device__ __forceinline__ double elem_value(uint32_t t, uint32_t bits, uint32_t ftz_in)
{
    float v = 0.0f;
    uint32_t ex;
    bool wild = false;
    switch (t) {   // uniform
    case MMAEMU_FP8_E4M3: decode_elem<MMAEMU_FP8_E4M3>(bits, ftz_in, 0u, v, ex, wild); break;
    case MMAEMU_FP8_E5M2: decode_elem<MMAEMU_FP8_E5M2>(bits, ftz_in, 0u, v, ex, wild); break;
    case MMAEMU_FP6_E2M3: decode_elem<MMAEMU_FP6_E2M3>(bits, ftz_in, 0u, v, ex, wild); break;
    case MMAEMU_FP6_E3M2: decode_elem<MMAEMU_FP6_E3M2>(bits, ftz_in, 0u, v, ex, wild); break;
    case MMAEMU_FP4_E2M1: decode_elem<MMAEMU_FP4_E2M1>(bits, ftz_in, 0u, v, ex, wild); break;
    case MMAEMU_FP16: decode_elem<MMAEMU_FP16>(bits, ftz_in, 0u, v, ex, wild); break;
    case MMAEMU_TF32: decode_elem<MMAEMU_TF32>(bits, ftz_in, 0u, v, ex, wild); break;
    case MMAEMU_FP32: v = __uint_as_float((ftz_in && (bits & 0x7F800000u) == 0) ? 0u : bits); break;
    default: decode_elem<MMAEMU_BF16>(bits, ftz_in, 0u, v, ex, wild); break;
    }
    return (double)v;
}

// the same for N elements of one type with a single (uniform) branch on the type
template <int N>
__device__ __forceinline__ void elem_values(uint32_t t, const uint32_t (&bits)[N], uint32_t ftz_in, double (&v)[N])
{
    auto all = [&](auto type_tag) {
        constexpr int T = decltype(type_tag)::value;
#pragma unroll
        for (int q = 0; q < N; ++q) {
            float f = 0.0f;
            uint32_t ex;
            bool wild = false;
            decode_elem<T>(bits[q], ftz_in, 0u, f, ex, wild);
            v[q] = (double)f;
        }
    };
    switch (t) {
    case MMAEMU_FP8_E4M3: all(std::integral_constant<int, MMAEMU_FP8_E4M3>{}); break;
    case MMAEMU_FP8_E5M2: all(std::integral_constant<int, MMAEMU_FP8_E5M2>{}); break;
    case MMAEMU_FP6_E2M3: all(std::integral_constant<int, MMAEMU_FP6_E2M3>{}); break;
    case MMAEMU_FP6_E3M2: all(std::integral_constant<int, MMAEMU_FP6_E3M2>{}); break;
    case MMAEMU_FP4_E2M1: all(std::integral_constant<int, MMAEMU_FP4_E2M1>{}); break;
    case MMAEMU_FP16: all(std::integral_constant<int, MMAEMU_FP16>{}); break;
    case MMAEMU_TF32: all(std::integral_constant<int, MMAEMU_TF32>{}); break;
    case MMAEMU_FP32:
#pragma unroll
        for (int q = 0; q < N; ++q) v[q] = (double)__uint_as_float((ftz_in && (bits[q] & 0x7F800000u) == 0) ? 0u : bits[q]);
        break;
    default: all(std::integral_constant<int, MMAEMU_BF16>{}); break;
    }
}

// s + e = a + b exactly (s = RN(a + b)), for finite operands
__device__ __forceinline__ void two_sum(double a, double b, double &s, double &e)
{
    s = a + b;
    const double bb = s - a;
    e = (a - (s - bb)) + (b - bb);
}

struct ExactPair {
    double hi, lo;
    double lost;                    // what the pair could not hold: 0 while the sum is exact, NaN after an infinity

    // a group starts from its accumulator (a binary32 pattern, already flushed where the model flushes inputs)
    __device__ __forceinline__ void start(uint32_t c) { hi = (double)__uint_as_float(c); lo = 0.0; lost = 0.0; }

    __device__ __forceinline__ void add(double x, double y)
    {
        const double prod = x * y;                                 // exact
        double s, e, l2, e2;
        two_sum(hi, prod, s, e);
        two_sum(lo, e, l2, e2);
        hi = s;
        lo = l2;
        lost += __builtin_fabs(e2);
    }

    // The group's result where the pair decides it: a special value, or the conversion of the exact sum.  Returns false
    // where the sum left the pair's reach (the caller then runs the group through the integer routine).
    __device__ __forceinline__ bool finish(const ModelArgs &p, uint32_t &out) const
    {
        const uint64_t hb = (uint64_t)__double_as_longlong(hi);
        if ((hb & 0x7FFFFFFFFFFFFFFFull) > 0x7FF0000000000000ull) { out = p.nan_bits; return true; }
        if ((hb & 0x7FFFFFFFFFFFFFFFull) == 0x7FF0000000000000ull) { out = (hb >> 63) ? 0xFF800000u : 0x7F800000u; return true; }
        if (!(lost == 0.0)) return false;
        double h, l;
        two_sum(hi, lo, h, l);                                     // h = RN(sum), l = sum - h
        if (l != 0.0) {
            // round to odd: of h and its neighbour on l's side, the one whose last bit is set
            long long b = __double_as_longlong(h);
            if ((b & 1ll) == 0) b += ((l > 0.0) == (h > 0.0)) ? 1ll : -1ll;              // (h is not zero here: |l| <= ulp(h) / 2)
            h = __longlong_as_double(b);
        }
        uint32_t o = __float_as_uint((float)h);                    // RNE, gradual underflow, overflow to infinity
        if (p.out_round == MMAEMU_ROUND_RZ) {
            const double back = (double)__uint_as_float(o);
            if (__builtin_fabs(back) > __builtin_fabs(h)) o -= 1u;                       // rounded away from zero: step back
        }
        if (h == 0.0) o = 0u;                                      // an exact zero is +0.0
        o &= p.out_mask;                                           // (RZ-E8M13)
        if (p.ftz_out && (o & 0x7F800000u) == 0) o &= 0x80000000u;
        if (p.zero_result_positive && (o & 0x7FFFFFFFu) == 0) o = 0u;
        out = o;
        return true;
    }
};

} // namespace mmaemu
