// Integer-arithmetic FDPA group (device code), shared by the general kernel and by the
// fall-back route of the tiled kernels: paper Algorithms "T-FDPA", "TR-FDPA" and "GTR-FDPA"
// step by step on raw operands, with the special-value rules of Sec. 4.2 and both flush rules.
#pragma once
#include "common.hpp"

namespace mmaemu {

enum { CLS_ZERO = 0, CLS_SUB = 1, CLS_NORMAL = 2, CLS_INF = 3, CLS_NAN = 4 };

struct Dec {
    uint32_t sig;
    int exp;
    uint32_t sign;
    int cls;
};

// An operand format as this routine sees it.  StaticFmt<T>: every property a compile-time constant (the general kernel:
// one instantiation per type pair).  DynFmt: the properties are run-time values (the tiled kernels' rare fall-back: one
// instantiation for every type pair, an order of magnitude less code).
template <int T> struct StaticFmt {
    __device__ __forceinline__ constexpr int eb() const { return Fmt<T>::EB; }
    __device__ __forceinline__ constexpr int mb() const { return Fmt<T>::MB; }
    __device__ __forceinline__ constexpr int bias() const { return Fmt<T>::BIAS; }
    __device__ __forceinline__ constexpr bool ieee() const { return Fmt<T>::IEEE; }
    __device__ __forceinline__ constexpr bool nospec() const { return Fmt<T>::NOSPEC; }
    __device__ __forceinline__ constexpr int shift() const { return T == MMAEMU_TF32 ? 13 : 0; }   // surplus low bits of the word
    __device__ __forceinline__ uint32_t load(const void *p, uint32_t k) const { return static_cast<const typename Fmt<T>::elem *>(p)[k]; }
};
struct DynFmt {
    int eb_, mb_, bias_, width_;
    bool ieee_, nospec_;
    __device__ __forceinline__ int eb() const { return eb_; }
    __device__ __forceinline__ int mb() const { return mb_; }
    __device__ __forceinline__ int bias() const { return bias_; }
    __device__ __forceinline__ bool ieee() const { return ieee_; }
    __device__ __forceinline__ bool nospec() const { return nospec_; }
    __device__ __forceinline__ constexpr int shift() const { return 0; }                            // (TF32: dropped at the load)
    __device__ __forceinline__ uint32_t load(const void *p, uint32_t k) const
    {
        // 32-bit words are TF32 here (FP32 operands never take the tiled kernels): the 13 surplus bits go at once
        return width_ == 8 ? static_cast<const uint8_t *>(p)[k] : (width_ == 16 ? static_cast<const uint16_t *>(p)[k] : static_cast<const uint32_t *>(p)[k] >> 13);
    }
};
__device__ __forceinline__ DynFmt dyn_fmt(uint32_t t)
{
    switch (t) {
    case MMAEMU_FP8_E4M3: return DynFmt{4, 3, 7, 8, false, false};
    case MMAEMU_FP8_E5M2: return DynFmt{5, 2, 15, 8, true, false};
    case MMAEMU_FP16: return DynFmt{5, 10, 15, 16, true, false};
    case MMAEMU_FP6_E2M3: return DynFmt{2, 3, 1, 8, false, true};
    case MMAEMU_FP6_E3M2: return DynFmt{3, 2, 3, 8, false, true};
    case MMAEMU_FP4_E2M1: return DynFmt{2, 1, 1, 8, false, true};
    case MMAEMU_TF32: return DynFmt{8, 10, 127, 32, true, false};
    default: return DynFmt{8, 7, 127, 16, true, false};                                             // BF16
    }
}

template <class FT>
__device__ __forceinline__ Dec decode_as(const FT &f, uint32_t bits, uint32_t ftz_in)
{
    const uint32_t EMASK = (1u << f.eb()) - 1u, MMASK = (1u << f.mb()) - 1u;
    bits >>= f.shift();
    const uint32_t E = (bits >> f.mb()) & EMASK, M = bits & MMASK;
    Dec d;
    d.sign = (bits >> (f.eb() + f.mb())) & 1u;
    d.exp = (E ? (int)E : 1) - f.bias();
    d.sig = E ? (M | (1u << f.mb())) : M;
    d.cls = E ? CLS_NORMAL : (M ? CLS_SUB : CLS_ZERO);
    if (f.ieee()) {
        if (E == EMASK) d.cls = M ? CLS_NAN : CLS_INF;
    } else if (!f.nospec()) {
        if (E == EMASK && M == MMASK) d.cls = CLS_NAN;                             // the E4M3 rule: one NaN code
    }
    if (ftz_in && d.cls == CLS_SUB) { d.cls = CLS_ZERO; d.sig = 0; d.sign = 0; }   // FlushSubnormal: -> +0.0
    return d;
}

template <int T>
__device__ __forceinline__ Dec decode(uint32_t bits, uint32_t ftz_in) { return decode_as(StaticFmt<T>{}, bits, ftz_in); }

typedef __int128 i128;
typedef unsigned __int128 u128;

// RD: v counts units of 2^lsb; the result counts units of 2^unit, rounded toward minus infinity.
// Left shifts are bounded by the entry point's limits on the precisions.
__device__ __forceinline__ i128 align_rd(i128 v, int lsb, int unit)
{
    const int sh = lsb - unit;
    if (sh >= 0) return (i128)((u128)v << sh);
    return sh > -127 ? (v >> (-sh)) : (v >> 127);      // arithmetic shift = floor
}

// The rounding of the summation's second step (the sum of the products and the accumulator brought to E, the merges of
// a split group): toward minus infinity as the algorithms print it, or -- Sec. 6.2.4's hypothetical instruction -- toward
// zero: the magnitude of a negative value loses its low bits instead.
__device__ __forceinline__ i128 align_step(const ModelArgs &p, i128 v, int lsb, int unit)
{
    if (p.rd_toward_zero && v < 0 && unit > lsb) {
        const int drop = unit - lsb;
        const u128 mag = (u128)(-v);
        return drop > 127 ? (i128)0 : -(i128)(mag >> drop);
    }
    return align_rd(v, lsb, unit);
}

__device__ __forceinline__ int bitlen128(u128 x)
{
    const uint64_t hi = (uint64_t)(x >> 64), lo = (uint64_t)x;
    return hi ? 128 - __builtin_clzll(hi) : (lo ? 64 - __builtin_clzll(lo) : 0);
}

// rho for a 128-bit magnitude: the value is first cut to 64 bits with the lost bits remembered
// (they lie at least 40 places below the leading bit, far under the rounding position).
__device__ __forceinline__ uint32_t round128_to_fp32(uint32_t neg, u128 mag, int lsb, uint32_t mode)
{
    const int bl = bitlen128(mag);
    if (bl <= 64) return round_to_fp32(neg, (uint64_t)mag, lsb, 0, mode);
    const int sh = bl - 64;
    const uint32_t lost = (mag & ((((u128)1) << sh) - 1)) != 0;
    return round_to_fp32(neg, (uint64_t)(mag >> sh), lsb + sh, lost, mode);
}

// E8M0 block scales of one row of A and one row of B (Algorithm "ST-FDPA"): sa[q], sb[q] scale the products
// q * block .. (q + 1) * block - 1 of the row; null pointers mean no scaling.  k0 is the group's first k.
struct ScaleRef {
    const uint8_t *sa, *sb;
    uint32_t block, k0;
};
__device__ __forceinline__ ScaleRef no_scales() { return ScaleRef{nullptr, nullptr, 1u, 0u}; }
// Exp(alpha) + Exp(beta) for product k of the group (0 without scales)
__device__ __forceinline__ int scale_exp(const ScaleRef &sr, uint32_t k)
{
    if (!sr.sa) return 0;
    const uint32_t q = (sr.k0 + k) / sr.block;
    return (int)sr.sa[q] + (int)sr.sb[q] - 254;
}

// Exact product of two significands (at most 24 bits each): only a pair of FP32 operands needs the 64-bit multiply.
template <class FTA, class FTB>
__device__ __forceinline__ uint64_t sig_product(const FTA &fa, const FTB &fb, const Dec &x, const Dec &y)
{
    return (fa.mb() + fb.mb() > 30) ? (uint64_t)x.sig * (uint64_t)y.sig : (uint64_t)(x.sig * y.sig);
}

// One sub-group of products k = first, first + stride, ... (count of them): maximum exponent
// over the terms that take part, then the sum of the terms aligned at that exponent with F
// fractional bits, truncated toward zero.  Returns false when no term takes part.
template <class FTA, class FTB>
__device__ bool fused_part(const ModelArgs &p, const FTA &fa, const FTB &fb, const void *a, const void *b, const ScaleRef &sr,
                           uint32_t first, uint32_t stride, uint32_t count, int &emax, int64_t &T)
{
    const int FA = fa.mb(), FB = fb.mb();
    bool any = false;
    emax = 0;
    for (uint32_t q = 0; q < count; ++q) {
        const uint32_t k = first + q * stride;
        const Dec x = decode_as(fa, fa.load(a, k), p.ftz_in), y = decode_as(fb, fb.load(b, k), p.ftz_in);
        if (p.skip_zero_terms && (x.sig == 0 || y.sig == 0)) continue;
        const int e = x.exp + y.exp + scale_exp(sr, k);
        emax = (!any || e > emax) ? e : emax;
        any = true;
    }
    T = 0;
    if (!any) return false;
    const int unit = emax - p.F;
    for (uint32_t q = 0; q < count; ++q) {
        const uint32_t k = first + q * stride;
        const Dec x = decode_as(fa, fa.load(a, k), p.ftz_in), y = decode_as(fb, fb.load(b, k), p.ftz_in);
        const uint64_t prod = sig_product(fa, fb, x, y);                    // <= 22 bits (48 for FP32 operands)
        const int sh = (x.exp + y.exp + scale_exp(sr, k) - FA - FB) - unit; // <= F
        const uint64_t al = sh >= 0 ? (prod << sh) : (sh > -64 ? (prod >> (-sh)) : 0ull);
        T += (x.sign ^ y.sign) ? -(int64_t)al : (int64_t)al;
    }
    return true;
}

// Algorithm "TR-FDPA", steps 3 and 4 (Algorithm "GTR-FDPA", steps 4 and 5) and their variations:
// T counts units of 2^unit_T.  E = max(e_max, e_c) over the terms that take part; s_c' = RD_Fc(c at E),
// dropped by the special truncation when e_c < E - F_c - 1 (and T' = 0 when E - e_max >= sum_drop_distance);
// then either RD_F2(T at E) + s_c', or the
// exact T + s_c' rounded down to F2 bits below its own leading bit; d = rho of that.
__device__ __forceinline__ uint32_t rounded_sum_with_c(const ModelArgs &p, bool have_T, int64_t T64, int emax, int unit_T,
                                                       const Dec &dc)
{
    // the accumulator always takes part, a zero one with the exponent of the subnormals
    const int E = have_T ? (dc.exp > emax ? dc.exp : emax) : dc.exp;
    const i128 sc = dc.sign ? -(i128)dc.sig : (i128)dc.sig;
    i128 sc2 = align_step(p, sc, dc.exp - 23, E - p.Fc);
    if (p.acc_special_truncation && dc.exp < E - p.Fc - 1) sc2 = 0;
    const int unit_c = E - p.Fc;
    if (have_T && p.sum_drop_distance && E - emax >= p.sum_drop_distance) have_T = false;      // T' = 0
    i128 T = have_T ? (i128)T64 : (i128)0;
    if (!have_T) unit_T = unit_c;
    i128 S;
    int unit;
    if (p.f2_at_leading_bit) {
        // T far below the accumulator's unit is first rounded down to units of 2^(unit_c - 64):
        // rounding down in two steps equals rounding down once
        if (unit_c - unit_T > 64) { T = align_step(p, T, unit_T, unit_c - 64); unit_T = unit_c - 64; }
        unit = unit_T < unit_c ? unit_T : unit_c;
        S = (i128)((u128)T << (unit_T - unit)) + (i128)((u128)sc2 << (unit_c - unit));
        if (S == 0) return 0u;
        int lead = bitlen128((u128)(S < 0 ? -S : S)) - 1 + unit;
        lead = lead < -126 ? -126 : lead;                  // no lower than binary32's smallest normal exponent
        if (lead - p.F2 > unit) { S = align_step(p, S, unit, lead - p.F2); unit = lead - p.F2; }
    } else {
        const i128 T2 = align_step(p, T, unit_T, E - p.F2);
        unit = (E - p.F2) < unit_c ? (E - p.F2) : unit_c;
        S = (i128)((u128)T2 << ((E - p.F2) - unit)) + (i128)((u128)sc2 << (unit_c - unit));
    }
    if (S == 0) return 0u;
    const uint32_t neg = S < 0;
    return round128_to_fp32(neg, (u128)(neg ? -S : S), unit, p.out_round);
}

// The accumulator (a binary32 pattern) as sign, Exp and a 24-bit significand with value sig 2^(Exp - 23).  A binary16
// accumulator keeps binary16's exponent range: Exp = -14 for zero and for |c| < 2^-14 (its subnormals), whose
// significand then has leading zeros; FlushSubnormal applies to those.
__device__ __forceinline__ Dec decode_acc(const ModelArgs &p, uint32_t c)
{
    Dec d = decode<MMAEMU_FP32>(c, p.ftz_in);
    if ((p.flags & FL_ACC16) && d.cls != CLS_NAN && d.cls != CLS_INF && d.exp < -14) {
        const int sh = -14 - d.exp;
        d.sig = sh < 32 ? d.sig >> sh : 0u;             // exact: a binary16 subnormal has at most 10 significant bits
        d.exp = -14;
        d.cls = d.sig ? CLS_SUB : CLS_ZERO;
        if (p.ftz_in && d.cls == CLS_SUB) { d.cls = CLS_ZERO; d.sig = 0; d.sign = 0; }
    }
    return d;
}

__device__ __forceinline__ uint32_t finish_group(const ModelArgs &p, uint32_t d)
{
    if (p.flags & FL_ACC16) {                            // d is the binary32 pattern of a binary16 number
        if (p.ftz_out && (d & 0x7F800000u) < (113u << 23)) d &= 0x80000000u;      // |d| < 2^-14
        if (p.zero_result_positive && (d & 0x7FFFFFFFu) == 0) d = 0u;
        return d;
    }
    d &= p.out_mask;                                     // RZ-E8M13: low mantissa bits cut (toward zero, like RZ itself)
    if (p.ftz_out && (d & 0x7F800000u) == 0) d &= 0x80000000u;
    if (p.zero_result_positive && (d & 0x7FFFFFFFu) == 0) d = 0u;
    return d;
}

// ---- Algorithm "E-FDPA": the exact sum ----------------------------------------------------------------------
// A fixed-point number of XL 32-bit limbs, two's complement, bit 0 of limb 0 weighing 2^XBASE.  The lowest bit any
// term can have is 2^-298 (two binary32 subnormals multiplied), the largest product is below 2^256, and 2^20 of those
// add 20 bits: 640 bits hold every sum with its sign.
constexpr int XL = 20;
constexpr int XBASE = -320;

// w += (-1)^neg * mag * 2^lsb, mag below 2^48
__device__ __forceinline__ void wide_add(uint32_t (&w)[XL], uint64_t mag, int lsb, uint32_t neg)
{
    if (mag == 0) return;
    const int pos = lsb - XBASE, first = pos >> 5;
    const u128 v = (u128)mag << (pos & 31);                       // below 2^79: three limbs
    uint32_t part[3] = {(uint32_t)v, (uint32_t)(v >> 32), (uint32_t)(v >> 64)};
    uint32_t carry = 0;                                           // carry of the addition, or borrow of the subtraction
    for (int i = first; i < XL; ++i) {
        const uint32_t x = (i - first) < 3 ? part[i - first] : 0u;
        if (i - first >= 3 && !carry) break;
        const uint64_t old = w[i];
        if (!neg) {
            const uint64_t t = old + x + carry;
            w[i] = (uint32_t)t;
            carry = (uint32_t)(t >> 32);
        } else {
            const uint64_t t = old - x - carry;
            w[i] = (uint32_t)t;
            carry = (uint32_t)((t >> 32) & 1u);
        }
    }
}

// rho of the number held in w (consumed: it is negated in place when negative)
__device__ __forceinline__ uint32_t wide_round(uint32_t (&w)[XL], uint32_t mode)
{
    const uint32_t neg = w[XL - 1] >> 31;
    if (neg) {                                                    // magnitude: two's complement negation
        uint32_t carry = 1;
        for (int i = 0; i < XL; ++i) {
            const uint64_t t = (uint64_t)(~w[i]) + carry;
            w[i] = (uint32_t)t;
            carry = (uint32_t)(t >> 32);
        }
    }
    int top = XL - 1;
    while (top >= 0 && w[top] == 0) --top;
    if (top < 0) return 0u;                                       // an exact zero is +0.0
    // the 64 bits from the leading bit downward, and whether anything lies below them
    const int lead = 31 - __builtin_clz(w[top]);                  // bit index inside limb `top`
    const int hi_bit = 32 * top + lead;                           // index of the leading bit in the whole number
    uint64_t mag = 0;
    uint32_t sticky = 0;
    const int low_bit = hi_bit - 63;                              // index of the lowest bit taken (may be negative: then exact)
    if (low_bit <= 0) {
        // at most 64 bits in all: limbs 0 and 1 (and 2 cannot be non-zero here unless hi_bit >= 64)
        mag = ((uint64_t)w[1] << 32) | w[0];
        return round_to_fp32(neg, mag, XBASE, 0, mode);
    }
    const int l0 = low_bit >> 5, sh = low_bit & 31;               // the window starts inside limb l0
    const uint32_t a0 = w[l0], a1 = w[l0 + 1], a2 = (l0 + 2 < XL) ? w[l0 + 2] : 0u;
    const u128 win = ((u128)a2 << 64) | ((u128)a1 << 32) | a0;
    mag = (uint64_t)(win >> sh);
    if (sh && (a0 & ((1u << sh) - 1u))) sticky = 1;
    for (int i = 0; i < l0; ++i) sticky |= (w[i] != 0);
    return round_to_fp32(neg, mag, XBASE + low_bit, sticky, mode);
}

template <class FTA, class FTB>
__device__ uint32_t exact_group(const ModelArgs &p, const FTA &fa, const FTB &fb, const void *a, const void *b, uint32_t L, const Dec &dc)
{
    uint32_t w[XL];
    for (int i = 0; i < XL; ++i) w[i] = 0;
    const int FA = fa.mb(), FB = fb.mb();
    for (uint32_t k = 0; k < L; ++k) {
        const Dec x = decode_as(fa, fa.load(a, k), p.ftz_in), y = decode_as(fb, fb.load(b, k), p.ftz_in);
        wide_add(w, sig_product(fa, fb, x, y), x.exp + y.exp - FA - FB, x.sign ^ y.sign);
    }
    wide_add(w, dc.sig, dc.exp - 23, dc.sign);
    return wide_round(w, p.out_round);
}

// WITH_EXACT: the exact mode is compiled in (the general kernel only: its wide accumulator lives in private memory, which
// the tiled kernels' fall-back must not drag into every tiled kernel)
template <bool WITH_EXACT = false, class FTA, class FTB>
__device__ uint32_t fdpa_group(const ModelArgs &p, const FTA &fa, const FTB &fb, const void *a, const void *b, uint32_t L,
                               uint32_t c, const ScaleRef &sr)
{
    const int FA = fa.mb(), FB = fb.mb();
    const Dec dc = decode_acc(p, c);
    const bool acc16 = (p.flags & FL_ACC16) != 0;
    if (sr.sa) {                                                              // a NaN scale factor (E8M0 pattern 0xFF)
        for (uint32_t q = sr.k0 / sr.block; q <= (sr.k0 + L - 1) / sr.block; ++q)
            if (sr.sa[q] == 0xFFu || sr.sb[q] == 0xFFu) return p.nan_bits;
    }

    if (p.flags & FL_NAN_PROPAGATE) {
        // the payload variation, in its order of precedence (FP32 operands: the element is the binary32 pattern);
        // what it leaves is handled below as usual
        for (uint32_t k = 0; k < L; ++k) {
            const uint32_t xa = fa.load(a, k), xb = fb.load(b, k);
            if (decode_as(fa, xa, p.ftz_in).cls == CLS_NAN) return xa | 0x00400000u;
            if (decode_as(fb, xb, p.ftz_in).cls == CLS_NAN) return xb | 0x00400000u;
        }
        for (uint32_t k = 0; k < L; ++k) {
            const Dec x = decode_as(fa, fa.load(a, k), p.ftz_in), y = decode_as(fb, fb.load(b, k), p.ftz_in);
            if ((x.cls == CLS_INF && y.cls == CLS_ZERO) || (y.cls == CLS_INF && x.cls == CLS_ZERO)) return p.nan_bits;
        }
        if (dc.cls == CLS_NAN) return c | 0x00400000u;
    }
    // special values (Sec. 4.2)
    bool any_nan = dc.cls == CLS_NAN, pinf = false, ninf = false;
    for (uint32_t k = 0; k < L; ++k) {
        const Dec x = decode_as(fa, fa.load(a, k), p.ftz_in), y = decode_as(fb, fb.load(b, k), p.ftz_in);
        if (x.cls == CLS_NAN || y.cls == CLS_NAN) any_nan = true;
        else if (x.cls == CLS_INF || y.cls == CLS_INF) {
            if (x.cls == CLS_ZERO || y.cls == CLS_ZERO) any_nan = true;      // inf * 0
            else if (x.sign ^ y.sign) ninf = true;
            else pinf = true;
        } else if (p.c_mode == MMAEMU_C_AFTER_RD && !p.wide_products) {       // |a b| >= 2^128 is an infinity
            const uint64_t prod = sig_product(fa, fb, x, y);
            if (prod && (63 - __builtin_clzll(prod)) + x.exp + y.exp + scale_exp(sr, k) - FA - FB >= 128) {
                if (x.sign ^ y.sign) ninf = true; else pinf = true;
            }
        }
    }
    if (dc.cls == CLS_INF) { if (dc.sign) ninf = true; else pinf = true; }
    if (any_nan || (pinf && ninf)) return p.nan_bits;
    if (pinf) return 0x7F800000u;
    if (ninf) return 0xFF800000u;

    if constexpr (WITH_EXACT) {
        if (p.c_mode == MMAEMU_C_EXACT) return finish_group(p, exact_group(p, fa, fb, a, b, L, dc));
    }

    if (p.c_mode == MMAEMU_C_AFTER_RD) {
        if (p.split == MMAEMU_SPLIT_NONE) {
            int emax; int64_t T;
            const bool have = fused_part(p, fa, fb, a, b, sr, 0, 1, L, emax, T);
            return finish_group(p, rounded_sum_with_c(p, have, T, emax, emax - p.F, dc));
        }
        // two or four sub-groups, each fused at its own maximum exponent, merged with RD at F_m bits
        const int np_ = p.split == MMAEMU_SPLIT_QUARTERS ? 4 : 2;
        const uint32_t len = L / (uint32_t)np_, stride = p.split == MMAEMU_SPLIT_EVEN_ODD ? 2u : 1u;
        int ep[4] = {0, 0, 0, 0}, emax = 0; int64_t Tp[4] = {0, 0, 0, 0}; bool hp[4] = {false, false, false, false}, any = false;
        for (int g = 0; g < np_; ++g) {
            const uint32_t first = p.split == MMAEMU_SPLIT_EVEN_ODD ? (uint32_t)g : (uint32_t)g * len;
            hp[g] = fused_part(p, fa, fb, a, b, sr, first, stride, len, ep[g], Tp[g]);
            if (hp[g] && (!any || ep[g] > emax)) emax = ep[g];
            any |= hp[g];
        }
        i128 T = 0;
        for (int g = 0; g < np_; ++g)
            if (hp[g]) T += align_step(p, (i128)Tp[g], ep[g] - p.F, emax - p.Fm);
        return finish_group(p, rounded_sum_with_c(p, any, (int64_t)T, emax, emax - p.Fm, dc));
    }

    int emax; int64_t S;
    bool have = fused_part(p, fa, fb, a, b, sr, 0, 1, L, emax, S);          // S aligned at the products' own maximum
    uint32_t d;
    if (p.c_mode == MMAEMU_C_IN_GROUP) {
        if (!have || dc.exp > emax) {
            // the accumulator raises the maximum: align the products again at the new exponent
            const int unit = dc.exp - p.F;
            S = 0;
            for (uint32_t k = 0; k < L; ++k) {
                const Dec x = decode_as(fa, fa.load(a, k), p.ftz_in), y = decode_as(fb, fb.load(b, k), p.ftz_in);
                const uint64_t prod = sig_product(fa, fb, x, y);
                const int sh = (x.exp + y.exp + scale_exp(sr, k) - FA - FB) - unit;
                const uint64_t al = sh >= 0 ? (prod << sh) : (sh > -64 ? (prod >> (-sh)) : 0ull);
                S += (x.sign ^ y.sign) ? -(int64_t)al : (int64_t)al;
            }
            emax = dc.exp;
        }
        const int unit = emax - p.F;
        const int sh = (dc.exp - 23) - unit;
        const uint64_t al = sh >= 0 ? ((uint64_t)dc.sig << sh) : (sh > -32 ? ((uint64_t)dc.sig >> (-sh)) : 0ull);
        S += dc.sign ? -(int64_t)al : (int64_t)al;
        const uint32_t neg = S < 0;
        const uint64_t mag = (uint64_t)(neg ? -S : S);
        d = mag ? round_out(acc16, neg, mag, unit, 0, p.out_round) : 0u;
    } else {                                                            // C_AFTER_EXACT
        if (!have) { emax = 0; S = 0; }
        const uint32_t neg = S < 0;
        d = add_exact_round(neg, (uint64_t)(neg ? -S : S), emax - p.F, dc.sign, (uint64_t)dc.sig, dc.exp - 23, p.out_round, acc16);
    }
    return finish_group(p, d);
}


// run-time operand types: the tiled kernels' fall-back (a template per type pair there multiplied the code size)
// (parameters by value: a reference would force the caller to keep a copy of them in scratch memory)
__device__ __noinline__ uint32_t fdpa_group_raw(ModelArgs p, uint32_t ta, uint32_t tb, const void *a, const void *b,
                                                uint32_t L, uint32_t c, ScaleRef sr)
{
    return fdpa_group(p, dyn_fmt(ta), dyn_fmt(tb), a, b, L, c, sr);
}

// the same without block scales
__device__ __noinline__ uint32_t fdpa_group_raw_unscaled(ModelArgs p, uint32_t ta, uint32_t tb, const void *a, const void *b,
                                                         uint32_t L, uint32_t c)
{
    return fdpa_group(p, dyn_fmt(ta), dyn_fmt(tb), a, b, L, c, no_scales());
}

} // namespace mmaemu
