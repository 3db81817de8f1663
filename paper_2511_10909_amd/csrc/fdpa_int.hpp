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

template <int T>
__device__ __forceinline__ Dec decode(uint32_t bits, uint32_t ftz_in)
{
    using F = Fmt<T>;
    constexpr uint32_t EMASK = (1u << F::EB) - 1u, MMASK = (1u << F::MB) - 1u;
    const uint32_t E = (bits >> F::MB) & EMASK, M = bits & MMASK;
    Dec d;
    d.sign = (bits >> (F::EB + F::MB)) & 1u;
    d.exp = (E ? (int)E : 1) - F::BIAS;
    d.sig = E ? (M | (1u << F::MB)) : M;
    d.cls = E ? CLS_NORMAL : (M ? CLS_SUB : CLS_ZERO);
    if (F::IEEE) {
        if (E == EMASK) d.cls = M ? CLS_NAN : CLS_INF;
    } else {
        if (E == EMASK && M == MMASK) d.cls = CLS_NAN;
    }
    if (ftz_in && d.cls == CLS_SUB) { d.cls = CLS_ZERO; d.sig = 0; d.sign = 0; }   // FlushSubnormal: -> +0.0
    return d;
}

// RD: v counts units of 2^lsb; the result counts units of 2^unit, rounded toward minus infinity.
// Left shifts are bounded by the entry point's limits on F and F2.
__device__ __forceinline__ int64_t align_rd(int64_t v, int lsb, int unit)
{
    const int sh = lsb - unit;
    if (sh >= 0) return (int64_t)((uint64_t)v << sh);
    return sh > -64 ? (v >> (-sh)) : (v >> 63);        // arithmetic shift = floor
}

// Algorithm "TR-FDPA", steps 3 and 4 (Algorithm "GTR-FDPA", steps 4 and 5): T counts units of
// 2^(emax - F).  E = max(e_max, e_c); T' = RD_F2(T at E); s_c' = RD_F(c at E), dropped by the
// special truncation when e_c < E - F - 1; d = rho(T' + s_c').
__device__ __forceinline__ uint32_t rounded_sum_with_c(const ModelArgs &p, int64_t T, int emax, const Dec &dc,
                                                       bool special_truncation)
{
    const int E = dc.exp > emax ? dc.exp : emax;
    const int64_t T2 = align_rd(T, emax - p.F, E - p.F2);
    const int64_t sc = dc.sign ? -(int64_t)dc.sig : (int64_t)dc.sig;
    int64_t sc2 = align_rd(sc, dc.exp - 23, E - p.F);
    if (special_truncation && dc.exp < E - p.F - 1) sc2 = 0;
    const int Fm = p.F2 > p.F ? p.F2 : p.F;
    const int64_t S = (int64_t)((uint64_t)T2 << (Fm - p.F2)) + (int64_t)((uint64_t)sc2 << (Fm - p.F));
    if (S == 0) return 0u;
    const uint32_t neg = S < 0;
    return round_to_fp32(neg, (uint64_t)(neg ? -S : S), E - Fm, 0, p.out_round);
}

template <int TA, int TB>
__device__ uint32_t fdpa_group(const ModelArgs &p, const typename Fmt<TA>::elem *a,
                               const typename Fmt<TB>::elem *b, uint32_t L, uint32_t c)
{
    constexpr int FA = Fmt<TA>::MB, FB = Fmt<TB>::MB;
    const Dec dc = decode<MMAEMU_FP32>(c, p.ftz_in);

    // pass 1: special values and the maximum exponent
    bool any_nan = dc.cls == CLS_NAN, pinf = false, ninf = false;
    const bool rd_mode = p.c_mode == MMAEMU_C_AFTER_RD || p.c_mode == MMAEMU_C_AFTER_RD_EVEN_ODD;
    int emax = -100000, eeven = -100000, eodd = -100000;
    for (uint32_t k = 0; k < L; ++k) {
        const Dec x = decode<TA>(a[k], p.ftz_in), y = decode<TB>(b[k], p.ftz_in);
        if (x.cls == CLS_NAN || y.cls == CLS_NAN) any_nan = true;
        else if (x.cls == CLS_INF || y.cls == CLS_INF) {
            if (x.cls == CLS_ZERO || y.cls == CLS_ZERO) any_nan = true;      // inf * 0
            else if (x.sign ^ y.sign) ninf = true;
            else pinf = true;
        } else {
            const int e = x.exp + y.exp;
            emax = e > emax ? e : emax;
            if (k & 1u) eodd = e > eodd ? e : eodd;
            else eeven = e > eeven ? e : eeven;
            if (rd_mode) {                                                   // |a b| >= 2^128 is an infinity
                const uint32_t prod = x.sig * y.sig;
                if (prod && (31 - __builtin_clz(prod)) + e - FA - FB >= 128) {
                    if (x.sign ^ y.sign) ninf = true; else pinf = true;
                }
            }
        }
    }
    if (dc.cls == CLS_INF) { if (dc.sign) ninf = true; else pinf = true; }
    if (any_nan || (pinf && ninf)) return p.nan_bits;
    if (pinf) return 0x7F800000u;
    if (ninf) return 0xFF800000u;

    if (p.c_mode == MMAEMU_C_AFTER_RD_EVEN_ODD) {
        // even and odd products fused apart, each at its own maximum exponent
        int64_t Te = 0, To = 0;
        for (uint32_t k = 0; k < L; ++k) {
            const Dec x = decode<TA>(a[k], p.ftz_in), y = decode<TB>(b[k], p.ftz_in);
            const uint64_t prod = (uint64_t)(x.sig * y.sig);
            const int sh = (x.exp + y.exp - FA - FB) - (((k & 1u) ? eodd : eeven) - p.F);
            const uint64_t al = sh >= 0 ? (prod << sh) : (sh > -32 ? (prod >> (-sh)) : 0ull);
            const int64_t t = (x.sign ^ y.sign) ? -(int64_t)al : (int64_t)al;
            if (k & 1u) To += t; else Te += t;
        }
        const int64_t T = align_rd(Te, eeven - p.F, emax - p.F) + align_rd(To, eodd - p.F, emax - p.F);
        uint32_t d = rounded_sum_with_c(p, T, emax, dc, true);
        if (p.ftz_out && (d & 0x7F800000u) == 0) d &= 0x80000000u;
        return d;
    }

    if (p.c_mode == MMAEMU_C_IN_GROUP && dc.exp > emax) emax = dc.exp;
    const int unit = emax - p.F;            // aligned terms count multiples of 2^unit

    // pass 2: align, truncate toward zero, sum exactly
    int64_t S = 0;
    for (uint32_t k = 0; k < L; ++k) {
        const Dec x = decode<TA>(a[k], p.ftz_in), y = decode<TB>(b[k], p.ftz_in);
        const uint64_t prod = (uint64_t)(x.sig * y.sig);                    // <= 22 bits
        const int sh = (x.exp + y.exp - FA - FB) - unit;                    // <= F
        const uint64_t al = sh >= 0 ? (prod << sh) : (sh > -32 ? (prod >> (-sh)) : 0ull);
        S += (x.sign ^ y.sign) ? -(int64_t)al : (int64_t)al;
    }
    uint32_t d;
    if (p.c_mode == MMAEMU_C_IN_GROUP) {
        const int sh = (dc.exp - 23) - unit;
        const uint64_t al = sh >= 0 ? ((uint64_t)dc.sig << sh) : (sh > -32 ? ((uint64_t)dc.sig >> (-sh)) : 0ull);
        S += dc.sign ? -(int64_t)al : (int64_t)al;
        const uint32_t neg = S < 0;
        const uint64_t mag = (uint64_t)(neg ? -S : S);
        d = mag ? round_to_fp32(neg, mag, unit, 0, p.out_round) : 0u;
    } else if (p.c_mode == MMAEMU_C_AFTER_RD) {
        d = rounded_sum_with_c(p, S, emax, dc, false);
    } else {
        const uint32_t neg = S < 0;
        d = add_exact_round(neg, (uint64_t)(neg ? -S : S), unit, dc.sign, (uint64_t)dc.sig, dc.exp - 23, p.out_round);
    }
    if (p.ftz_out && (d & 0x7F800000u) == 0) d &= 0x80000000u;
    return d;
}


// run-time operand types (used where a template per type pair is not worth its code size)
// (parameters by value: a reference would force the caller to keep a copy of them in scratch memory)
__device__ __noinline__ uint32_t fdpa_group_raw(ModelArgs p, uint32_t ta, uint32_t tb, const void *a, const void *b,
                                                uint32_t L, uint32_t c)
{
#define MMAEMU_CASE(X, Y)                                                                             \
    if (ta == X && tb == Y)                                                                           \
        return fdpa_group<X, Y>(p, reinterpret_cast<const typename Fmt<X>::elem *>(a),                \
                                reinterpret_cast<const typename Fmt<Y>::elem *>(b), L, c)
    MMAEMU_CASE(MMAEMU_FP8_E4M3, MMAEMU_FP8_E4M3); MMAEMU_CASE(MMAEMU_FP8_E4M3, MMAEMU_FP8_E5M2);
    MMAEMU_CASE(MMAEMU_FP8_E4M3, MMAEMU_FP16);     MMAEMU_CASE(MMAEMU_FP8_E4M3, MMAEMU_BF16);
    MMAEMU_CASE(MMAEMU_FP8_E5M2, MMAEMU_FP8_E4M3); MMAEMU_CASE(MMAEMU_FP8_E5M2, MMAEMU_FP8_E5M2);
    MMAEMU_CASE(MMAEMU_FP8_E5M2, MMAEMU_FP16);     MMAEMU_CASE(MMAEMU_FP8_E5M2, MMAEMU_BF16);
    MMAEMU_CASE(MMAEMU_FP16, MMAEMU_FP8_E4M3);     MMAEMU_CASE(MMAEMU_FP16, MMAEMU_FP8_E5M2);
    MMAEMU_CASE(MMAEMU_FP16, MMAEMU_FP16);         MMAEMU_CASE(MMAEMU_FP16, MMAEMU_BF16);
    MMAEMU_CASE(MMAEMU_BF16, MMAEMU_FP8_E4M3);     MMAEMU_CASE(MMAEMU_BF16, MMAEMU_FP8_E5M2);
    MMAEMU_CASE(MMAEMU_BF16, MMAEMU_FP16);
#undef MMAEMU_CASE
    return fdpa_group<MMAEMU_BF16, MMAEMU_BF16>(p, reinterpret_cast<const uint16_t *>(a),
                                                reinterpret_cast<const uint16_t *>(b), L, c);
}

} // namespace mmaemu
