/*
 * CPU oracle, second form: the chained truncated fused-dot-product-add model in
 * plain C with fixed wide integers, one output element at a time, OpenMP over rows.
 *
 * TEST INFRASTRUCTURE ONLY: used by the test-suite, the smoke check and the
 * CPU-baseline leg of the benchmark.  It shares no code with the HIP library.
 *
 * What it computes (paper Sec. 4.1.3): Algorithm "Phi_FDPA" (chain of groups of
 * L = min(K, L_max) products, d <- c first) around Algorithm "T-FDPA" (exact
 * unnormalised products, e_max over the L products and the accumulator, alignment
 * with truncation toward zero to F fractional bits, exact fixed-point sum,
 * conversion rho), the special-value rules of Sec. 4.2, the output flush of
 * Algorithm "FTZ-Add/FTZ-Mul" and the input flush of Algorithm "Phi_FTZ-AddMul".
 * c_mode 2 is Algorithm "TR-FDPA" and c_mode 3 Algorithm "GTR-FDPA" (Sec. 4.1.3):
 * the products are fused without the accumulator (in GTR-FDPA, even and odd products
 * apart, the two sums then rounded down to F bits at their common exponent), the sum
 * is rounded down to F2 and the accumulator to F fractional bits at E = max(e_max,
 * e_c), and the two are added; a product of magnitude 2^128 or more counts as an
 * infinity (Sec. 4.2).
 * It is checked bit for bit against the rational-arithmetic form in ../fdpa.py and
 * against the paper's printed values by the CPU tests.
 *
 * Number representation: every aligned term is an integer count of 2^(e_max - F);
 * products have at most 22 significant bits, so with F <= 64 and at most 2^20
 * terms per group every sum fits a signed 128-bit integer.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>
#include <omp.h>
#include <stdlib.h>

typedef __int128 i128;
typedef unsigned __int128 u128;

enum { T_E4M3 = 0, T_E5M2 = 1, T_FP16 = 2, T_BF16 = 3, T_FP32 = 4, T_E8M0 = 5, T_E2M3 = 6, T_E3M2 = 7, T_E2M1 = 8, T_TF32 = 9 };
enum { CLS_ZERO, CLS_SUB, CLS_NORMAL, CLS_INF, CLS_NAN };
enum { C_IN_GROUP = 0, C_AFTER_EXACT = 1, C_AFTER_RD = 2, C_AFTER_RD_EVEN_ODD = 3 };
enum { R_RNE = 0, R_RZ = 1 };

typedef struct {
    uint32_t group_len, frac_bits, align_round, c_mode, out_round, ftz_in, ftz_out, nan_bits, frac_bits2;
    uint32_t split, acc_special_truncation, frac_bits_merge, frac_bits_acc, skip_zero_terms, f2_at_leading_bit, zero_result_positive;
    uint32_t sum_drop_distance;
    uint32_t family;     /* 0: chained FDPA, 1: FTZ-AddMul with P = group_len */
    uint32_t out_mant_bits; /* 23, or 13 (RZ-E8M13, with out_round = RZ) */
    uint32_t wide_products; /* RD mode: no infinity from a single product of magnitude >= 2^128 */
    uint32_t acc_fp16;      /* accumulator and output are binary16 patterns (rho = RNE-FP16 / RZ-FP16); T-FDPA modes only */
    uint32_t nan_propagate; /* FP32 operands: a NaN result carries a payload (first NaN operand in the order a_0, b_0, a_1, ...,
                               made quiet; else nan_bits for infinity times zero; else a NaN accumulator, made quiet; else
                               nan_bits for infinities of both signs) */
    uint32_t rd_toward_zero; /* RD modes: every round-down of the summation truncates toward zero instead (Sec. 6.2.4's
                                hypothetical instruction) */
} o2_params;

/* ieee: 1 = exponent field all ones is Inf / NaN, 0 = the E4M3 rule (one NaN code), 2 = every code finite (FP6, FP4) */
typedef struct { int ebits, mbits, bias, ieee; } fmt_t;
static const fmt_t FMT[10] = {
    {4, 3, 7, 0}, {5, 2, 15, 1}, {5, 10, 15, 1}, {8, 7, 127, 1}, {8, 23, 127, 1}, {8, 0, 127, 2},
    {2, 3, 1, 2}, {3, 2, 3, 2}, {2, 1, 1, 2}, {8, 10, 127, 1}};      /* TF32: the top 19 bits of a binary32 word */

typedef struct { int cls, sign, exp; uint32_t sig; } dec_t;

static dec_t decode(uint32_t bits, int t)
{
    const fmt_t f = FMT[t];
    dec_t d;
    uint32_t emask = (1u << f.ebits) - 1u;
    uint32_t E = (bits >> f.mbits) & emask;
    uint32_t M = bits & ((1u << f.mbits) - 1u);
    d.sign = (bits >> (f.ebits + f.mbits)) & 1u;
    d.exp = 0; d.sig = 0;
    if (f.ieee == 1 && E == emask) { d.cls = M ? CLS_NAN : CLS_INF; return d; }
    if (f.ieee == 0 && E == emask && M == ((1u << f.mbits) - 1u)) { d.cls = CLS_NAN; return d; }
    if (E == 0) { d.cls = M ? CLS_SUB : CLS_ZERO; d.exp = 1 - f.bias; d.sig = M; return d; }
    d.cls = CLS_NORMAL; d.exp = (int)E - f.bias; d.sig = (1u << f.mbits) | M;
    return d;
}

static uint32_t load_elem(const void *p, size_t i, int t)
{
    switch (t) {
    case T_E4M3: case T_E5M2: case T_E2M3: case T_E3M2: case T_E2M1: return ((const uint8_t *)p)[i];
    case T_FP16: case T_BF16: return ((const uint16_t *)p)[i];
    case T_TF32: return ((const uint32_t *)p)[i] >> 13;       /* the low 13 mantissa bits are ignored */
    default: return ((const uint32_t *)p)[i];
    }
}

static int bitlen128(u128 x)
{
    uint64_t hi = (uint64_t)(x >> 64), lo = (uint64_t)x;
    if (hi) return 128 - __builtin_clzll(hi);
    if (lo) return 64 - __builtin_clzll(lo);
    return 0;
}

/* rho: round (-1)^neg * mag * 2^lsb to binary32.  `sticky` says the true magnitude is
 * a little more (sticky > 0) or less (sticky < 0) than mag * 2^lsb, by less than one
 * unit of 2^lsb; the caller guarantees the unit is far below any rounding boundary. */
static uint32_t to_bin(int neg, u128 mag, int lsb, int sticky, int mode, int mb, int emin, int emax)
{
    if (mag == 0) return 0u; /* exact zero -> +0.0 */
    if (sticky < 0) { mag -= 1; sticky = 1; } /* value in (mag-1, mag) units: floor is mag-1, remainder non-zero */
    int bl = bitlen128(mag);
    int e = bl - 1 + lsb;               /* floor(log2 |value|) */
    int eg = e < emin ? emin : e;       /* exponent of the grid */
    int qexp = eg - mb;                 /* weight of the last place */
    int sh = qexp - lsb;                /* drop `sh` low bits of mag (if positive) */
    u128 n; int half = 0, rest = sticky != 0;
    if (sh <= 0) {
        n = mag << (-sh);               /* exact; fits since the result has <= 24 bits */
    } else if (sh > 127) {
        n = 0; rest |= (mag != 0);
    } else {
        n = mag >> sh;
        u128 rem = mag & ((((u128)1) << sh) - 1);
        u128 h = ((u128)1) << (sh - 1);
        half = (rem & h) != 0;
        rest |= (rem & (h - 1)) != 0;
    }
    if (mode == R_RNE && half && (rest || (n & 1))) n += 1;
    if (n == ((u128)1 << (mb + 1))) { n >>= 1; eg += 1; }
    uint32_t out;
    const uint32_t inf = (uint32_t)(2 * emax + 1) << mb;                 /* exponent field all ones */
    if (eg > emax) out = (mode == R_RNE) ? inf : inf - 1u;
    else if (n < ((u128)1 << mb)) out = (uint32_t)n;           /* subnormal / zero, eg == emin */
    else out = ((uint32_t)(eg + emax) << mb) | ((uint32_t)n & ((1u << mb) - 1u));
    return ((uint32_t)neg << (mb == 23 ? 31 : 15)) | out;
}

static uint32_t to_fp32(int neg, u128 mag, int lsb, int sticky, int mode) { return to_bin(neg, mag, lsb, sticky, mode, 23, -126, 127); }
/* rho of the model: binary32, or binary16 when the accumulator and the output are FP16 */
static uint32_t rho(const o2_params *p, int neg, u128 mag, int lsb, int sticky)
{
    return p->acc_fp16 ? to_bin(neg, mag, lsb, sticky, (int)p->out_round, 10, -14, 15) : to_fp32(neg, mag, lsb, sticky, (int)p->out_round);
}

/* exact x + y with x = sx*mx*2^lx, y likewise, then rho */
static uint32_t add_exact_round(int sx, u128 mx, int lx, int sy, u128 my, int ly, const o2_params *p)
{
    if (mx == 0 && my == 0) return 0u;
    if (mx == 0) return rho(p, sy, my, ly, 0);
    if (my == 0) return rho(p, sx, mx, lx, 0);
    if (lx < ly) { /* make x the one with the larger last-place exponent */
        int ts = sx; sx = sy; sy = ts; u128 tm = mx; mx = my; my = tm; int tl = lx; lx = ly; ly = tl;
    }
    int d = lx - ly;
    if (bitlen128(my) + 26 > d) {
        /* the terms overlap or nearly do: both magnitudes have at most 50 bits (checked
         * by the caller), so d < 76 and the exact sum fits 127 bits */
        i128 v = (i128)(mx << d) * (sx ? -1 : 1) + (i128)my * (sy ? -1 : 1);
        if (v == 0) return 0u;
        int neg = v < 0;
        return rho(p, neg, (u128)(neg ? -v : v), ly, 0);
    }
    /* |y| < 2^(lx - 26): y lies more than 26 binary places below x's last place, while
     * binary32 rounding boundaries of x + y are multiples of 2^(lx - 25) or coarser;
     * so y only decides on which side of x the sum falls */
    u128 big = mx << 60;
    int st = (sx == sy) ? 1 : -1;
    return rho(p, sx, big, lx - 60, st);
}

/* align magnitude `mag` (units 2^lsb) to units 2^(unit) with truncation toward zero */
static u128 align_rz(u128 mag, int lsb, int unit)
{
    int sh = lsb - unit;
    if (sh >= 0) return mag << sh;
    if (-sh > 127) return 0;
    return mag >> (-sh);
}

/* RD: v (units 2^lsb) to units 2^unit, rounding toward minus infinity */
static i128 align_rd(i128 v, int lsb, int unit)
{
    int sh = lsb - unit;
    if (sh >= 0) return v * ((i128)1 << sh);
    if (-sh > 126) return v < 0 ? -1 : 0;
    i128 q = v / ((i128)1 << (-sh)), r = v % ((i128)1 << (-sh));   /* C division truncates toward zero */
    return (r < 0) ? q - 1 : q;
}

/* the rounding of the second summation step: RD, or RZ for the hypothetical variant of Sec. 6.2.4 */
static i128 align_step(const o2_params *p, i128 v, int lsb, int unit)
{
    if (p->rd_toward_zero && v < 0) return -align_rd(-v, lsb, unit);
    return align_rd(v, lsb, unit);
}

static dec_t dec_in(const o2_params *p, uint32_t bits, int t)
{
    dec_t x = decode(bits, t);
    if (p->ftz_in && x.cls == CLS_SUB) x = decode(0u, t);          /* FlushSubnormal: -> +0.0 */
    return x;
}

/* maximum exponent over the products first, first+stride, ... (count of them); returns 0 when
 * no product takes part (count = 0, or all significands zero and skip_zero_terms set) */
static int part_emax(const o2_params *p, const uint32_t *a, const uint32_t *b, const int *se, uint32_t first, uint32_t stride,
                     uint32_t count, int ta, int tb, int *emax)
{
    int any = 0;
    for (uint32_t q = 0; q < count; ++q) {
        uint32_t k = first + q * stride;
        dec_t x = dec_in(p, a[k], ta), y = dec_in(p, b[k], tb);
        if (p->skip_zero_terms && (x.sig == 0 || y.sig == 0)) continue;
        int e = x.exp + y.exp + (se ? se[k] : 0);               /* ST-FDPA: + Exp(alpha) + Exp(beta) */
        if (!any || e > *emax) *emax = e;
        any = 1;
    }
    return any;
}

/* sum of the same products, each aligned to units of 2^unit with truncation toward zero */
static i128 part_sum(const o2_params *p, const uint32_t *a, const uint32_t *b, const int *se, uint32_t first, uint32_t stride,
                     uint32_t count, int ta, int tb, int unit)
{
    i128 S = 0;
    for (uint32_t q = 0; q < count; ++q) {
        uint32_t k = first + q * stride;
        dec_t x = dec_in(p, a[k], ta), y = dec_in(p, b[k], tb);
        u128 prod = (u128)((uint64_t)x.sig * (uint64_t)y.sig);      /* exact product of significands */
        int e = x.exp + y.exp + (se ? se[k] : 0);                    /* sum of exponents (and of the scales') */
        u128 al = align_rz(prod, e - FMT[ta].mbits - FMT[tb].mbits, unit);
        if (x.sign ^ y.sign) S -= (i128)al; else S += (i128)al;
    }
    return S;
}

/* The rounded sum with the accumulator (Algorithm "TR-FDPA" steps 3-4, "GTR-FDPA" steps 4-5):
 * T counts units of 2^unit_T (T = 0 and have_T = 0 when no product took part). */
static uint32_t rounded_sum_with_c(const o2_params *p, int have_T, i128 T, int emax, int unit_T, dec_t dc, int special_truncation)
{
    const int F = (int)p->frac_bits, F2 = (int)p->frac_bits2;
    const int Fc = p->frac_bits_acc ? (int)p->frac_bits_acc : F;
    /* the accumulator always takes part, a zero one with the exponent of the subnormals, -126 */
    const int E = (have_T && emax > dc.exp) ? emax : dc.exp;
    i128 sc = dc.sign ? -(i128)dc.sig : (i128)dc.sig;
    i128 sc2 = align_step(p, sc, dc.exp - 23, E - Fc);
    if (special_truncation && dc.exp < E - Fc - 1) sc2 = 0;
    const int unit_c = E - Fc;
    if (have_T && p->sum_drop_distance && E - emax >= (int)p->sum_drop_distance) have_T = 0;   /* T' = 0 */
    if (!have_T) { T = 0; unit_T = unit_c; }
    i128 S; int unit;
    if (p->f2_at_leading_bit) {
        /* exact sum first.  If T lies far below the accumulator's unit it is first rounded down to
         * units of 2^(unit_c - 64): rounding down in two steps equals rounding down once. */
        if (unit_c - unit_T > 64) { T = align_step(p, T, unit_T, unit_c - 64); unit_T = unit_c - 64; }
        unit = unit_T < unit_c ? unit_T : unit_c;
        S = T * ((i128)1 << (unit_T - unit)) + sc2 * ((i128)1 << (unit_c - unit));
        if (S == 0) return 0u;
        int lead = bitlen128((u128)(S < 0 ? -S : S)) - 1 + unit;
        if (lead < -126) lead = -126;                     /* no lower than binary32's smallest normal exponent */
        if (lead - F2 > unit) { S = align_step(p, S, unit, lead - F2); unit = lead - F2; }
    } else {
        i128 T2 = align_step(p, T, unit_T, E - F2);
        unit = (E - F2) < unit_c ? (E - F2) : unit_c;
        S = T2 * ((i128)1 << ((E - F2) - unit)) + sc2 * ((i128)1 << (unit_c - unit));
    }
    int neg = S < 0;
    return to_fp32(neg, (u128)(neg ? -S : S), unit, 0, (int)p->out_round);
}

static uint32_t finish(const o2_params *p, uint32_t d)
{
    if (p->acc_fp16) {
        if (p->ftz_out && (d & 0x7C00u) == 0) d &= 0x8000u;
        if (p->zero_result_positive && (d & 0x7FFFu) == 0) d = 0u;
        return d;
    }
    if (p->out_mant_bits == 13) d &= 0xFFFFFC00u;         /* RZ-E8M13: the low 10 mantissa bits cut, toward zero */
    if (p->ftz_out && (d & 0x7F800000u) == 0) d &= 0x80000000u;
    if (p->zero_result_positive && (d & 0x7FFFFFFFu) == 0) d = 0u;
    return d;
}

#define SCALE_NAN (-100000)          /* entry of the scale-exponent array for a NaN scale (E8M0 pattern 0xFF) */

/* the NaN pattern of the output type (binary16: the low half of nan_bits) */
static uint32_t nan_out(const o2_params *p) { return p->acc_fp16 ? (p->nan_bits & 0xFFFFu) : p->nan_bits; }

/* the accumulator as sign, Exp and a 24-bit significand (value = sig 2^(exp - 23)); a binary16 accumulator keeps its own
 * exponent range (Exp = -14 for zero and subnormals) and its 11-bit significand is moved up by 13 places */
static dec_t dec_acc(const o2_params *p, uint32_t c)
{
    if (!p->acc_fp16) return dec_in(p, c, T_FP32);
    dec_t d = dec_in(p, c & 0xFFFFu, T_FP16);
    d.sig <<= 13;
    return d;
}

static uint32_t fdpa_group(const o2_params *p, const uint32_t *a, const uint32_t *b, const int *se, uint32_t c,
                           uint32_t L, int ta, int tb)
{
    if (se) for (uint32_t k = 0; k < L; ++k) if (se[k] == SCALE_NAN) return nan_out(p);
    const int F = (int)p->frac_bits;
    const int fa = FMT[ta].mbits, fb = FMT[tb].mbits;
    uint32_t c_mode = p->c_mode, split = p->split, trunc = p->acc_special_truncation;
    if (c_mode == C_AFTER_RD_EVEN_ODD) { c_mode = C_AFTER_RD; split = 1; trunc = 1; }   /* GTR-FDPA by name */
    dec_t dc = dec_acc(p, c);

    if (p->nan_propagate) {      /* payload rule, in its order of precedence; what it leaves goes on below */
        for (uint32_t k = 0; k < L; ++k) {
            if (dec_in(p, a[k], ta).cls == CLS_NAN) return a[k] | 0x00400000u;
            if (dec_in(p, b[k], tb).cls == CLS_NAN) return b[k] | 0x00400000u;
        }
        for (uint32_t k = 0; k < L; ++k) {
            dec_t x = dec_in(p, a[k], ta), y = dec_in(p, b[k], tb);
            if ((x.cls == CLS_INF && y.cls == CLS_ZERO) || (y.cls == CLS_INF && x.cls == CLS_ZERO)) return nan_out(p);
        }
        if (dc.cls == CLS_NAN) return c | 0x00400000u;
    }
    /* special values (Sec. 4.2) */
    int any_nan = dc.cls == CLS_NAN, pinf = 0, ninf = 0;
    for (uint32_t k = 0; k < L; ++k) {
        dec_t x = dec_in(p, a[k], ta), y = dec_in(p, b[k], tb);
        if (x.cls == CLS_NAN || y.cls == CLS_NAN) any_nan = 1;
        else if (x.cls == CLS_INF || y.cls == CLS_INF) {
            if (x.cls == CLS_ZERO || y.cls == CLS_ZERO) any_nan = 1;
            else if (x.sign ^ y.sign) ninf = 1; else pinf = 1;
        } else if (c_mode == C_AFTER_RD && !p->wide_products) {       /* product overflow, Sec. 4.2 */
            uint64_t prod = (uint64_t)x.sig * (uint64_t)y.sig;
            if (prod && bitlen128((u128)prod) - 1 + x.exp + y.exp + (se ? se[k] : 0) - fa - fb >= 128) { if (x.sign ^ y.sign) ninf = 1; else pinf = 1; }
        }
    }
    if (dc.cls == CLS_INF) { if (dc.sign) ninf = 1; else pinf = 1; }
    if (any_nan || (pinf && ninf)) return nan_out(p);
    if (pinf) return p->acc_fp16 ? 0x7C00u : 0x7F800000u;
    if (ninf) return p->acc_fp16 ? 0xFC00u : 0xFF800000u;

    if (c_mode == C_AFTER_RD) {
        if (split == 0) {
            int emax = 0;
            int have = part_emax(p, a, b, se, 0, 1, L, ta, tb, &emax);
            i128 T = have ? part_sum(p, a, b, se, 0, 1, L, ta, tb, emax - F) : 0;
            return finish(p, rounded_sum_with_c(p, have, T, emax, emax - F, dc, (int)trunc));
        }
        /* sub-groups: even / odd products (split 1), first / second half (split 2), or the four quarters (split 3) */
        const int Fm = p->frac_bits_merge ? (int)p->frac_bits_merge : F;
        const int np_ = split == 3 ? 4 : 2;
        const uint32_t len = L / (uint32_t)np_, stride = split == 1 ? 2u : 1u;
        int e_part[4] = {0, 0, 0, 0}, have[4] = {0, 0, 0, 0}, emax = 0, any = 0;
        i128 T_part[4] = {0, 0, 0, 0};
        for (int g = 0; g < np_; ++g) {
            const uint32_t first = split == 1 ? (uint32_t)g : (uint32_t)g * len;
            have[g] = part_emax(p, a, b, se, first, stride, len, ta, tb, &e_part[g]);
            if (!have[g]) continue;
            T_part[g] = part_sum(p, a, b, se, first, stride, len, ta, tb, e_part[g] - F);
            if (!any || e_part[g] > emax) emax = e_part[g];
            any = 1;
        }
        i128 T = 0;
        for (int g = 0; g < np_; ++g)
            if (have[g]) T += align_step(p, T_part[g], e_part[g] - F, emax - Fm);
        return finish(p, rounded_sum_with_c(p, any, T, emax, emax - Fm, dc, (int)trunc));
    }

    int emax = 0;
    int have = part_emax(p, a, b, se, 0, 1, L, ta, tb, &emax);
    if (c_mode == C_IN_GROUP) {
        if (!have || dc.exp > emax) emax = dc.exp;       /* the accumulator always takes part */
        const int unit = emax - F;
        i128 S = part_sum(p, a, b, se, 0, 1, L, ta, tb, unit);
        u128 al = align_rz((u128)dc.sig, dc.exp - 23, unit);
        if (dc.sign) S -= (i128)al; else S += (i128)al;
        int neg = S < 0;
        return finish(p, rho(p, neg, (u128)(neg ? -S : S), unit, 0));
    }
    /* C_AFTER_EXACT */
    if (!have) emax = 0;
    const int unit = emax - F;
    i128 S = part_sum(p, a, b, se, 0, 1, L, ta, tb, unit);
    int neg = S < 0;
    return finish(p, add_exact_round(neg, (u128)(neg ? -S : S), unit, dc.sign, (u128)dc.sig, dc.exp - 23, p));
}

/* ---- Algorithm "Phi_FTZ-AddMul" (Sec. 4.1.1) on the host's own binary32 arithmetic -------------------------
 * The host's float + and * are RNE-FP32 of the exact result (IEEE-754 basic operations; the file is built without
 * contraction or extended intermediate precision), which is what Algorithm "FTZ-Add and FTZ-Mul" asks for; the
 * flush of results below 2^-126 and the NaN encoding are applied by hand. */
static float f_of(uint32_t b) { float f; memcpy(&f, &b, 4); return f; }
static uint32_t b_of(float f) { uint32_t b; memcpy(&b, &f, 4); return b; }

static uint32_t ftz_fix(const o2_params *p, float z)
{
    uint32_t b = b_of(z);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return p->nan_bits;
    if ((b & 0x7F800000u) == 0) b &= 0x80000000u;           /* |z| < 2^-126: zero, sign kept */
    return b;
}

/* operand of type t (flushed if subnormal) as a float: every FP8 / FP16 / BF16 value is a binary32 number */
static float operand_as_float(uint32_t bits, int t)
{
    dec_t x = decode(bits, t);
    if (x.cls == CLS_NAN) return NAN;
    if (x.cls == CLS_INF) return x.sign ? -INFINITY : INFINITY;
    if (x.cls == CLS_SUB || x.cls == CLS_ZERO) return x.cls == CLS_ZERO && x.sign ? -0.0f : 0.0f;   /* FlushSubnormal: +0.0 */
    float v = ldexpf((float)x.sig, x.exp - FMT[t].mbits);
    return x.sign ? -v : v;
}

static uint32_t addmul_element(const o2_params *p, const void *A, const void *B, uint32_t c,
                               size_t arow, size_t brow, uint32_t k, int ta, int tb)
{
    const uint32_t P = p->group_len;
    uint32_t d = c;
    if ((d & 0x7F800000u) == 0 && (d & 0x007FFFFFu)) d = 0u;      /* subnormal accumulator -> +0.0 */
    if ((d & 0x7FFFFFFFu) > 0x7F800000u) d = p->nan_bits;
    for (uint32_t k0 = 0; k0 < k; k0 += P) {
        uint32_t pr[4];
        for (uint32_t l = 0; l < P; ++l) {
            volatile float x = operand_as_float(load_elem(A, arow + k0 + l, ta), ta);
            volatile float y = operand_as_float(load_elem(B, brow + k0 + l, tb), tb);
            volatile float z = x * y;
            pr[l] = ftz_fix(p, z);
        }
        volatile float s0 = f_of(pr[0]) + f_of(pr[1]);
        uint32_t s = ftz_fix(p, s0);
        if (P == 4) {
            volatile float s1 = f_of(pr[2]) + f_of(pr[3]);
            uint32_t s2 = ftz_fix(p, s1);
            volatile float s3 = f_of(s) + f_of(s2);
            s = ftz_fix(p, s3);
        }
        volatile float dn = f_of(d) + f_of(s);
        d = ftz_fix(p, dn);
    }
    return d;
}

static int check(const o2_params *p, uint32_t k, int ta, int tb, uint32_t *L_out)
{
    if (ta < 0 || tb < 0 || ta > T_TF32 || tb > T_TF32 || ta == T_E8M0 || tb == T_E8M0) return -2;
    if (p->family == 1) {
        if (p->acc_fp16) return -2;
        if (p->group_len != 2 && p->group_len != 4) return -2;
        if (k == 0 || k > (1u << 20) || k % p->group_len) return -3;
        *L_out = p->group_len;
        return 0;
    }
    if (p->family > 1) return -2;
    if (p->acc_fp16 && (p->c_mode >= C_AFTER_RD || p->out_mant_bits != 23)) return -2;
    if (p->nan_propagate && (ta != T_FP32 || tb != T_FP32 || p->acc_fp16)) return -2;
    if (p->out_mant_bits != 23 && !(p->out_mant_bits == 13 && p->out_round == R_RZ)) return -2;
    if (p->align_round != 0 || p->c_mode > 3 || p->out_round > 1 || p->frac_bits > 64) return -2;
    if (k == 0 || k > (1u << 20)) return -3;
    uint32_t L = (p->group_len == 0 || p->group_len > k) ? k : p->group_len;
    if (k % L) return -3;
    if (p->c_mode == C_AFTER_EXACT) {   /* add_exact_round() needs magnitudes of at most 50 bits */
        int lg = 0; while ((1u << lg) < L) ++lg;
        if ((int)p->frac_bits + 2 + lg > 50) return -2;
    }
    if (p->c_mode >= C_AFTER_RD) {      /* keep every intermediate of the RD steps below 2^126 */
        int lg = 0; while ((1u << lg) < L) ++lg;
        uint32_t fmax = p->frac_bits;
        if (p->frac_bits2 > fmax) fmax = p->frac_bits2;
        if (p->frac_bits_merge > fmax) fmax = p->frac_bits_merge;
        if (p->frac_bits_acc > fmax) fmax = p->frac_bits_acc;
        if (fmax > 48 || lg > 20) return -2;
        uint32_t fc = p->frac_bits_acc ? p->frac_bits_acc : p->frac_bits;
        if (p->frac_bits2 > fc + 40) return -2;                 /* see rounded_sum_with_c(), two-step rounding */
        uint32_t split = p->c_mode == C_AFTER_RD_EVEN_ODD ? 1u : p->split;
        if (split > 3) return -2;
        if ((split && (L & 1)) || (split == 3 && (L & 3))) return -3;
    }
    *L_out = L;
    return 0;
}

/* block scales of the call (NULL pointers: none): SA[rows of A][k / block], SB[rows of B][k / block], E8M0 bytes */
typedef struct { const uint8_t *sa, *sb; uint32_t block; } scales_t;
static const scales_t NO_SCALES = {0, 0, 1};

static uint32_t element(const o2_params *p, const void *A, const void *B, uint32_t c,
                        size_t arow, size_t brow, uint32_t k, uint32_t L, int ta, int tb,
                        uint32_t *abuf, uint32_t *bbuf, int *sebuf, scales_t sc)
{
    uint32_t d = c;
    for (uint32_t k0 = 0; k0 < k; k0 += L) {
        for (uint32_t q = 0; q < L; ++q) {
            abuf[q] = load_elem(A, arow + k0 + q, ta);
            bbuf[q] = load_elem(B, brow + k0 + q, tb);
            if (sc.sa) {
                uint32_t xa = sc.sa[(arow / k) * (k / sc.block) + (k0 + q) / sc.block];
                uint32_t xb = sc.sb[(brow / k) * (k / sc.block) + (k0 + q) / sc.block];
                sebuf[q] = (xa == 0xFF || xb == 0xFF) ? SCALE_NAN : ((int)xa - 127) + ((int)xb - 127);
            }
        }
        d = fdpa_group(p, abuf, bbuf, sc.sa ? sebuf : 0, d, L, ta, tb);
    }
    return d;
}

/* D[b][i][j] for A[b][m][k], B[b][n][k], C[b][m][n].  Returns 0, or a negative code
 * (-2 unsupported parameter, -3 bad shape).  *threads_used receives the team size. */
static int emulate_mma_impl(const o2_params *p, const void *A, const void *B, const uint32_t *C, uint32_t *D,
                            uint32_t m, uint32_t n, uint32_t k, uint64_t batch, int ta, int tb,
                            int nthreads, int *threads_used, scales_t sc)
{
    uint32_t L;
    int rc = check(p, k, ta, tb, &L);
    if (rc) return rc;
    if (sc.sa && (p->family != 0 || sc.block == 0 || k % sc.block)) return -3;
    if (nthreads > 0) omp_set_num_threads(nthreads);
    int used = 1;
    int64_t rows = (int64_t)batch * m;
    int nomem = 0;
#pragma omp parallel
    {
        /* one group's operands per thread, on the heap: L goes up to 2^20, far beyond a thread's stack */
        uint32_t *abuf = malloc((size_t)L * 4), *bbuf = malloc((size_t)L * 4); int *sebuf = malloc((size_t)L * sizeof(int));
        if (!abuf || !bbuf || !sebuf) {
#pragma omp atomic write
            nomem = 1;
        }
#pragma omp barrier
#pragma omp single
        used = omp_get_num_threads();
#pragma omp for schedule(dynamic, 4)
        for (int64_t r = 0; r < rows; ++r) {
            if (nomem) continue;
            uint64_t t = (uint64_t)r / m; uint32_t i = (uint32_t)((uint64_t)r % m);
            for (uint32_t j = 0; j < n; ++j) {
                size_t o = ((size_t)t * m + i) * n + j;
                D[o] = p->family == 1 ? addmul_element(p, A, B, C[o], ((size_t)t * m + i) * k, ((size_t)t * n + j) * k, k, ta, tb)
                                      : element(p, A, B, C[o], ((size_t)t * m + i) * k, ((size_t)t * n + j) * k, k, L, ta, tb, abuf, bbuf, sebuf, sc);
            }
        }
        free(abuf); free(bbuf); free(sebuf);
    }
    if (threads_used) *threads_used = used;
    return nomem ? -4 : 0;
}

int o2_emulate_mma(const o2_params *p, const void *A, const void *B, const uint32_t *C, uint32_t *D,
                   uint32_t m, uint32_t n, uint32_t k, uint64_t batch, int ta, int tb,
                   int nthreads, int *threads_used)
{
    return emulate_mma_impl(p, A, B, C, D, m, n, k, batch, ta, tb, nthreads, threads_used, NO_SCALES);
}

/* Algorithm "ST-FDPA": the same with E8M0 block scales SA[batch][m][k / block], SB[batch][n][k / block]. */
int o2_emulate_mma_scaled(const o2_params *p, const void *A, const void *B, const uint32_t *C, uint32_t *D,
                          const uint8_t *SA, const uint8_t *SB, uint32_t block,
                          uint32_t m, uint32_t n, uint32_t k, uint64_t batch, int ta, int tb,
                          int nthreads, int *threads_used)
{
    scales_t sc = {SA, SB, block};
    if (!SA || !SB) return -3;
    return emulate_mma_impl(p, A, B, C, D, m, n, k, batch, ta, tb, nthreads, threads_used, sc);
}

/* ---- Algorithm "GST-FDPA" (Sec. 4.1.3): FP4 operands, one scale factor pair per k_block elements, exact dot product
 * per group of G products, truncated fused sum of the L / G group terms and the accumulator.  Integer form: an FP4
 * value is sig * 2^(exp - 1) with sig in 0..3, so a product counts units of 2^-2; a scale significand counts units of
 * 2^-3 (UE4M3; E8M0's 1.0 is 8 of them), so s_g counts units of 2^-8. */
typedef struct { uint32_t L, G, k_block, F, out_round, scale_format, nan_bits; } gst_params;

static int gst_scale(uint32_t code, uint32_t fmt, int *sig8, int *exp)
{
    code &= 0xFFu;
    if (fmt == 0) { if (code == 0xFF) return 0; *sig8 = 8; *exp = (int)code - 127; return 1; }
    dec_t d = decode(code & 0x7Fu, T_E4M3);
    if (d.cls == CLS_NAN) return 0;
    *sig8 = (int)d.sig; *exp = d.exp;
    return 1;
}

static uint32_t gst_group_op(const gst_params *g, const uint8_t *a, const uint8_t *b, uint32_t c, const uint8_t *al, const uint8_t *be)
{
    dec_t dc = decode(c, T_FP32);
    if (dc.cls == CLS_NAN) return g->nan_bits;
    const uint32_t ng = g->L / g->G;
    int64_t s[65]; int e[65];
    for (uint32_t q = 0; q < ng; ++q) {
        int sa, ea, sb, eb;
        const uint32_t blk = q * g->G / g->k_block;
        if (!gst_scale(al[blk], g->scale_format, &sa, &ea) || !gst_scale(be[blk], g->scale_format, &sb, &eb)) return g->nan_bits;
        int64_t p = 0;
        for (uint32_t k = q * g->G; k < (q + 1) * g->G; ++k) {
            dec_t x = decode(a[k], T_E2M1), y = decode(b[k], T_E2M1);
            int64_t t = (int64_t)(x.sig * y.sig) << (x.exp + y.exp);          /* units of 2^-2 */
            p += (x.sign ^ y.sign) ? -t : t;
        }
        s[q] = p * sa * sb;                                                   /* units of 2^-8 */
        e[q] = ea + eb;
    }
    if (dc.cls == CLS_INF) return dc.sign ? 0xFF800000u : 0x7F800000u;
    int emax = dc.exp;
    for (uint32_t q = 0; q < ng; ++q) if (e[q] > emax) emax = e[q];
    const int F = (int)g->F;
    i128 S = 0;
    for (uint32_t q = 0; q < ng; ++q) {
        u128 mag = (u128)(s[q] < 0 ? -s[q] : s[q]);
        u128 al_ = align_rz(mag, e[q] - 8, emax - F);
        if (s[q] < 0) S -= (i128)al_; else S += (i128)al_;
    }
    u128 ac = align_rz((u128)dc.sig, dc.exp - 23, emax - F);
    if (dc.sign) S -= (i128)ac; else S += (i128)ac;
    int neg = S < 0;
    return to_fp32(neg, (u128)(neg ? -S : S), emax - F, 0, (int)g->out_round);
}

/* D = Phi_GST-FDPA(A, B, C): A[batch][m][k], B[batch][n][k] FP4 codes (one per byte), SA[batch][m][k / k_block],
 * SB[batch][n][k / k_block].  Returns 0, -2 (parameter) or -3 (shape). */
int o2_emulate_gst(const gst_params *g, const uint8_t *A, const uint8_t *B, const uint32_t *C, uint32_t *D,
                   const uint8_t *SA, const uint8_t *SB, uint32_t m, uint32_t n, uint32_t k, uint64_t batch, int nthreads)
{
    gst_params p = *g;
    if (p.L == 0 || p.L > k) p.L = k;
    if (p.G == 0 || p.k_block == 0 || p.F > 64 || p.out_round > 1 || p.scale_format > 1) return -2;
    if (k == 0 || k % p.L || p.L % p.k_block || p.k_block % p.G || p.L / p.G > 64) return -3;
    if (nthreads > 0) omp_set_num_threads(nthreads);
    const uint32_t nblk = k / p.k_block;
    int64_t rows = (int64_t)batch * m;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t r = 0; r < rows; ++r) {
        uint64_t t = (uint64_t)r / m; uint32_t i = (uint32_t)((uint64_t)r % m);
        for (uint32_t j = 0; j < n; ++j) {
            size_t o = ((size_t)t * m + i) * n + j;
            const uint8_t *a = A + ((size_t)t * m + i) * k, *b = B + ((size_t)t * n + j) * k;
            const uint8_t *al = SA + ((size_t)t * m + i) * nblk, *be = SB + ((size_t)t * n + j) * nblk;
            uint32_t d = C[o];
            for (uint32_t k0 = 0; k0 < k; k0 += p.L)
                d = gst_group_op(&p, a + k0, b + k0, d, al + k0 / p.k_block, be + k0 / p.k_block);
            D[o] = d;
        }
    }
    return 0;
}

/* The same, only at the flattened output indices idx[0..count) (index = (b*m + i)*n + j). */
int o2_emulate_sample(const o2_params *p, const void *A, const void *B, const uint32_t *C,
                      const uint64_t *idx, uint64_t count, uint32_t *D_sample,
                      uint32_t m, uint32_t n, uint32_t k, uint64_t batch, int ta, int tb,
                      int nthreads, int *threads_used)
{
    uint32_t L;
    int rc = check(p, k, ta, tb, &L);
    if (rc) return rc;
    for (uint64_t s = 0; s < count; ++s) if (idx[s] >= batch * m * n) return -3;
    if (nthreads > 0) omp_set_num_threads(nthreads);
    int used = 1;
    int nomem = 0;
#pragma omp parallel
    {
        uint32_t *abuf = malloc((size_t)L * 4), *bbuf = malloc((size_t)L * 4); int *sebuf = malloc((size_t)L * sizeof(int));
        const scales_t sc = NO_SCALES;
        if (!abuf || !bbuf || !sebuf) {
#pragma omp atomic write
            nomem = 1;
        }
#pragma omp barrier
#pragma omp single
        used = omp_get_num_threads();
#pragma omp for schedule(dynamic, 16)
        for (int64_t s = 0; s < (int64_t)count; ++s) {
            if (nomem) continue;
            uint64_t o = idx[s];
            uint64_t t = o / ((uint64_t)m * n);
            uint32_t i = (uint32_t)((o / n) % m), j = (uint32_t)(o % n);
            D_sample[s] = p->family == 1 ? addmul_element(p, A, B, C[o], ((size_t)t * m + i) * k, ((size_t)t * n + j) * k, k, ta, tb)
                                         : element(p, A, B, C[o], ((size_t)t * m + i) * k, ((size_t)t * n + j) * k, k, L, ta, tb, abuf, bbuf, sebuf, sc);
        }
        free(abuf); free(bbuf); free(sebuf);
    }
    if (threads_used) *threads_used = used;
    return nomem ? -4 : 0;
}

/* Exact dot products (C = 0) and the error of D against them, at flattened indices
 * 0, stride, 2*stride, ... of one m x n output (A[m][k], B[n][k]).  Only FP8 operand
 * pairs: every product is a multiple of 2^-(32) below 2^33, so a signed 128-bit
 * accumulator in units of 2^lsb0 is exact for any k <= 2^20.
 *
 * int_out[0..4] = n_samples, n_equal_rne, n_above, n_below; int_out[4..38) = ulp_hist[34]
 * dbl_out[0..5) = sum_abs_err, max_abs_err, sum_rel_err, max_rel_err, sum_signed_err */
static int64_t okey(uint32_t b) { return (b & 0x80000000u) ? -(int64_t)(b & 0x7FFFFFFFu) : (int64_t)b; }

static long double ld_of(int neg, u128 mag, int lsb)
{
    long double v = ldexpl((long double)(uint64_t)(mag >> 64), 64) + (long double)(uint64_t)mag;
    v = ldexpl(v, lsb);
    return neg ? -v : v;
}

int o2_exact_dot_stats(const void *A, const void *B, const uint32_t *D, uint32_t m, uint32_t n, uint32_t k,
                       int ta, int tb, uint64_t stride, uint64_t *int_out, double *dbl_out)
{
    if (ta > T_E5M2 || tb > T_E5M2 || ta < 0 || tb < 0) return -2;
    if (stride == 0 || k == 0 || k > (1u << 20)) return -3;
    const int lsb0 = (1 - FMT[ta].bias - FMT[ta].mbits) + (1 - FMT[tb].bias - FMT[tb].mbits);
    memset(int_out, 0, 38 * sizeof(uint64_t));
    long double sabs = 0, srel = 0, ssgn = 0, mabs = 0, mrel = 0;
    for (uint64_t o = 0; o < (uint64_t)m * n; o += stride) {
        uint32_t i = (uint32_t)(o / n), j = (uint32_t)(o % n);
        i128 acc = 0;
        for (uint32_t q = 0; q < k; ++q) {
            dec_t x = decode(load_elem(A, (size_t)i * k + q, ta), ta);
            dec_t y = decode(load_elem(B, (size_t)j * k + q, tb), tb);
            if (x.cls >= CLS_INF || y.cls >= CLS_INF) return -2;
            int sh = (x.exp - FMT[ta].mbits) + (y.exp - FMT[tb].mbits) - lsb0;   /* >= 0 */
            i128 pr = (i128)((uint64_t)x.sig * y.sig) << sh;
            acc += (x.sign ^ y.sign) ? -pr : pr;
        }
        int neg = acc < 0; u128 mag = (u128)(neg ? -acc : acc);
        uint32_t r = to_fp32(neg, mag, lsb0, 0, R_RNE);
        uint32_t d = D[o];
        if ((d & 0x7FFFFFFFu) > 0x7F800000u) return -2;
        int_out[0] += 1;
        if (d == r) int_out[1] += 1;
        int64_t kd = okey(d), kr = okey(r);
        if (kd > kr) int_out[2] += 1; else if (kd < kr) int_out[3] += 1;
        uint64_t dist = (uint64_t)(kd > kr ? kd - kr : kr - kd);
        int_out[4 + (dist ? 64 - __builtin_clzll(dist) : 0)] += 1;
        /* D - exact, exactly: D = sig * 2^(e-23) */
        dec_t dd = decode(d, T_FP32);
        if (dd.cls == CLS_INF) return -2;
        int ld = dd.exp - 23;
        int lo = ld < lsb0 ? ld : lsb0;
        if (ld - lo > 60 || lsb0 - lo > 30) return -2;   /* cannot happen for FP32 D near the exact value */
        i128 dv = (i128)dd.sig << (ld - lo); if (dd.sign) dv = -dv;
        i128 ev = acc << (lsb0 - lo);
        i128 err = dv - ev;
        int eneg = err < 0; u128 emag = (u128)(eneg ? -err : err);
        long double e_ld = ld_of(eneg, emag, lo);
        long double ae = fabsl(e_ld);
        sabs += ae; ssgn += e_ld; if (ae > mabs) mabs = ae;
        if (mag != 0) {
            long double rel = ae / ld_of(0, mag, lsb0);
            srel += rel; if (rel > mrel) mrel = rel;
        }
    }
    dbl_out[0] = (double)sabs; dbl_out[1] = (double)mabs; dbl_out[2] = (double)srel;
    dbl_out[3] = (double)mrel; dbl_out[4] = (double)ssgn;
    return 0;
}
