// Internal declarations shared by the translation units of libmmaemu.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "mmaemu.h"

namespace mmaemu {

// Operand encodings (OCP FP8, IEEE binary16, bfloat16, binary32).
template <int T> struct Fmt;
// W: storage width; IEEE: exponent field all ones is Inf / NaN; NOSPEC: every code is finite (else, without IEEE, the
// E4M3 rule: one NaN code)
template <> struct Fmt<MMAEMU_FP8_E4M3> { static constexpr int EB = 4, MB = 3, BIAS = 7, W = 8; static constexpr bool IEEE = false, NOSPEC = false; using elem = uint8_t; };
template <> struct Fmt<MMAEMU_FP8_E5M2> { static constexpr int EB = 5, MB = 2, BIAS = 15, W = 8; static constexpr bool IEEE = true, NOSPEC = false; using elem = uint8_t; };
template <> struct Fmt<MMAEMU_FP16> { static constexpr int EB = 5, MB = 10, BIAS = 15, W = 16; static constexpr bool IEEE = true, NOSPEC = false; using elem = uint16_t; };
template <> struct Fmt<MMAEMU_BF16> { static constexpr int EB = 8, MB = 7, BIAS = 127, W = 16; static constexpr bool IEEE = true, NOSPEC = false; using elem = uint16_t; };
template <> struct Fmt<MMAEMU_FP32> { static constexpr int EB = 8, MB = 23, BIAS = 127, W = 32; static constexpr bool IEEE = true, NOSPEC = false; using elem = uint32_t; };
template <> struct Fmt<MMAEMU_FP6_E2M3> { static constexpr int EB = 2, MB = 3, BIAS = 1, W = 8; static constexpr bool IEEE = false, NOSPEC = true; using elem = uint8_t; };
template <> struct Fmt<MMAEMU_FP6_E3M2> { static constexpr int EB = 3, MB = 2, BIAS = 3, W = 8; static constexpr bool IEEE = false, NOSPEC = true; using elem = uint8_t; };
template <> struct Fmt<MMAEMU_TF32> { static constexpr int EB = 8, MB = 10, BIAS = 127, W = 32; static constexpr bool IEEE = true, NOSPEC = false; using elem = uint32_t; };   // fields after dropping the low 13 bits
template <> struct Fmt<MMAEMU_FP4_E2M1> { static constexpr int EB = 2, MB = 1, BIAS = 1, W = 8; static constexpr bool IEEE = false, NOSPEC = true; using elem = uint8_t; };

struct FmtInfo { int ebits, mbits, bias, width; bool ieee, nospec; };      // width: storage bits
inline FmtInfo fmt_info(uint32_t t)
{
    switch (t) {
    case MMAEMU_FP8_E4M3: return {4, 3, 7, 8, false, false};
    case MMAEMU_FP8_E5M2: return {5, 2, 15, 8, true, false};
    case MMAEMU_FP16: return {5, 10, 15, 16, true, false};
    case MMAEMU_BF16: return {8, 7, 127, 16, true, false};
    case MMAEMU_E8M0: return {8, 0, 127, 8, false, true};
    case MMAEMU_FP6_E2M3: return {2, 3, 1, 8, false, true};
    case MMAEMU_FP6_E3M2: return {3, 2, 3, 8, false, true};
    case MMAEMU_FP4_E2M1: return {2, 1, 1, 8, false, true};
    case MMAEMU_TF32: return {8, 10, 127, 32, true, false};
    default: return {8, 23, 127, 32, true, false};
    }
}
inline bool is_narrow_type(uint32_t t) { return t == MMAEMU_FP6_E2M3 || t == MMAEMU_FP6_E3M2 || t == MMAEMU_FP4_E2M1; }   // FP6 / FP4
inline bool is_byte_type(uint32_t t) { return t <= MMAEMU_FP8_E5M2 || is_narrow_type(t); }

enum : uint32_t {
    FL_RZ = 1u, FL_FTZ_OUT = 2u, FL_ZERO_POSITIVE = 4u, FL_FTZ_IN = 8u, FL_SPECIAL_TRUNC = 16u, FL_F2_LEADING = 32u,
    FL_SKIP_ZERO = 64u, FL_WIDE_PRODUCTS = 128u,
    FL_ACC16 = 256u,     // accumulator and output are binary16 (C and D hold 16-bit patterns)
    FL_NAN_PROPAGATE = 512u,  // FP32 operands: a NaN result carries an operand's payload (general kernel only)
    FL_RD_AS_RZ = 1024u       // RD modes: the round-downs of the summation truncate toward zero (Sec. 6.2.4's hypothetical variant)
};

// Model parameters as the kernels take them (by value).
struct ModelArgs {
    uint32_t L;          // group length actually used: min(K, L_max)
    int32_t F;           // fractional bits of the aligned terms
    int32_t F2;          // fractional bits kept of the product sum (TR-FDPA / GTR-FDPA)
    uint32_t c_mode, out_round, ftz_in, ftz_out, nan_bits;
    // variations of the RD mode (c_mode is never C_AFTER_RD_EVEN_ODD here: the entry point rewrites it)
    uint32_t split, acc_special_truncation;
    int32_t Fm, Fc;      // merge and accumulator precisions, already defaulted to F
    uint32_t f2_at_leading_bit, skip_zero_terms, zero_result_positive, wide_products;
    int32_t sum_drop_distance;
    uint32_t rd_toward_zero;
    uint32_t out_mask;   // 0xFFFFFFFF, or 0xFFFFFC00 for the E8M13 output conversion
    uint32_t flags;      // the switches above once more, one FL_* bit each (the tiled kernels test these)
    // FL_ACC16: inside the kernels a binary16 accumulator travels as the binary32 pattern of the same value (every
    // binary16 number is one); nan_bits is then a binary32 quiet NaN and nan16 the pattern written to D for it
    uint32_t nan16;
};

// error plumbing (api.hip)
void set_error(const char *fmt, ...);
void set_last_kernel(const char *fmt, ...);
mmaemu_status hip_fail(hipError_t e, const char *what);
#define MMAEMU_HIP(call)                                            \
    do {                                                            \
        hipError_t e__ = (call);                                    \
        if (e__ != hipSuccess) return ::mmaemu::hip_fail(e__, #call); \
    } while (0)

// launchers implemented in the kernel translation units; all validate nothing (the
// entry points do) and return the launch status
// SA / SB: E8M0 block scales (device), or null for the unscaled operation
mmaemu_status launch_emulate(const ModelArgs &p, const void *A, const void *B, const void *C, void *D,
                             uint32_t m, uint32_t n, uint32_t k, uint64_t batch, uint32_t ta, uint32_t tb,
                             hipStream_t s, const uint8_t *SA = nullptr, const uint8_t *SB = nullptr, uint32_t block = 1);
// Several models over the same operands, each compared with a reference inside the kernel (the closed-loop scan;
// emulate_scan.hip): at most MULTI_MAX models of any group length and width per launch.
constexpr int MULTI_MAX = 16;
struct MultiLaunch {
    uint32_t count;
    uint32_t slot[MULTI_MAX];          // place of each model in the caller's arrays (D_out, statistics)
    ModelArgs models[MULTI_MAX];
    uint32_t kind[MULTI_MAX];          // arithmetic kind of each model, as scan_takes names it
    uint32_t cls;                      // the class all of them belong to, as scan_takes names it
    bool ref_is_first;                 // the first model's outputs are the reference (dref is not read)
    const uint32_t *dref;
    uint32_t *dout;                    // null, or the start of the caller's output array
    uint64_t out_stride, index_base;
    mmaemu_stats *stats;               // the start of the caller's statistics array
};
// scan_takes: whether that kernel takes a model on this problem, and the arithmetic kind the model needs there
// (0: a group's aligned terms summed in 32 bits; 1: folded into binary64 every four terms; 2: every term; 3: F of 30
// and more, terms truncated and summed in binary64), and the class of models that can share its launch
bool scan_takes(const ModelArgs &p, uint32_t ta, uint32_t tb, uint32_t m, uint32_t n, uint32_t k, const void *A, const void *B, uint32_t &kind,
                uint32_t &cls);
mmaemu_status launch_scan(const MultiLaunch &ml, const void *A, const void *B, const void *C, uint32_t m, uint32_t n, uint32_t k,
                          uint64_t batch, uint32_t ta, uint32_t tb, hipStream_t s);
// Algorithm "E-FDPA" in 16 x 16 blocks with the operands shared through LDS (emulate_efdpa.hip); efdpa_blocks_take: whether
// it takes the problem (else the general kernel does)
bool efdpa_blocks_take(const ModelArgs &p, uint32_t ta, uint32_t tb, uint32_t m, uint32_t n, uint32_t k);
mmaemu_status launch_emulate_efdpa(const ModelArgs &p, const void *A, const void *B, const void *C, void *D, uint32_t m, uint32_t n,
                                   uint32_t k, uint64_t batch, uint32_t ta, uint32_t tb, hipStream_t s);
// the same model for any shape and FP32 operands too: one thread per output, the pair alone, then the marked outputs
bool efdpa_pairs_take(const ModelArgs &p, const void *C, const void *D, uint32_t k);
mmaemu_status launch_emulate_efdpa_pairs(const ModelArgs &p, const void *A, const void *B, const void *C, void *D, uint32_t m, uint32_t n,
                                         uint32_t k, uint64_t batch, uint32_t ta, uint32_t tb, hipStream_t s);
mmaemu_status launch_emulate_generic(const ModelArgs &p, const void *A, const void *B, const void *C, void *D,
                                     uint32_t m, uint32_t n, uint32_t k, uint64_t batch, uint32_t ta,
                                     uint32_t tb, hipStream_t s, const uint8_t *SA = nullptr, const uint8_t *SB = nullptr,
                                     uint32_t block = 1);
mmaemu_status launch_emulate_addmul(const ModelArgs &p, const void *A, const void *B, const void *C, void *D,
                                    uint32_t m, uint32_t n, uint32_t k, uint64_t batch, uint32_t ta,
                                    uint32_t tb, hipStream_t s);
// Algorithm "Phi_FMA": binary32 operands and accumulators, a chain of fused multiply-adds in k order
mmaemu_status launch_emulate_fma(const void *A, const void *B, const void *C, void *D, uint32_t m, uint32_t n, uint32_t k,
                                 uint64_t batch, uint32_t nan_bits, bool nan_propagate, hipStream_t s);
// the same chain on binary64 patterns (one v_fma_f64 per step)
mmaemu_status launch_emulate_fma64(const void *A, const void *B, const void *C, void *D, uint32_t m, uint32_t n, uint32_t k,
                                   uint64_t batch, uint32_t nan_bits, bool nan_propagate, hipStream_t s);
// Algorithm "GST-FDPA": FP4 operands, scale codes SA / SB per `block` elements (L, G, F, rho, NaN pattern, scale format)
struct GstArgs { uint32_t L, G, block, F, out_round, scale_format, nan_bits; };
mmaemu_status launch_emulate_gst(const GstArgs &g, const void *A, const void *B, const void *C, void *D, const uint8_t *SA,
                                 const uint8_t *SB, uint32_t m, uint32_t n, uint32_t k, uint64_t batch, hipStream_t s);
mmaemu_status launch_stats_reset(mmaemu_stats *st, hipStream_t s);
mmaemu_status launch_compare(const void *d0, const void *d1, uint64_t count, uint64_t base, bool half,
                             mmaemu_stats *st, hipStream_t s);
mmaemu_status launch_compare64(const void *d0, const void *d1, uint64_t count, uint64_t base, mmaemu_stats *st, hipStream_t s);
mmaemu_status launch_generate(const mmaemu_gen_params &g, void *out, uint32_t dtype, uint64_t ept,
                              uint64_t first_tile, uint64_t n_tiles, void *workspace, hipStream_t s);
// the same with the running maximum of the per-tensor scaling in the library's own static device array
mmaemu_status launch_generate_noalloc(const mmaemu_gen_params &g, void *out, uint32_t dtype, uint64_t ept,
                                      uint64_t first_tile, uint64_t n_tiles, hipStream_t s);
mmaemu_status launch_mfma_probe(uint32_t instr, const void *A, const void *B, const void *C, void *D,
                                uint32_t k, uint64_t batch, hipStream_t s);
mmaemu_status launch_mfma_probe_scaled(uint32_t instr, const void *A, const void *B, const void *C, void *D,
                                       const void *SA, const void *SB, uint32_t k, uint64_t batch, hipStream_t s);
mmaemu_status launch_err_stats_reset(mmaemu_err_stats *st, hipStream_t s);
mmaemu_status launch_exact_dot_sample(const void *A, const void *B, const uint32_t *D, uint32_t m, uint32_t n,
                                      uint32_t k, uint32_t ta, uint32_t tb, uint64_t stride,
                                      mmaemu_err_stats *st, hipStream_t s);
mmaemu_status launch_deviation_reset(mmaemu_deviation_hist *h, hipStream_t s);
mmaemu_status launch_deviation_sample(const void *A, const void *B, const uint32_t *C, const uint32_t *D, uint32_t m, uint32_t n,
                                      uint32_t k, uint64_t batch, uint32_t ta, uint32_t tb, uint64_t stride, int bin_exp,
                                      mmaemu_deviation_hist *h, hipStream_t s);

// issue-rate probes (issue_rate.hip)
uint32_t issue_probe_count();
const char *issue_probe_name(uint32_t op);
mmaemu_status launch_issue_probe(uint32_t op, uint32_t iters, uint32_t workgroups, uint32_t *out, hipStream_t s);

// ---- device helpers -----------------------------------------------------------------
#if defined(__HIPCC__)

// rho (paper Table "Conversion functions"): (-1)^neg * mag * 2^lsb -> binary32 bits, RNE or
// RZ.  `sticky` != 0 means the true magnitude lies strictly between mag and mag + 1 units;
// callers only set it when mag >= 2^60, far above the rounding position.  mag != 0.
__device__ __forceinline__ uint32_t round_to_fp32(uint32_t neg, uint64_t mag, int lsb, uint32_t sticky, uint32_t mode)
{
    const int bl = 64 - __builtin_clzll(mag);
    const int e = bl - 1 + lsb;
    int eg = e < -126 ? -126 : e;
    const int sh = eg - 23 - lsb;
    uint64_t n;
    uint32_t half = 0, rest = sticky;
    if (sh <= 0) {
        n = mag << (-sh);
    } else if (sh >= 64) {
        n = 0;
        if (sh == 64) { half = (uint32_t)(mag >> 63); rest |= (mag << 1) != 0; }
        else rest |= 1u;
    } else {
        n = mag >> sh;
        half = (uint32_t)(mag >> (sh - 1)) & 1u;
        rest |= (mag & ((1ull << (sh - 1)) - 1ull)) != 0;
    }
    if (mode == MMAEMU_ROUND_RNE && half && (rest || (n & 1ull))) n += 1;
    if (n == (1ull << 24)) { n >>= 1; eg += 1; }
    uint32_t out;
    if (eg > 127) out = (mode == MMAEMU_ROUND_RNE) ? 0x7F800000u : 0x7F7FFFFFu;
    else if (n < (1ull << 23)) out = (uint32_t)n;
    else out = ((uint32_t)(eg + 127) << 23) | ((uint32_t)n & 0x7FFFFFu);
    return (neg << 31) | out;
}

// The same onto the binary16 grid (10 mantissa bits, exponents -14 .. 15: rho = RNE-FP16 of the paper's table, or its
// RZ counterpart); the result is returned as the binary32 pattern of that binary16 number.
__device__ __forceinline__ uint32_t round_to_fp16_as_fp32(uint32_t neg, uint64_t mag, int lsb, uint32_t sticky, uint32_t mode)
{
    const int bl = 64 - __builtin_clzll(mag);
    const int e = bl - 1 + lsb;
    int eg = e < -14 ? -14 : e;
    const int sh = eg - 10 - lsb;
    uint64_t n;
    uint32_t half = 0, rest = sticky;
    if (sh <= 0) {
        n = mag << (-sh);
    } else if (sh >= 64) {
        n = 0;
        if (sh == 64) { half = (uint32_t)(mag >> 63); rest |= (mag << 1) != 0; }
        else rest |= 1u;
    } else {
        n = mag >> sh;
        half = (uint32_t)(mag >> (sh - 1)) & 1u;
        rest |= (mag & ((1ull << (sh - 1)) - 1ull)) != 0;
    }
    if (mode == MMAEMU_ROUND_RNE && half && (rest || (n & 1ull))) n += 1;
    if (n == (1ull << 11)) { n >>= 1; eg += 1; }
    uint32_t out;
    if (eg > 15) out = (mode == MMAEMU_ROUND_RNE) ? 0x7F800000u : 0x477FE000u;       // infinity, or 65504
    else if (n == 0) out = 0u;
    else {
        const int nb = 32 - __builtin_clz((uint32_t)n);                              // n < 2^11: value n 2^(eg - 10)
        out = ((uint32_t)(eg - 10 + nb - 1 + 127) << 23) | (((uint32_t)n << (24 - nb)) & 0x7FFFFFu);
    }
    return (neg << 31) | out;
}
__device__ __forceinline__ uint32_t round_out(bool acc16, uint32_t neg, uint64_t mag, int lsb, uint32_t sticky, uint32_t mode)
{
    return acc16 ? round_to_fp16_as_fp32(neg, mag, lsb, sticky, mode) : round_to_fp32(neg, mag, lsb, sticky, mode);
}

// binary16 pattern <-> the binary32 pattern of the same value
__device__ __forceinline__ uint32_t half_bits_to_float_bits(uint32_t h)
{
    _Float16 x;
    const uint16_t hb = (uint16_t)h;
    __builtin_memcpy(&x, &hb, 2);
    return __float_as_uint((float)x);                     // exact; NaN stays NaN
}
__device__ __forceinline__ uint32_t float_bits_to_half_bits(uint32_t f)      // f holds a binary16 number (or inf / NaN)
{
    const _Float16 x = (_Float16)__uint_as_float(f);
    uint16_t hb;
    __builtin_memcpy(&hb, &x, 2);
    return hb;
}

// rho(x + y) with the two-term sum exact: x = (-1)^sx mx 2^lx, y likewise; magnitudes
// below 2^60.  Both are left-justified to bit 62; the smaller is shifted down with the
// lost bits remembered, which happens only when the gap exceeds 3 places, i.e. when at
// most one leading bit can cancel, so the remembered bits stay below the rounding place.
__device__ __forceinline__ uint32_t add_exact_round(uint32_t sx, uint64_t mx, int lx, uint32_t sy, uint64_t my, int ly, uint32_t mode, bool acc16 = false)
{
    if (mx == 0 && my == 0) return 0u;
    if (mx == 0) return round_out(acc16, sy, my, ly, 0, mode);
    if (my == 0) return round_out(acc16, sx, mx, lx, 0, mode);
    int nx = __builtin_clzll(mx) - 1, ny = __builtin_clzll(my) - 1;
    mx <<= nx; lx -= nx;
    my <<= ny; ly -= ny;
    if (lx < ly || (lx == ly && mx < my)) {
        uint64_t tm = mx; mx = my; my = tm;
        int tl = lx; lx = ly; ly = tl;
        uint32_t ts = sx; sx = sy; sy = ts;
    }
    const int g = lx - ly;                 // >= 0; |x| >= |y|
    uint64_t ys; uint32_t lost;
    if (g >= 64) { ys = 0; lost = 1; }
    else { ys = my >> g; lost = (g > 0) && ((my & ((1ull << g) - 1ull)) != 0); }
    uint64_t r;
    if (sx == sy) r = mx + ys;             // true sum in [r, r+1)
    else r = mx - ys - lost;               // true difference in (r, r+1) when lost, == r otherwise
    if (r == 0 && !lost) return 0u;        // exact cancellation -> +0.0
    return round_out(acc16, sx, r, lx, lost, mode);
}

#endif // __HIPCC__
} // namespace mmaemu
