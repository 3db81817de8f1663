// Tiled emulation kernels: the fast path of mmaemu_emulate_mma.
//
// What is computed is the chained FDPA model (paper Algorithm "Phi_FDPA") around the
// truncated fused dot-product-add (Algorithm "T-FDPA"); how it is computed is specific
// to CDNA4:
//
//   * A workgroup of 256 threads owns a block of D (one TMxTN block of a large problem,
//     or several whole 16x16 / 32x32 tiles of a batch); each thread owns an RxC register
//     block of D elements (outputs are independent: paper Sec. 3.1 Step 1).
//   * A and B are decoded once per workgroup while being staged into LDS: each element
//     becomes its exact binary32 value and a 16-bit biased copy of its unnormalised
//     exponent e' = max(E, 1) - 1.  Two exponents share one LDS dword.
//   * Pass 1 per group, e_max: packed 16-bit add and max (two products per instruction).
//   * Pass 2 per group: the product a*b is exact in binary32 (<= 22 significant bits);
//     multiplying by 2^(F - e_max) aligns it, and the float->int conversion truncates
//     toward zero -- exactly RZ_F of the paper.  Terms are summed in a 32-bit integer for
//     as many terms as cannot overflow, then folded exactly into a binary64 accumulator.
//   * rho: the integer sum times 2^(e_max - F) is exact in binary64; one hardware
//     binary64->binary32 conversion gives RNE with gradual underflow and overflow.
//     With the accumulator outside the truncated sum (C_AFTER_EXACT) the exact two-term
//     sum is formed by an error-free binary64 addition whose result is rounded to odd
//     when inexact, so that the conversion to binary32 still rounds once.
//
// Value modes (template parameter VM):
//   0  binary32 values only: FP8 / FP16 operands, whose products always fit binary32;
//   1  adaptive: BF16 operands.  A staged chunk whose elements all lie in [2^-31, 2^32) (or
//      are zero) is handled in binary32 as above; a chunk with any element outside that
//      range is staged as binary64 values and pass 2 runs in binary64 (product and
//      alignment exact for any finite operands), still truncating with the float->int
//      conversion;
//   2  wide F (30..40): binary64 values, terms truncated with v_trunc_f64 and summed in
//      binary64 (exact below 2^53);
//   3  mode 0 with E8M0 block scales (Algorithm "ST-FDPA") whose blocks hold whole groups: all products of a group
//      then share one scale exponent s, the aligned terms are those of the unscaled group, and s only moves the
//      group's maximum exponent (and with it everything the accumulator meets).
//   4  mode 1 for TF32 operands (binary32 words whose low 13 mantissa bits do not count): the same exponent range as
//      BF16 with 11-bit significands, so products still fit binary32 exactly; elements arrive four to a 128-bit load.
// Accumulation modes (template parameter CMODE): MMAEMU_C_IN_GROUP, MMAEMU_C_AFTER_EXACT, MMAEMU_C_AFTER_RD (paper
// Algorithm "TR-FDPA" and its variations), and the two split forms of the latter (Algorithm "GTR-FDPA"):
// CM_RD_EVEN_ODD, where the packed exponent maxima of pass 1 already are the even and the odd maximum (even k in
// the low halves, odd k in the high halves) and pass 2 alternates between two scales and two sums, and CM_RD_HALVES,
// where each half of a group runs through passes 1 and 2 as a group of its own before the halves are merged, and
// CM_RD_QUARTERS, where pass 1 runs over the four quarters first (their maxima and the largest of them), then pass 2
// quarter by quarter, each sum rounded down into the merged sum as soon as it is complete.
// NaN and infinities are tagged with an exponent sentinel; a group that meets one is
// recomputed by the integer routine of the general kernel from the raw operands in
// global memory.
#pragma once
#include "fdpa_int.hpp"

#include <type_traits>

namespace mmaemu {

constexpr int CM_RD_EVEN_ODD = 3, CM_RD_HALVES = 4, CM_RD_QUARTERS = 5;   // template-only values of CMODE (ModelArgs::c_mode stays C_AFTER_RD)

constexpr uint32_t SENTINEL = 0x4000u;      // exponent tag of an element the fast path cannot take
constexpr uint32_t SENTINEL_MASK = 0xC000C000u;

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_add_u16(uint32_t a, uint32_t b)
{
    u16x2 x, y;
    __builtin_memcpy(&x, &a, 4); __builtin_memcpy(&y, &b, 4);
    x = x + y;
    uint32_t r; __builtin_memcpy(&r, &x, 4);
    return r;
}
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b)
{
    u16x2 x, y;
    __builtin_memcpy(&x, &a, 4); __builtin_memcpy(&y, &b, 4);
    x = __builtin_elementwise_max(x, y);
    uint32_t r; __builtin_memcpy(&r, &x, 4);
    return r;
}

// ---- decode while staging --------------------------------------------------------------

// One element -> exact binary32 value (every supported operand value is a binary32 number)
// and e' = max(E, 1) - 1, or the sentinel tag for NaN / infinities (whose staged value is a NaN, or the infinity itself:
// the sums of a group that meets one are not used, and special_products reads the group's classes off these values).  `wild` is raised by a
// finite non-zero value outside [2^-31, 2^32), whose products may leave binary32 (BF16 only).
// `zbias` (0, or ZBIAS when terms with a zero significand must not take part in exponent maxima):
// a non-zero element's e' is raised by zbias and a zero element's e' is 0, so that a product with
// a zero factor has an exponent sum below 2 * ZBIAS and every other product one at or above it.
constexpr uint32_t ZBIAS = 0x100u;

template <int T>
__device__ __forceinline__ void decode_elem(uint32_t bits, uint32_t ftz_in, uint32_t zbias, float &val, uint32_t &ex, bool &wild)
{
    using F = Fmt<T>;
    constexpr uint32_t EMASK = (1u << F::EB) - 1u, MMASK = (1u << F::MB) - 1u;
    const uint32_t E = (bits >> F::MB) & EMASK;
    const bool is_zero = (bits & ((1u << (F::EB + F::MB)) - 1u)) == 0 || (ftz_in && E == 0);
    ex = (E ? E : 1u) - 1u + zbias;
    if (zbias && is_zero) ex = 0;
    if (T == MMAEMU_BF16) {
        // the value is the pattern moved to the top half of a binary32 word
        const bool flushed = ftz_in && E == 0;                  // FlushSubnormal: -> +0.0
        val = __uint_as_float(flushed ? 0u : bits << 16);
        if (E == EMASK) ex = SENTINEL;                          // (the value stays the NaN or infinity it is)
        else wild |= !flushed && (bits & 0x7FFFu) != 0 && (E - 96u) > 62u;
    } else if (T == MMAEMU_TF32) {
        // (bits: the word without its 13 surplus bits) the value is the pattern moved back into place
        const bool flushed = ftz_in && E == 0;
        val = __uint_as_float(flushed ? 0u : bits << 13);
        if (E == EMASK) ex = SENTINEL;
        else wild |= !flushed && (bits & 0x3FFFFu) != 0 && (E - 96u) > 62u;
    } else if (T == MMAEMU_FP16) {
        _Float16 h;
        const uint16_t hb = (uint16_t)bits;
        __builtin_memcpy(&h, &hb, 2);
        val = (float)h;                                          // exact, subnormals included; NaN and infinity as themselves
        if (ftz_in && E == 0) val = 0.0f;
        if (E == EMASK) ex = SENTINEL;
    } else if (T == MMAEMU_FP8_E4M3 || T == MMAEMU_FP8_E5M2) {
        // the hardware's own conversion (gfx950 takes the OCP encodings): exact, subnormals included
        const uint32_t M = bits & MMASK, sign = (bits >> 7) & 1u;
        val = T == MMAEMU_FP8_E4M3 ? __builtin_amdgcn_cvt_f32_fp8((int)bits, 0) : __builtin_amdgcn_cvt_f32_bf8((int)bits, 0);
        if (ftz_in && E == 0) val = 0.0f;
        if (F::IEEE ? (E == EMASK) : (E == EMASK && M == MMASK)) {
            ex = SENTINEL;
            val = __uint_as_float((F::IEEE && M == 0) ? (0x7F800000u | (sign << 31)) : 0x7FC00000u);
        }
    } else {
        uint32_t M = bits & MMASK, sign = (bits >> (F::EB + F::MB)) & 1u;
        const bool special = F::IEEE ? (E == EMASK) : (!F::NOSPEC && E == EMASK && M == MMASK);
        if (ftz_in && E == 0) { M = 0; sign = 0; }
        const uint32_t sig = E ? (M | (1u << F::MB)) : M;
        const float mag = ldexpf((float)sig, (int)(E ? E : 1u) - F::BIAS - F::MB);   // exact
        val = __uint_as_float(__float_as_uint(mag) | (sign << 31));
        if (special) {
            ex = SENTINEL;
            val = __uint_as_float((F::IEEE && M == 0) ? (0x7F800000u | (sign << 31)) : 0x7FC00000u);
        }
    }
}

// four consecutive k elements of one row: raw little-endian bytes in `raw`
template <int T>
__device__ __forceinline__ void decode4(uint2 raw, uint32_t ftz_in, uint32_t zbias, float (&f)[4], uint2 &e, bool &wild)
{
    uint32_t b[4];
    if (Fmt<T>::W == 8) {
        b[0] = raw.x & 0xFFu; b[1] = (raw.x >> 8) & 0xFFu; b[2] = (raw.x >> 16) & 0xFFu; b[3] = raw.x >> 24;
    } else {
        b[0] = raw.x & 0xFFFFu; b[1] = raw.x >> 16; b[2] = raw.y & 0xFFFFu; b[3] = raw.y >> 16;
    }
    uint32_t x[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) decode_elem<T>(b[q], ftz_in, zbias, f[q], x[q], wild);
    e = make_uint2(x[0] | (x[1] << 16), x[2] | (x[3] << 16));
}

// the same for elements held in 32-bit words (TF32)
template <int T>
__device__ __forceinline__ void decode4(uint4 raw, uint32_t ftz_in, uint32_t zbias, float (&f)[4], uint2 &e, bool &wild)
{
    const uint32_t b[4] = {raw.x >> 13, raw.y >> 13, raw.z >> 13, raw.w >> 13};
    uint32_t x[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) decode_elem<T>(b[q], ftz_in, zbias, f[q], x[q], wild);
    e = make_uint2(x[0] | (x[1] << 16), x[2] | (x[3] << 16));
}

// smallest normal number of an operand format, 2^(1 - bias)
__device__ __forceinline__ float min_normal_of(uint32_t t)
{
    int bias;
    switch (t) {
    case MMAEMU_FP8_E4M3: bias = 7; break;
    case MMAEMU_FP8_E5M2: case MMAEMU_FP16: bias = 15; break;
    case MMAEMU_FP6_E2M3: case MMAEMU_FP4_E2M1: bias = 1; break;
    case MMAEMU_FP6_E3M2: bias = 3; break;
    default: bias = 127; break;                                   // BF16, TF32
    }
    return __uint_as_float((uint32_t)(128 - bias) << 23);
}

// item -> (tile, block index inside the tile) without a 64-bit division where it can be avoided
__device__ __forceinline__ void split_item(uint64_t it, uint32_t per_tile, uint64_t &tile, uint32_t &rem)
{
    if (per_tile == 1) { tile = it; rem = 0; }
    else if ((it >> 32) == 0) { const uint32_t i32 = (uint32_t)it; tile = i32 / per_tile; rem = i32 - (uint32_t)tile * per_tile; }
    else { tile = it / per_tile; rem = (uint32_t)(it - tile * per_tile); }
}

// Per-thread staging plan: each thread moves NQ quads (4 consecutive k elements of one
// row) per matrix and chunk; the quad's global row and its LDS offsets do not change
// along k, so they are worked out once.
template <int NQ>
struct StagePlan {
    const uint8_t *src[NQ];      // row start in global memory (bytes), + (k0 + 4*kq) * esize per chunk
    uint32_t voff[NQ], eoff[NQ]; // LDS dword offsets of the quad's values / packed exponents
    uint32_t kq4[NQ];            // 4 * kq
};

template <int ROWS, int KC, int SLOTS, int VS, int ES, bool IS_A, int NQ>
__device__ __forceinline__ void make_plan(StagePlan<NQ> &pl, const void *base, uint32_t esize, uint64_t item0, uint64_t nitems,
                                          uint32_t bm_count, uint32_t bn_count, uint32_t rows_per_tile, uint32_t k)
{
    constexpr int QUADS = SLOTS * ROWS * (KC / 4);
    static_assert(QUADS % 256 == 0 || QUADS < 256, "quads per thread");
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
        int q = threadIdx.x + 256 * i;
        q = q < QUADS ? q : QUADS - 1;                        // (threads beyond the panel repeat its last quad)
        const int kq = q % (KC / 4), row = (q / (KC / 4)) % ROWS, slot = q / ((KC / 4) * ROWS);
        uint64_t it = item0 + slot;
        it = it < nitems ? it : nitems - 1;                   // surplus slots re-read the last item
        uint64_t tile; uint32_t rem;
        split_item(it, bm_count * bn_count, tile, rem);
        const uint32_t blk = IS_A ? rem / bn_count : rem % bn_count;
        uint32_t rit = blk * ROWS + row;                      // row inside the tile
        rit = rit < rows_per_tile ? rit : rows_per_tile - 1;  // (a ragged edge block repeats the tile's last row)
        const uint64_t grow = tile * rows_per_tile + rit;
        pl.src[i] = reinterpret_cast<const uint8_t *>(base) + grow * k * esize;
        pl.voff[i] = (slot * ROWS + row) * VS + 4 * kq;
        pl.eoff[i] = (slot * ROWS + row) * ES + 2 * kq;
        pl.kq4[i] = 4 * kq;
    }
}

// global -> registers
template <int NQ>
__device__ __forceinline__ void load_panel(uint32_t esize, const StagePlan<NQ> &pl, uint32_t k0, uint2 (&raw)[NQ])
{
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
        const uint8_t *src = pl.src[i] + (uint64_t)(k0 + pl.kq4[i]) * esize;
        if (esize == 1) { raw[i].x = *reinterpret_cast<const uint32_t *>(src); raw[i].y = 0; }
        else raw[i] = *reinterpret_cast<const uint2 *>(src);
    }
}

template <int NQ>
__device__ __forceinline__ void load_panel(uint32_t esize, const StagePlan<NQ> &pl, uint32_t k0, uint4 (&raw)[NQ])
{
#pragma unroll
    for (int i = 0; i < NQ; ++i)
        raw[i] = *reinterpret_cast<const uint4 *>(pl.src[i] + (uint64_t)(k0 + pl.kq4[i]) * esize);    // (esize = 4)
}

// raw registers -> decoded registers; returns whether any element needs binary64 products
template <int T, int NQ, typename RAW>
__device__ __forceinline__ bool decode_panel(const RAW (&raw)[NQ], uint32_t ftz_in, uint32_t zbias, float (&f)[NQ][4], uint2 (&e)[NQ])
{
    bool wild = false;
#pragma unroll
    for (int i = 0; i < NQ; ++i) decode4<T>(raw[i], ftz_in, zbias, f[i], e[i], wild);
    return wild;
}

template <int NQ>
__device__ __forceinline__ bool decode_any(uint32_t t, const uint2 (&raw)[NQ], uint32_t ftz_in, uint32_t zbias, float (&f)[NQ][4],
                                           uint2 (&e)[NQ])
{
    switch (t) {   // uniform
    case MMAEMU_FP8_E4M3: return decode_panel<MMAEMU_FP8_E4M3, NQ>(raw, ftz_in, zbias, f, e);
    case MMAEMU_FP8_E5M2: return decode_panel<MMAEMU_FP8_E5M2, NQ>(raw, ftz_in, zbias, f, e);
    case MMAEMU_FP16: return decode_panel<MMAEMU_FP16, NQ>(raw, ftz_in, zbias, f, e);
    case MMAEMU_FP6_E2M3: return decode_panel<MMAEMU_FP6_E2M3, NQ>(raw, ftz_in, zbias, f, e);
    case MMAEMU_FP6_E3M2: return decode_panel<MMAEMU_FP6_E3M2, NQ>(raw, ftz_in, zbias, f, e);
    case MMAEMU_FP4_E2M1: return decode_panel<MMAEMU_FP4_E2M1, NQ>(raw, ftz_in, zbias, f, e);
    default: return decode_panel<MMAEMU_BF16, NQ>(raw, ftz_in, zbias, f, e);
    }
}
template <int NQ>
__device__ __forceinline__ bool decode_any(uint32_t, const uint4 (&raw)[NQ], uint32_t ftz_in, uint32_t zbias, float (&f)[NQ][4],
                                           uint2 (&e)[NQ])
{
    return decode_panel<MMAEMU_TF32, NQ>(raw, ftz_in, zbias, f, e);
}

// decoded registers -> LDS.  `as_double`: values are written as binary64 (row stride VSD
// doubles) instead of binary32 (row stride VS floats); WHAT bit 0: exponents, bit 1: values.
template <int NQ, int VS, int VSD>
__device__ __forceinline__ void store_panel(const StagePlan<NQ> &pl, const float (&f)[NQ][4], const uint2 (&e)[NQ], void *lv,
                                            uint32_t *le, bool as_double, int what)
{
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
        if (what & 1) *reinterpret_cast<uint2 *>(le + pl.eoff[i]) = e[i];
        if (what & 2) {
            if (as_double) {
                // voff = row * VS + 4*kq  ->  row * VSD + 4*kq
                const uint32_t row = pl.voff[i] / VS, kq4 = pl.voff[i] - row * VS;
                double *dst = reinterpret_cast<double *>(lv) + row * VSD + kq4;
                *reinterpret_cast<double2 *>(dst) = make_double2((double)f[i][0], (double)f[i][1]);
                *reinterpret_cast<double2 *>(dst + 2) = make_double2((double)f[i][2], (double)f[i][3]);
            } else {
                *reinterpret_cast<float4 *>(reinterpret_cast<float *>(lv) + pl.voff[i]) = make_float4(f[i][0], f[i][1], f[i][2], f[i][3]);
            }
        }
    }
}

// ---- per-group arithmetic ---------------------------------------------------------------

struct TiledArgs {
    ModelArgs p;
    uint32_t ta, tb;
    int32_t ebase;       // Exp = e' + ebase for a product: 2 - bias_a - bias_b
    // value mode 3: E8M0 codes SA[batch][m][k / block], SB[batch][n][k / block]; block is a multiple of the group length
    const uint8_t *sa, *sb;
    uint32_t block;
};

constexpr int STATS_WORDS = 39;        // sizeof(mmaemu_stats) / 8 in 64-bit words

// Binary32 rounding mode of the wavefront (bits 1:0 of the MODE register): to nearest even, or toward zero.
__device__ __forceinline__ void set_f32_round_toward_zero(bool on)
{
#if defined(__HIP_DEVICE_COMPILE__)
    if (on) __builtin_amdgcn_s_setreg((1 | (0 << 6) | (1 << 11)), 3);      // hwreg(MODE, offset 0, 2 bits) = 3
    else __builtin_amdgcn_s_setreg((1 | (0 << 6) | (1 << 11)), 0);
#endif
}

// Reduction over the 64 lanes of a wavefront with row shifts and row broadcasts of the data-parallel primitives (no LDS
// traffic); the result is valid in lane 63.
template <bool IS_MAX>
__device__ __forceinline__ uint32_t wave_reduce_to_lane63(uint32_t v)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int ident = IS_MAX ? 0 : -1;             // 0 for the maximum, 0xFFFFFFFF for the minimum (unsigned)
    auto op = [](uint32_t a, uint32_t b) -> uint32_t { return IS_MAX ? (a > b ? a : b) : (a < b ? a : b); };
    // lanes whose source lies outside their row keep the identity (bound_ctrl off, `old` = identity)
    v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(ident, (int)v, 0x111, 0xF, 0xF, false));    // row_shr:1
    v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(ident, (int)v, 0x112, 0xF, 0xF, false));    // row_shr:2
    v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(ident, (int)v, 0x114, 0xF, 0xF, false));    // row_shr:4
    v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(ident, (int)v, 0x118, 0xF, 0xF, false));    // row_shr:8: lane 15 of each row holds the row
    v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(ident, (int)v, 0x142, 0xA, 0xF, false));    // row_bcast:15 into rows 1 and 3
    v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(ident, (int)v, 0x143, 0xC, 0xF, false));    // row_bcast:31 into rows 2 and 3
#endif
    return v;
}

// start of the running kernel's argument segment, as a pointer the optimiser cannot trace back to the arguments
__device__ __forceinline__ const void *opaque_kernarg_ptr()
{
#if defined(__HIP_DEVICE_COMPILE__)
    const void *kp = __builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(kp));
    return kp;
#else
    return nullptr;
#endif
}

// ---- special values of a thread's register block, from the raw operands ---------------------
// A group that holds a NaN or an infinity (operand or accumulator) has a NaN or an infinity for its result (Sec. 4.2),
// and which one follows from the classes and signs of the operands alone.  For the tagged outputs of one thread's
// R x C block this routine classifies each row of A and of B once per group into bit masks over k (NaN, infinity,
// zero, sign) and applies the rules to the masks: no value is decoded, and a row shared by several outputs is read
// once.  Outputs it cannot settle (no special operand after all: the group was tagged for another reason; or an
// infinity where the model's overflow rule or a NaN scale factor may still turn it into NaN) are left to the integer
// routine.  Kept out of line so that its registers do not count against the hot loops.  (The model's parameters come
// in as arguments: the kernel-argument segment pointer is null inside a called function.)
template <int N> struct BlockVals { uint32_t v[N]; uint32_t settled; };      // settled: bit r * C + c

struct RowMasks { uint64_t nan, inf, zero, sign; };

__device__ __forceinline__ RowMasks classify_row(const DynFmt &f, const void *row, uint32_t len, uint32_t ftz_in)
{
    const uint32_t MAG = (1u << (f.eb() + f.mb())) - 1u, EXPM = ((1u << f.eb()) - 1u) << f.mb();
    RowMasks r = {0ull, 0ull, 0ull, 0ull};
    for (uint32_t k = 0; k < len; ++k) {
        const uint32_t bits = f.load(row, k), mag = bits & MAG;
        const uint64_t bit = 1ull << k;
        if (f.ieee()) {
            if (mag > EXPM) r.nan |= bit;
            if (mag == EXPM) r.inf |= bit;
        } else if (!f.nospec()) {
            if (mag == MAG) r.nan |= bit;                                     // the E4M3 rule: one NaN code, no infinity
        }
        if (ftz_in ? (mag & EXPM) == 0 : mag == 0) r.zero |= bit;            // (FlushSubnormal: a subnormal counts as zero)
        if ((bits >> (f.eb() + f.mb())) & 1u) r.sign |= bit;
    }
    return r;
}

// inf_final: an infinity stands (nothing else can still make it NaN: no product-overflow rule, which adds infinities
// of its own, and no scale factors, of which a NaN one overrides)
template <int R, int C, int TI, int TJ>
__device__ __noinline__ BlockVals<R * C> special_block(const void *A, const void *B, uint64_t arow0, uint64_t brow0, uint32_t k,
                                                       uint32_t kg, BlockVals<R * C> cin, uint32_t tagged, uint32_t ta, uint32_t tb,
                                                       uint32_t L, uint32_t ftz_in, uint32_t nan_bits, bool inf_final)
{
    const DynFmt fa = dyn_fmt(ta), fb = dyn_fmt(tb);
    const uint32_t esa = (uint32_t)fa.width_ / 8u, esb = (uint32_t)fb.width_ / 8u;
    uint32_t any_nan = 0, pinf = 0, ninf = 0;                                 // one bit per output
    uint32_t rows = 0, cols = 0;                                              // rows of A / of B that a tagged output needs
#pragma unroll
    for (int i = 0; i < R * C; ++i)
        if ((tagged >> i) & 1u) { rows |= 1u << (i / C); cols |= 1u << (i % C); }
    for (uint32_t k0 = 0; k0 < L; k0 += 64u) {
        const uint32_t len = L - k0 < 64u ? L - k0 : 64u;
        RowMasks mb[C];
#pragma unroll
        for (int c = 0; c < C; ++c) {
            mb[c] = RowMasks{0ull, 0ull, 0ull, 0ull};
            if ((cols >> c) & 1u)
                mb[c] = classify_row(fb, reinterpret_cast<const uint8_t *>(B) + ((brow0 + (uint64_t)(TJ * c)) * k + kg + k0) * esb, len, ftz_in);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (!((rows >> r) & 1u)) continue;
            const RowMasks ma = classify_row(fa, reinterpret_cast<const uint8_t *>(A) + ((arow0 + (uint64_t)(TI * r)) * k + kg + k0) * esa, len, ftz_in);
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const uint64_t nanp = ma.nan | mb[c].nan | (ma.inf & mb[c].zero) | (mb[c].inf & ma.zero);
                const uint64_t infp = (ma.inf | mb[c].inf) & ~nanp, neg = ma.sign ^ mb[c].sign;
                const uint32_t bit = 1u << (r * C + c);
                if (nanp) any_nan |= bit;
                if (infp & ~neg) pinf |= bit;
                if (infp & neg) ninf |= bit;
            }
        }
    }
    BlockVals<R * C> out;
    out.settled = 0;
#pragma unroll
    for (int i = 0; i < R * C; ++i) {
        out.v[i] = 0;
        if (!((tagged >> i) & 1u)) continue;
        const uint32_t c = cin.v[i], bit = 1u << i;
        bool n = (any_nan & bit) != 0, p = (pinf & bit) != 0, m = (ninf & bit) != 0;
        if ((c & 0x7FFFFFFFu) > 0x7F800000u) n = true;
        else if ((c & 0x7FFFFFFFu) == 0x7F800000u) { if (c >> 31) m = true; else p = true; }
        if (n || (p && m)) { out.v[i] = nan_bits; out.settled |= bit; }
        else if ((p || m) && inf_final) { out.v[i] = p ? 0x7F800000u : 0xFF800000u; out.settled |= bit; }
    }
    return out;
}

// The special values of Sec. 4.2 for the tagged outputs of a thread's R x C block, from the group's staged values
// (binary32, or binary64 when DBL; a[r * SA + kk], b[c * SB + kk], kk < LEN; NaN and infinite elements are staged as
// themselves, flushed ones as zeros).  IEEE multiplication of the staged values classifies every product:
// NaN for a NaN operand and for infinity times zero, an infinity of the product's sign for an infinite operand; with
// `overflow_rule` (TR-FDPA: a finite product of magnitude 2^128 or more counts as an infinity) the threshold moves from
// infinity down to 2^128 (binary64 products are exact; a group held in binary32 has no such product).  Per output two
// running maxima over the products' bit patterns are kept, one signed and one unsigned: patterns of positive numbers
// order like the numbers with +infinity and the positive NaNs on top (signed maximum), patterns of negative numbers
// order by magnitude above every positive pattern (unsigned maximum).  For binary64 the high words do: a NaN the
// multiplier makes is the quiet one, and an infinity has a zero low word.  The caller lets the accumulator join and
// applies the rules.  Out of line, like special_block.
template <int R, int C, int SA, int SB, int LEN, bool DBL>
__device__ __forceinline__ uint2 special_products_of(const void *a_, const void *b_, bool overflow_rule)
{
    typedef typename std::conditional<DBL, double, float>::type V;
    const V *a = static_cast<const V *>(a_), *b = static_cast<const V *>(b_);
    constexpr uint32_t INF_PAT = DBL ? 0x7FF00000u : 0x7F800000u;
    const uint32_t thr = (DBL && overflow_rule) ? 0x47F00000u : INF_PAT;       // high word of 2^128
    int32_t pmax[R][C];
    uint32_t nmax[R][C];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int c = 0; c < C; ++c) { pmax[r][c] = (int32_t)0x80000000u; nmax[r][c] = 0u; }
#pragma unroll 1
    for (int kk = 0; kk < LEN; ++kk) {
        V av[R], bv[C];
#pragma unroll
        for (int r = 0; r < R; ++r) av[r] = a[r * SA + kk];
#pragma unroll
        for (int c = 0; c < C; ++c) bv[c] = b[c * SB + kk];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const V pr = av[r] * bv[c];
                uint32_t w;
                if constexpr (DBL) w = (uint32_t)__double2hiint(pr);
                else w = __float_as_uint(pr);
                pmax[r][c] = (int32_t)w > pmax[r][c] ? (int32_t)w : pmax[r][c];
                nmax[r][c] = w > nmax[r][c] ? w : nmax[r][c];
            }
    }
    uint32_t nan = 0, pos = 0, neg = 0;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const uint32_t bit = 1u << (r * C + c);
            if (pmax[r][c] > (int32_t)INF_PAT || nmax[r][c] > (0x80000000u | INF_PAT)) nan |= bit;
            if (pmax[r][c] >= (int32_t)thr) pos |= bit;
            if (nmax[r][c] >= (0x80000000u | thr)) neg |= bit;
        }
    return make_uint2(nan, pos | (neg << 16));
}

// SA_F, SB_F / SA_D, SB_D: row strides of a thread's rows of A and B in the binary32 / binary64 staging (elements);
// how: bit 0, the values are binary64; bit 1, the product-overflow rule applies.
// Returns x: outputs (bit r * C + c) with a NaN product; y: with a product counted as +infinity (low half) / -infinity
// (high half).
template <int R, int C, int SA_F, int SB_F, int SA_D, int SB_D, int LEN>
__device__ __noinline__ uint2 special_products(const void *a, const void *b, uint32_t how)
{
    static_assert(R * C <= 16, "one bit per output in each half of a word");
    if (how & 1u) return special_products_of<R, C, SA_D, SB_D, LEN, true>(a, b, (how & 2u) != 0);
    return special_products_of<R, C, SA_F, SB_F, LEN, false>(a, b, (how & 2u) != 0);
}

// ---- the kernel -------------------------------------------------------------------------
// TM x TN : block of D per slot;  R x C: register block per thread;
// KC      : k elements staged at a time;
// LT      : group length if it divides KC, 0 if a group spans whole chunks (L % KC == 0);
// NF      : terms summed in 32 bits between folds into binary64 (0: once per group/chunk);
// VM      : value mode (see the head of this file).
// Per-workgroup statistics of the multi-model kernels, in LDS: filled by every pass of a workgroup over its tiles,
// written out once at the end of the kernel.
constexpr int HIST_COPIES = 2;
struct MultiLds {
    uint32_t hist[MULTI_MAX][34][HIST_COPIES];     // pairs that differ, by bucket (bucket 0: patterns differ at distance 0)
    uint32_t naneq[MULTI_MAX], maxd[MULTI_MAX];
    unsigned long long first[MULTI_MAX];
};

template <int TM, int TN, int R, int C, int KC, int LT, int CMODE, int NF, int VM_>
__device__ __forceinline__ void
tiled_body(const TiledArgs &ta_, const void *__restrict__ A, const void *__restrict__ B, const uint32_t *Cm,
           uint32_t *D, uint32_t m, uint32_t n, uint32_t k, uint64_t nitems, uint32_t bm_count,
           uint32_t bn_count, uint32_t xcd_remap, uint32_t wg_index)
{
    constexpr bool SC = VM_ == 3;                     // block scales
    constexpr bool WIDE = VM_ == 4;                   // elements in 32-bit words (TF32)
    constexpr int VM = SC ? 0 : (WIDE ? 1 : VM_);     // how values are held
    constexpr int TI = TM / R, TJ = TN / C, TPS = TI * TJ, SLOTS = 256 / TPS;
    static_assert(TPS * SLOTS == 256, "thread layout");
    static_assert(!SC || LT != 0, "scaled groups have a fixed length");
    constexpr int VS = KC + 4;                       // LDS row stride of binary32 values (floats), padded
    constexpr int VSD = KC + 2;                      // LDS row stride of binary64 values (doubles)
    constexpr int ES = KC / 2 + (KC == 16 ? 2 : 4);  // LDS row stride of packed exponents (dwords)
    constexpr bool IS_RD = CMODE == MMAEMU_C_AFTER_RD || CMODE == CM_RD_EVEN_ODD || CMODE == CM_RD_HALVES || CMODE == CM_RD_QUARTERS;
    static_assert(!(CMODE == CM_RD_EVEN_ODD || CMODE == CM_RD_HALVES || CMODE == CM_RD_QUARTERS) || (LT >= 4 && VM == 0 && NF == 0), "split groups: fixed length, binary32 values, one fold");
    static_assert(CMODE != CM_RD_HALVES || LT >= 8, "halves of at least four terms");
    static_assert(CMODE != CM_RD_QUARTERS || LT >= 16, "quarters of at least four terms");
    constexpr int GL = CMODE == CM_RD_HALVES ? LT / 2 : CMODE == CM_RD_QUARTERS ? LT / 4 : (LT ? LT : KC);   // terms per inner step
    constexpr int FOLD = NF ? NF : GL;
    constexpr bool USE_SD = (NF != 0) || (LT == 0) || (VM == 2);   // binary64 accumulator needed
    constexpr int VBYTES_A = SLOTS * TM * (VM == 0 ? VS * 4 : VSD * 8);
    constexpr int VBYTES_B = SLOTS * TN * (VM == 0 ? VS * 4 : VSD * 8);
    constexpr int EBYTES_A = SLOTS * TM * ES * 4, EBYTES_B = SLOTS * TN * ES * 4;
    constexpr int LDS_BYTES = VBYTES_A + VBYTES_B + EBYTES_A + EBYTES_B;
    __shared__ __attribute__((aligned(16))) unsigned char smem[LDS_BYTES];
    unsigned char *Av_raw = smem, *Bv_raw = smem + VBYTES_A;
    uint32_t *Ae = reinterpret_cast<uint32_t *>(smem + VBYTES_A + VBYTES_B);
    uint32_t *Be = reinterpret_cast<uint32_t *>(smem + VBYTES_A + VBYTES_B + EBYTES_A);

    const ModelArgs &p = ta_.p;
    int F = p.F;
    uint32_t fl = p.flags;                            // the model's switches, one bit each (one scalar register)
    uint32_t out_mask = p.out_mask, nan_bits = p.nan_bits;
    // the kernel's arguments once more, through a pointer the optimiser cannot see through (see slow_group)
    auto fetch_args = [&]() -> TiledArgs { return *reinterpret_cast<const TiledArgs *>(opaque_kernarg_ptr()); };
    // The group epilogues test the switches on a copy that is made opaque each time: otherwise every test is
    // hoisted out of the loops as a wave-wide mask (two scalar registers apiece, live across the hot loops).
    const int ec_floor = (fl & FL_ACC16) ? -14 : -126;          // smallest Exp of the accumulator's type
    uint32_t fe = fl;
    auto refresh_switches = [&]() {
#if defined(__HIP_DEVICE_COMPILE__)
        fe = fl;
        asm volatile("" : "+s"(fe));
#endif
    };
    const uint32_t tid = threadIdx.x, slot = tid / TPS, ti = (tid % TPS) / TJ, tj = tid % TJ;

    // workgroup -> items.  Consecutive workgroup ids go to different XCDs (8 of them, each
    // with its own L2); the remap hands every XCD a contiguous range of blocks so that
    // neighbours sharing A/B panels share an L2.
    // (with several models a workgroup makes several passes, each over the items of one logical workgroup: what depends
    // on the pass is set by the two routines below, the staging plans apart from the outputs' places, so that the
    // next pass's operands can be fetched while the current pass's models run)
    uint64_t item0;
    constexpr int NQA = (SLOTS * TM * (KC / 4) + 255) / 256, NQB = (SLOTS * TN * (KC / 4) + 255) / 256;
    const uint32_t esa = WIDE ? 4u : ((ta_.ta <= MMAEMU_FP8_E5M2 || ta_.ta >= MMAEMU_FP6_E2M3) ? 1u : 2u);      // bytes per element
    const uint32_t esb = WIDE ? 4u : ((ta_.tb <= MMAEMU_FP8_E5M2 || ta_.tb >= MMAEMU_FP6_E2M3) ? 1u : 2u);
    StagePlan<NQA> plan_a;
    StagePlan<NQB> plan_b;
    auto logical_wg = [&](uint32_t w) -> uint32_t { return xcd_remap ? (w & 7u) * (gridDim.x >> 3) + (w >> 3) : w; };
    auto set_plans = [&](uint32_t w) {
        const uint64_t it0 = (uint64_t)logical_wg(w) * SLOTS;
        make_plan<TM, KC, SLOTS, VS, ES, true, NQA>(plan_a, A, esa, it0, nitems, bm_count, bn_count, m, k);
        make_plan<TN, KC, SLOTS, VS, ES, false, NQB>(plan_b, B, esb, it0, nitems, bm_count, bn_count, n, k);
    };
    bool live;
    uint64_t my_tile, d_off;                          // d_off: + TI*r*n + TJ*c
    uint32_t i_base, j_base;
    auto set_outputs = [&](uint32_t w) {
        item0 = (uint64_t)logical_wg(w) * SLOTS;
        live = item0 + slot < nitems;
        uint64_t my_it = item0 + slot;
        my_it = my_it < nitems ? my_it : nitems - 1;
        const uint32_t per_tile = bm_count * bn_count;
        uint32_t my_rem;
        split_item(my_it, per_tile, my_tile, my_rem);
        i_base = (my_rem / bn_count) * TM + ti;
        j_base = (my_rem % bn_count) * TN + tj;
        d_off = (my_tile * m + i_base) * (uint64_t)n + j_base;
    };
    set_plans(wg_index);
    set_outputs(wg_index);

    // C in (each thread its own elements; measured faster here than moving the block through LDS)
    uint32_t d[R][C];
    // Ragged m or n (32 x 32 blocks of a larger problem, groups inside a staged chunk): edge blocks stage the tile's last
    // row again for the rows beyond it, their threads load the accumulator of the clamped place and store nothing there.
    constexpr bool EDGES = TM == 32 && TN == 32 && !SC && LT != 0;
    const bool ragged = EDGES && ((m % TM) | (n % TN)) != 0;      // uniform
    auto load_acc = [&]() {
        auto take = [&](int r, int c, uint64_t o) {
            d[r][c] = (fl & FL_ACC16) ? half_bits_to_float_bits(reinterpret_cast<const uint16_t *>(Cm)[o]) : Cm[o];
        };
        if constexpr (EDGES) {
            if (ragged) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        const uint32_t i = i_base + TI * r, j = j_base + TJ * c;
                        take(r, c, (my_tile * m + (i < m ? i : m - 1)) * (uint64_t)n + (j < n ? j : n - 1));
                    }
                return;
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c) take(r, c, d_off + (uint64_t)(TI * r) * n + TJ * c);
    };
    load_acc();

    const float *av = reinterpret_cast<const float *>(Av_raw) + (slot * TM + ti) * VS;
    const float *bv = reinterpret_cast<const float *>(Bv_raw) + (slot * TN + tj) * VS;
    const double *avd = reinterpret_cast<const double *>(Av_raw) + (slot * TM + ti) * VSD;
    const double *bvd = reinterpret_cast<const double *>(Bv_raw) + (slot * TN + tj) * VSD;
    const uint32_t *ae = Ae + (slot * TM + ti) * ES;
    const uint32_t *be = Be + (slot * TN + tj) * ES;

    uint32_t m2[R][C];                                          // packed running maxima of e'
    // block scales: the codes of this thread's rows and columns for the group at hand, and per element
    // s = Exp(alpha) + Exp(beta), which the group's maximum exponent carries and pass 2 must leave out again
    uint32_t sca[SC ? R : 1], scb[SC ? C : 1];
    int sadj[SC ? R : 1][SC ? C : 1];
    auto load_scales = [&](uint32_t kg) {
        if constexpr (SC) {
            const TiledArgs q = fetch_args();
            const uint32_t nblk = k / q.block, qb = kg / q.block;
#pragma unroll
            for (int r = 0; r < R; ++r) sca[r] = q.sa[(my_tile * m + i_base + TI * r) * (uint64_t)nblk + qb];
#pragma unroll
            for (int c = 0; c < C; ++c) scb[c] = q.sb[(my_tile * n + j_base + TJ * c) * (uint64_t)nblk + qb];
        }
    };
    int32_t S32[R][C];
    int32_t S32o[CMODE == CM_RD_EVEN_ODD ? R : 1][CMODE == CM_RD_EVEN_ODD ? C : 1];   // odd products (even / odd split)
    double Sd[R][C];
    bool chunk_is_double = (VM == 2);                           // how the staged chunk's values are held

    // pass 1: running maxima of e' = e'_a + e'_b, two products per packed instruction;
    // EW dwords (2*EW exponents) per LDS read and row
    constexpr int EW = (ES % 4 == 0 && (GL / 2) % 4 == 0) ? 4 : 2;
    constexpr int U1 = (GL / 2 / EW <= 2) ? 2 : 1;
    auto pass1 = [&](int g) {
#pragma unroll U1
        for (int q = 0; q < GL / 2; q += EW) {
            uint32_t ea[R][EW], eb[C][EW];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint32_t *src = ae + TI * r * ES + g * (GL / 2) + q;
                if (EW == 4) { const uint4 v = *reinterpret_cast<const uint4 *>(src); ea[r][0] = v.x; ea[r][1] = v.y; ea[r][2 % EW] = v.z; ea[r][3 % EW] = v.w; }
                else { const uint2 v = *reinterpret_cast<const uint2 *>(src); ea[r][0] = v.x; ea[r][1] = v.y; }
            }
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const uint32_t *src = be + TJ * c * ES + g * (GL / 2) + q;
                if (EW == 4) { const uint4 v = *reinterpret_cast<const uint4 *>(src); eb[c][0] = v.x; eb[c][1] = v.y; eb[c][2 % EW] = v.z; eb[c][3 % EW] = v.w; }
                else { const uint2 v = *reinterpret_cast<const uint2 *>(src); eb[c][0] = v.x; eb[c][1] = v.y; }
            }
#pragma unroll
            for (int w = 0; w < EW; ++w)
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c) m2[r][c] = pk_max_u16(m2[r][c], pk_add_u16(ea[r][w], eb[c][w]));
        }
    };

    auto fold = [&]() {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c) { Sd[r][c] += (double)S32[r][c]; S32[r][c] = 0; }
    };

    // pass 2, binary32 values: aligned, truncated terms summed in 32 bits; four k per LDS read and row
    constexpr int U2 = (GL / 4 <= 2) ? 2 : 1;
    auto pass2f = [&](int g, const int (&emax)[R][C]) {
        float scale[R][C];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c) {
                int se = F + 127 - emax[r][c];                         // biased exponent of 2^(F - e_max)
                if constexpr (SC) se += sadj[r][c];                    // (values are unscaled: e_max without s)
                se = se < 1 ? 1 : (se > 254 ? 254 : se);               // the clamps never change a truncated term
                scale[r][c] = __uint_as_float((uint32_t)se << 23);
            }
#pragma unroll U2
        for (int q = 0; q < GL; q += 4) {
            float a[R][4], b[C][4];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float4 v = *reinterpret_cast<const float4 *>(av + TI * r * VS + g * GL + q);
                a[r][0] = v.x; a[r][1] = v.y; a[r][2] = v.z; a[r][3] = v.w;
            }
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const float4 v = *reinterpret_cast<const float4 *>(bv + TJ * c * VS + g * GL + q);
                b[c][0] = v.x; b[c][1] = v.y; b[c][2] = v.z; b[c][3] = v.w;
            }
#pragma unroll
            for (int w = 0; w < 4; ++w) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c) S32[r][c] += (int32_t)((a[r][w] * b[c][w]) * scale[r][c]);
                if (USE_SD && (FOLD < 4) && (w + 1) % FOLD == 0) fold();
            }
            if (USE_SD && (FOLD >= 4) && (q + 4) % FOLD == 0) fold();
        }
    };

    // pass 2 with the even / odd split: even k aligned at the even maximum into S32, odd k at the odd one into S32o
    auto pass2eo = [&](int g, const int (&emax_e)[R][C], const int (&emax_o)[R][C]) {
        float scale_e[R][C], scale_o[R][C];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c) {
                int se = F + 127 - emax_e[r][c], so = F + 127 - emax_o[r][c];     // (unscaled maxima, also with block scales)
                se = se < 1 ? 1 : (se > 254 ? 254 : se);
                so = so < 1 ? 1 : (so > 254 ? 254 : so);
                scale_e[r][c] = __uint_as_float((uint32_t)se << 23);
                scale_o[r][c] = __uint_as_float((uint32_t)so << 23);
            }
#pragma unroll U2
        for (int q = 0; q < GL; q += 4) {
            float a[R][4], b[C][4];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float4 v = *reinterpret_cast<const float4 *>(av + TI * r * VS + g * GL + q);
                a[r][0] = v.x; a[r][1] = v.y; a[r][2] = v.z; a[r][3] = v.w;
            }
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const float4 v = *reinterpret_cast<const float4 *>(bv + TJ * c * VS + g * GL + q);
                b[c][0] = v.x; b[c][1] = v.y; b[c][2] = v.z; b[c][3] = v.w;
            }
#pragma unroll
            for (int w = 0; w < 4; ++w)
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        if (w & 1) S32o[CMODE == CM_RD_EVEN_ODD ? r : 0][CMODE == CM_RD_EVEN_ODD ? c : 0] += (int32_t)((a[r][w] * b[c][w]) * scale_o[r][c]);
                        else S32[r][c] += (int32_t)((a[r][w] * b[c][w]) * scale_e[r][c]);
                    }
        }
    };

    // pass 2, binary64 values (any finite operands; also wide F): two k per LDS read and row
    auto pass2d = [&](int g, const int (&emax)[R][C]) {
        double scale[R][C];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c)
                scale[r][c] = __hiloint2double((F - emax[r][c] + 1023) << 20, 0);      // 2^(F - e_max), always normal
#pragma unroll 1
        for (int q = 0; q < GL; q += 2) {
            double a[R][2], b[C][2];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const double2 v = *reinterpret_cast<const double2 *>(avd + TI * r * VSD + g * GL + q);
                a[r][0] = v.x; a[r][1] = v.y;
            }
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const double2 v = *reinterpret_cast<const double2 *>(bvd + TJ * c * VSD + g * GL + q);
                b[c][0] = v.x; b[c][1] = v.y;
            }
#pragma unroll
            for (int w = 0; w < 2; ++w) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        const double t = (a[r][w] * b[c][w]) * scale[r][c];            // exact product, exact scaling
                        if (VM == 2) Sd[r][c] += __builtin_trunc(t);
                        else S32[r][c] += (int32_t)t;
                    }
                if (VM != 2 && USE_SD && FOLD == 1) fold();
            }
            if (VM != 2 && USE_SD && FOLD >= 2 && (q + 2) % FOLD == 0) fold();
        }
    };

    // end of pass 1 for one element: e_max (products, and the accumulator when it is a term)
    auto exponents = [&](int r, int c, int &emax, uint32_t &tagged) {
        uint32_t e = m2[r][c];
        const uint32_t lo = e & 0xFFFFu, hi = e >> 16;
        int em = (int)(lo > hi ? lo : hi) + ta_.ebase;
        // the product-overflow rule may apply (a product is below 2^(em + 2)); with `wide_products` such products keep
        // their values, which binary64 holds
        bool to_slow = IS_RD && VM != 0 && em >= 127 && !(fl & FL_WIDE_PRODUCTS);
        if constexpr (SC) {
            const int s = (int)sca[r] + (int)scb[c] - 254;
            sadj[r][c] = s;
            em += s;
            // a NaN scale; or a product that may reach 2^128 where that counts as an infinity
            to_slow = sca[r] == 0xFFu || scb[c] == 0xFFu || (IS_RD && !(fl & FL_WIDE_PRODUCTS) && em >= 126);
        }
        if (to_slow && !(e & SENTINEL_MASK)) {
            // (without scales: a product may reach 2^128, which this mode counts as an infinity) leave the group
            // to the integer routine
            e |= 0x8000u;
            m2[r][c] = e;
        }
        tagged |= e;
        if (CMODE == MMAEMU_C_IN_GROUP) {
            const uint32_t Ec = (d[r][c] >> 23) & 0xFFu;               // (a flushed subnormal keeps Exp = -126)
            int ec = (int)(Ec ? Ec : 1u) - 127;
            ec = ec > ec_floor ? ec : ec_floor;                        // (a binary16 accumulator: Exp >= -14)
            em = ec > em ? ec : em;
        }
        emax = em;
    };

    auto slow_group = [&](int r, int c, uint32_t kg, uint32_t cin) -> uint32_t {
        const uint64_t arow = my_tile * m + i_base + TI * r;
        const uint64_t brow = my_tile * n + j_base + TJ * c;
        const uint8_t *a = reinterpret_cast<const uint8_t *>(A) + (arow * k + kg) * esa;
        const uint8_t *b = reinterpret_cast<const uint8_t *>(B) + (brow * k + kg) * esb;
        // The model parameters are fetched again here, from the kernel-argument segment (they are its first
        // bytes), through a pointer the optimiser cannot see through: otherwise every parameter this rare path
        // needs stays in scalar registers for the whole kernel and crowds out the hot loops' values.
        const TiledArgs q = fetch_args();
        ScaleRef sr = no_scales();
        if constexpr (SC) {
            const uint32_t nblk = k / q.block;
            sr = ScaleRef{q.sa + arow * nblk, q.sb + brow * nblk, q.block, kg};
        }
        if constexpr (!SC) return fdpa_group_raw_unscaled(q.p, q.ta, q.tb, a, b, q.p.L, cin);   // (fewer arguments: none on the stack)
        else return fdpa_group_raw(q.p, q.ta, q.tb, a, b, q.p.L, cin, sr);
    };

    // Algorithm "TR-FDPA", steps 3 and 4 ("GTR-FDPA", steps 4 and 5), and the variations, in binary64 (every
    // quantity is an integer of fewer than 53 bits times a power of two, hence exact, except where noted):
    // T counts units of 2^(em - FT); returns the exact value whose conversion is the group's result.
    auto rd_value = [&](double T, bool have_T, int em, int FT, uint32_t cb) -> double {
        const int Fmax = p.F2 > p.Fc ? p.F2 : p.Fc;
        const uint32_t Ec = (cb >> 23) & 0xFFu;
        const int ec = (int)(Ec ? Ec : 1u) - 127;
        const int E = have_T ? (ec > em ? ec : em) : ec;           // the accumulator always takes part
        if (have_T && p.sum_drop_distance && E - em >= p.sum_drop_distance) have_T = false;
        if (!have_T) T = 0.0;
        const double sc_exact = ldexp((double)__uint_as_float(cb), p.Fc - E);
        double sc = __builtin_floor(sc_exact);                                                    // RD_Fc(c at E), units of 2^(E - Fc)
        // (Sec. 6.2.4's hypothetical variant: both roundings truncate toward zero; unsplit groups, plain F2 rule)
        if ((fe & FL_RD_AS_RZ)) sc = __builtin_trunc(sc_exact);
        if ((fe & FL_SPECIAL_TRUNC) && ec < E - p.Fc - 1 && Ec != 0xFFu) sc = 0.0;             // (an infinite or NaN accumulator stays)
        double val;
        if (!(fe & FL_F2_LEADING)) {
            const double T_exact = ldexp(T, (em - FT) - (E - p.F2));
            double T2 = __builtin_floor(T_exact);                                                 // RD_F2(T at E)
            if ((fe & FL_RD_AS_RZ)) T2 = __builtin_trunc(T_exact);
            val = ldexp(ldexp(T2, Fmax - p.F2) + ldexp(sc, Fmax - p.Fc), E - Fmax);
        } else {
            // exact two-term sum as s + err (Knuth's TwoSum); then round down to F2 bits below the leading bit
            // of the exact sum.  |err| is below half a last place of s, far under that unit.
            const double a = ldexp(T, em - FT), b = ldexp(sc, E - p.Fc);
            const double sm = a + b, bb = sm - a;
            const double err = (a - (sm - bb)) + (b - bb);
            const long long sbits = __double_as_longlong(sm);
            int lead = (int)((sbits >> 52) & 0x7FF) - 1023;
            const bool toward_zero = (err != 0.0) && ((err < 0.0) != (sm < 0.0));
            if ((sbits & 0xFFFFFFFFFFFFFll) == 0 && toward_zero) lead -= 1;                      // just inside the binade below
            lead = lead < -126 ? -126 : lead;                                                     // binary32's smallest normal exponent
            const int unit = lead - p.F2;
            double q = __builtin_floor(ldexp(sm, -unit));
            if (err < 0.0 && ldexp(q, unit) == sm) q -= 1.0;                                      // s on the grid, exact sum just below it
            val = sm == 0.0 ? 0.0 : ldexp(q, unit);
        }
        return val;
    };

    // End of a group: rho of (sum of aligned terms) * 2^unit.  The value to convert is held
    // in binary64, exact or rounded to odd, so that the single hardware conversion to
    // binary32 (RNE, gradual underflow, overflow to infinity) rounds correctly.
    // conversion of the exact group values v, output rounding variants, the rare integer route, d <- result
    auto finish_group = [&](uint32_t kg, const double (&v)[R][C], const uint32_t (&tg)[R][C], uint32_t tagged) {
        uint32_t dn[R][C];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c) dn[r][c] = __float_as_uint((float)v[r][c]);
        if ((fe & (FL_ACC16 | FL_RZ | FL_FTZ_OUT | FL_ZERO_POSITIVE))) {       // (one test on the common path: none of them)
            if ((fe & FL_ACC16)) {
                // rho onto the binary16 grid: the value is first brought to binary32 rounded to odd (24 bits, far more than
                // binary16's 11 plus a guard bit), then one hardware conversion gives RNE-FP16 with gradual underflow and
                // overflow; RZ steps back where that rounded away from zero.  The accumulator keeps travelling as the
                // binary32 pattern of the binary16 result.
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        uint32_t fb = dn[r][c];
                        const double back = (double)__uint_as_float(fb);
                        if (back != v[r][c]) {                                             // inexact (a NaN stays a NaN through this)
                            if (__builtin_fabs(back) > __builtin_fabs(v[r][c])) fb -= 1u;
                            fb |= 1u;
                        }
                        uint32_t hb = float_bits_to_half_bits(fb);
                        if ((fe & FL_RZ) && (hb & 0x7FFFu) <= 0x7C00u) {
                            const double hv = (double)__uint_as_float(half_bits_to_float_bits(hb));
                            if (__builtin_fabs(hv) > __builtin_fabs(v[r][c])) hb -= 1u;
                        }
                        uint32_t o = half_bits_to_float_bits(hb);
                        if ((fe & FL_FTZ_OUT) && (o & 0x7F800000u) < (113u << 23)) o &= 0x80000000u;   // |d| < 2^-14
                        if ((fe & FL_ZERO_POSITIVE) && (o & 0x7FFFFFFFu) == 0) o = 0u;
                        dn[r][c] = o;
                    }
            } else {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        uint32_t o = dn[r][c];
                        if ((fe & FL_RZ)) {
                            const double back = (double)__uint_as_float(o);
                            if (__builtin_fabs(back) > __builtin_fabs(v[r][c])) o -= 1u;   // rounded away from zero: step back
                            o &= out_mask;                                               // RZ-E8M13 cuts further, still toward zero
                        }
                        if ((fe & FL_FTZ_OUT) && (o & 0x7F800000u) == 0) o &= 0x80000000u;
                        if ((fe & FL_ZERO_POSITIVE) && (o & 0x7FFFFFFFu) == 0) o = 0u;
                        dn[r][c] = o;
                    }
            }
        }
        if (tagged & SENTINEL_MASK) {                                   // rare: the group met a tagged element
            // NaN and infinity results first, for the whole block at once; then the integer routine for what is left
            // (the model parameters are fetched from the kernel-argument segment here, as in slow_group)
            const TiledArgs q = fetch_args();
            if constexpr (!SC && LT != 0) {
                // the group lies inside the staged chunk: classes and signs from the staged values.  Under the
                // product-overflow rule (the RD modes without `wide_products`) BF16 / TF32 groups are also tagged for a
                // large maximum exponent alone; of those, what the routine leaves unsettled has no special operand and
                // no product of 2^128 or more, and the value computed above stands.
                const bool rule = IS_RD && !q.p.wide_products;
                const uint32_t off = kg % KC;
                const bool dbl = VM == 2 || (VM == 1 && chunk_is_double);
                const void *pa = dbl ? static_cast<const void *>(avd + off) : static_cast<const void *>(av + off);
                const void *pb = dbl ? static_cast<const void *>(bvd + off) : static_cast<const void *>(bv + off);
                const uint2 sp = special_products<R, C, TI * VS, TJ * VS, TI * VSD, TJ * VSD, LT>(pa, pb, (dbl ? 1u : 0u) | (rule ? 2u : 0u));
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c)
                        if (tg[r][c] & SENTINEL_MASK) {
                            const uint32_t i = r * C + c, cb = d[r][c];
                            bool nn = (sp.x >> i) & 1u, pp = (sp.y >> i) & 1u, mm = (sp.y >> (16 + i)) & 1u;
                            if ((cb & 0x7FFFFFFFu) > 0x7F800000u) nn = true;                       // the accumulator joins
                            else if ((cb & 0x7FFFFFFFu) == 0x7F800000u) { if (cb >> 31) mm = true; else pp = true; }
                            if (nn || (pp && mm)) dn[r][c] = q.p.nan_bits;
                            else if (pp || mm) dn[r][c] = pp ? 0x7F800000u : 0xFF800000u;
                            // (else: tagged for its large maximum exponent alone -- a tagged element always gives one
                            // of the above -- and no product reached 2^128: the value computed above stands)
                        }
            } else {
                BlockVals<R * C> cin;
                uint32_t tm = 0;
#pragma unroll
                for (int i = 0; i < R * C; ++i) cin.v[i] = 0;
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c)
                        if (tg[r][c] & SENTINEL_MASK) {
                            cin.v[r * C + c] = d[r][c];
                            tm |= 1u << (r * C + c);
                        }
                const bool inf_final = !SC && (q.p.c_mode != MMAEMU_C_AFTER_RD || q.p.wide_products);
                const BlockVals<R * C> sp = special_block<R, C, TI, TJ>(A, B, my_tile * m + i_base, my_tile * n + j_base, k, kg, cin, tm, q.ta, q.tb,
                                                                        q.p.L, q.p.ftz_in, q.p.nan_bits, inf_final);
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c)
                        if (tg[r][c] & SENTINEL_MASK)
                            dn[r][c] = ((sp.settled >> (r * C + c)) & 1u) ? sp.v[r * C + c] : slow_group(r, c, kg, d[r][c]);
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c) d[r][c] = dn[r][c];
    };

    auto flush_accumulators = [&]() {
        if ((fe & FL_FTZ_IN)) {                                                 // FlushSubnormal on the accumulator
            const uint32_t first_normal = (fe & FL_ACC16) ? (113u << 23) : (1u << 23);  // 2^-14 for binary16, 2^-126
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int c = 0; c < C; ++c)
                    if ((d[r][c] & 0x7F800000u) < first_normal) d[r][c] = 0;
        }
    };

    auto end_of_group = [&](uint32_t kg, const int (&emax)[R][C], uint32_t tagged) {
        refresh_switches();
        flush_accumulators();
        double v[R][C];
        if (CMODE == MMAEMU_C_IN_GROUP) {
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    const double T = USE_SD ? Sd[r][c] + (double)S32[r][c] : (double)S32[r][c];
                    const int unit = emax[r][c] - F;
                    // the accumulator, aligned and truncated like every other term
                    const double tc = __builtin_trunc(ldexp((double)__uint_as_float(d[r][c]), -unit));
                    v[r][c] = ldexp(T + tc, unit);                      // exact: integers below 2^53
                }
        } else if (CMODE == MMAEMU_C_AFTER_RD) {
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    const double T = USE_SD ? Sd[r][c] + (double)S32[r][c] : (double)S32[r][c];   // units of 2^(e_max - F)
                    const uint32_t mx = m2[r][c], mlo = mx & 0xFFFFu, mhi = mx >> 16;
                    const bool have_T = !(fe & FL_SKIP_ZERO) || (mlo > mhi ? mlo : mhi) >= 2 * ZBIAS;
                    v[r][c] = rd_value(T, have_T, emax[r][c], F, d[r][c]);
                }
        } else {
            // d = rho(T 2^unit + c) with the two-term sum exact.  s = RN(a + c) is that sum unless it was rounded, and
            // it was not exactly when bb = RN(s - a) equals c and RN(s - bb) equals a: the difference of s and the
            // larger of the two operands is always representable, so one of the two tests compares exact
            // quantities and the other then does as well.  Only an inexact s (rare: the operands lie more than 29
            // binary places apart) needs its error term (Knuth's TwoSum); it is then rounded to odd (truncated
            // toward zero, last bit set), which the conversion below cannot tell from the exact sum.
            bool inexact = false;
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    const double T = USE_SD ? Sd[r][c] + (double)S32[r][c] : (double)S32[r][c];
                    const double a = ldexp(T, emax[r][c] - F);
                    const double cd = (double)__uint_as_float(d[r][c]);
                    const double s = a + cd;
                    const double bb = s - a;
                    v[r][c] = s;
                    inexact |= (bb != cd) || ((s - bb) != a);          // (true for NaN: infinite operands)
                }
            if (inexact) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        const double T = USE_SD ? Sd[r][c] + (double)S32[r][c] : (double)S32[r][c];
                        const double a = ldexp(T, emax[r][c] - F);
                        const double cd = (double)__uint_as_float(d[r][c]);
                        const double s = v[r][c], bb = s - a;
                        const double err = (a - (s - bb)) + (cd - bb);
                        if (__builtin_fabs(err) > 0.0) {                // (false for NaN)
                            long long sb = __double_as_longlong(s);
                            const bool toward_zero = (err < 0.0) != (s < 0.0);               // true value nearer zero
                            sb -= toward_zero ? 1 : 0;
                            v[r][c] = __longlong_as_double(sb | 1ll);
                        }
                    }
            }
        }
        finish_group(kg, v, m2, tagged);
    };

    // End of a split group (Algorithm "GTR-FDPA", steps 3 to 5): the two sub-group sums T0, T1 (units of 2^(e - F) at
    // their own maxima e0, e1; h0, h1: whether any term took part) are rounded down to F_m bits at the larger maximum
    // and added; then as TR-FDPA.
    auto end_of_split_group = [&](uint32_t kg, const double (&T0)[R][C], const int (&e0)[R][C], const uint32_t (&x0)[R][C],
                                  const double (&T1)[R][C], const int (&e1)[R][C], const uint32_t (&x1)[R][C], bool halves,
                                  uint32_t tagged) {
        refresh_switches();
        flush_accumulators();
        double v[R][C];
        uint32_t tg[R][C];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c) {
                // x0 / x1: the packed exponent maxima the sub-sums came from (both halves of the word for a half
                // group, the low / high half for the even / odd split)
                const uint32_t m0 = halves ? ((x0[r][c] & 0xFFFFu) > (x0[r][c] >> 16) ? (x0[r][c] & 0xFFFFu) : (x0[r][c] >> 16)) : (x0[r][c] & 0xFFFFu);
                const uint32_t m1 = halves ? ((x1[r][c] & 0xFFFFu) > (x1[r][c] >> 16) ? (x1[r][c] & 0xFFFFu) : (x1[r][c] >> 16)) : (x1[r][c] >> 16);
                const bool h0 = !(fe & FL_SKIP_ZERO) || m0 >= 2 * ZBIAS, h1 = !(fe & FL_SKIP_ZERO) || m1 >= 2 * ZBIAS;
                const int em = (h0 && h1) ? (e0[r][c] > e1[r][c] ? e0[r][c] : e1[r][c]) : (h0 ? e0[r][c] : e1[r][c]);
                double T = 0.0;
                if (h0) T += __builtin_floor(ldexp(T0[r][c], (e0[r][c] - F) - (em - p.Fm)));
                if (h1) T += __builtin_floor(ldexp(T1[r][c], (e1[r][c] - F) - (em - p.Fm)));
                v[r][c] = rd_value(T, h0 || h1, em, p.Fm, d[r][c]);
                tg[r][c] = x0[r][c] | x1[r][c];
            }
        finish_group(kg, v, tg, tagged);
    };

    auto reset_group = [&]() {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c) {
                m2[r][c] = 0; S32[r][c] = 0; Sd[r][c] = 0.0;
                if (CMODE == CM_RD_EVEN_ODD) S32o[CMODE == CM_RD_EVEN_ODD ? r : 0][CMODE == CM_RD_EVEN_ODD ? c : 0] = 0;
            }
    };

    // Staging is split in two: `prefetch` issues the global loads of a chunk (they complete
    // while the previous chunk is being computed), `commit` decodes and writes LDS.
    // WHAT bit 0: exponents, bit 1: values.  Elements are decoded into registers first; in the adaptive mode the workgroup then agrees (through the barrier
    // that also protects the previous chunk's readers) on whether any of them needs
    // binary64, and the values go to LDS in that form.
    typedef typename std::conditional<WIDE, uint4, uint2>::type Raw;
    Raw raw_a[NQA], raw_b[NQB];                                 // the next chunk's operands, in flight
    auto prefetch = [&](uint32_t k0) {
        load_panel<NQA>(esa, plan_a, k0, raw_a);
        load_panel<NQB>(esb, plan_b, k0, raw_b);
    };
    auto commit = [&](int what) {
        float fa[NQA][4], fb[NQB][4];
        uint2 xa[NQA], xb[NQB];
        const uint32_t zbias = (IS_RD && (fl & FL_SKIP_ZERO)) ? ZBIAS : 0u;
        bool wild = decode_any<NQA>(ta_.ta, raw_a, fl & FL_FTZ_IN, zbias, fa, xa);
        wild |= decode_any<NQB>(ta_.tb, raw_b, fl & FL_FTZ_IN, zbias, fb, xb);
        if (VM == 1) chunk_is_double = __syncthreads_or(wild && (what & 2)) != 0;
        else __syncthreads();
        store_panel<NQA, VS, VSD>(plan_a, fa, xa, Av_raw, Ae, chunk_is_double, what);
        store_panel<NQB, VS, VSD>(plan_b, fb, xb, Bv_raw, Be, chunk_is_double, what);
        __syncthreads();
    };

    auto pass2 = [&](int g, const int (&emax)[R][C]) {
        if (VM == 0) pass2f(g, emax);
        else if (VM == 2) pass2d(g, emax);
        else if (chunk_is_double) pass2d(g, emax);
        else pass2f(g, emax);
    };

    // the groups of one staged chunk, unsplit modes
    auto plain_groups = [&](uint32_t k0) {
        constexpr int GU = (R * C <= 4 && KC / GL <= 4 && CMODE != MMAEMU_C_AFTER_RD) ? KC / GL : 1;
#pragma unroll GU
        for (int g = 0; g < KC / GL; ++g) {
            reset_group();
            load_scales(k0 + g * GL);
            pass1(g);
            int emax[R][C]; uint32_t tagged = 0;
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int c = 0; c < C; ++c) exponents(r, c, emax[r][c], tagged);
            pass2(g, emax);
            end_of_group(k0 + g * GL, emax, tagged);
        }
    };

    prefetch(0);
    if (LT != 0) {
        for (uint32_t k0 = 0; k0 < k; k0 += KC) {
            commit(3);
            if (k0 + KC < k) prefetch(k0 + KC);
            if constexpr (CMODE == CM_RD_EVEN_ODD) {
#pragma unroll 1
                for (int g = 0; g < KC / GL; ++g) {
                    reset_group();
                    load_scales(k0 + g * GL);
                    pass1(g);
                    int ee[R][C], eo[R][C]; uint32_t tagged = 0;
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) {
                            ee[r][c] = (int)(m2[r][c] & 0xFFFFu) + ta_.ebase;      // even k sit in the low halves
                            eo[r][c] = (int)(m2[r][c] >> 16) + ta_.ebase;
                            tagged |= m2[r][c];
                        }
                    pass2eo(g, ee, eo);
                    if constexpr (SC) {
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int c = 0; c < C; ++c) {
                                const int s = (int)sca[r] + (int)scb[c] - 254;
                                ee[r][c] += s;
                                eo[r][c] += s;
                                const int em = ee[r][c] > eo[r][c] ? ee[r][c] : eo[r][c];
                                if ((sca[r] == 0xFFu || scb[c] == 0xFFu || (!(fl & FL_WIDE_PRODUCTS) && em >= 126)) && !(m2[r][c] & SENTINEL_MASK)) {
                                    m2[r][c] |= 0x8000u;
                                    tagged |= 0x8000u;
                                }
                            }
                    }
                    double Te[R][C], To[R][C];
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) { Te[r][c] = (double)S32[r][c]; To[r][c] = (double)S32o[CMODE == CM_RD_EVEN_ODD ? r : 0][CMODE == CM_RD_EVEN_ODD ? c : 0]; }
                    end_of_split_group(k0 + g * GL, Te, ee, m2, To, eo, m2, false, tagged);
                }
            } else if constexpr (CMODE == CM_RD_HALVES) {
#pragma unroll 1
                for (int g = 0; g < KC / LT; ++g) {
                    double T0[R][C]; int e0[R][C]; uint32_t x0[R][C];
                    int emax[R][C]; uint32_t tagged = 0;
                    reset_group();
                    load_scales(k0 + g * LT);
                    pass1(2 * g);
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) exponents(r, c, emax[r][c], tagged);
                    pass2f(2 * g, emax);
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) { T0[r][c] = (double)S32[r][c]; e0[r][c] = emax[r][c]; x0[r][c] = m2[r][c]; }
                    reset_group();
                    pass1(2 * g + 1);
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) exponents(r, c, emax[r][c], tagged);
                    pass2f(2 * g + 1, emax);
                    double T1[R][C];
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) T1[r][c] = (double)S32[r][c];
                    end_of_split_group(k0 + g * LT, T0, e0, x0, T1, emax, m2, true, tagged);
                }
            } else if constexpr (CMODE == CM_RD_QUARTERS) {
#pragma unroll 1
                for (int g = 0; g < KC / LT; ++g) {
                    int ep[4][R][C]; uint32_t tg[R][C], have[R][C], tagged = 0;
                    refresh_switches();
                    load_scales(k0 + g * LT);
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) { tg[r][c] = 0; have[r][c] = 0; }
                    // pass 1 over the four quarters: their maxima, and which of them hold a live product
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        reset_group();
                        pass1(4 * g + q);
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int c = 0; c < C; ++c) {
                                exponents(r, c, ep[q][r][c], tagged);
                                const uint32_t x = m2[r][c], mx = (x & 0xFFFFu) > (x >> 16) ? (x & 0xFFFFu) : (x >> 16);
                                tg[r][c] |= x;
                                if (!(fe & FL_SKIP_ZERO) || mx >= 2 * ZBIAS) have[r][c] |= 1u << q;
                            }
                    }
                    int em[R][C];
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) {
                            int e = ep[0][r][c]; bool any = (have[r][c] & 1u) != 0;
#pragma unroll
                            for (int q = 1; q < 4; ++q)
                                if ((have[r][c] >> q) & 1u) { e = (!any || ep[q][r][c] > e) ? ep[q][r][c] : e; any = true; }
                            em[r][c] = e;
                        }
                    // pass 2 quarter by quarter; each sum is rounded down to F_m bits at the largest maximum and added
                    double Tm[R][C];
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) Tm[r][c] = 0.0;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int c = 0; c < C; ++c) S32[r][c] = 0;
                        pass2f(4 * g + q, ep[q]);
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int c = 0; c < C; ++c)
                                if ((have[r][c] >> q) & 1u)
                                    Tm[r][c] += __builtin_floor(ldexp((double)S32[r][c], (ep[q][r][c] - F) - (em[r][c] - p.Fm)));
                    }
                    flush_accumulators();
                    double v[R][C];
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) v[r][c] = rd_value(Tm[r][c], have[r][c] != 0, em[r][c], p.Fm, d[r][c]);
                    finish_group(k0 + g * LT, v, tg, tagged);
                }
            } else {
                // (the groups of a chunk unrolled for the 2 x 2 kernels of the T-FDPA modes: their LDS addresses become
                // immediate offsets, -3.5 % on the headline kernel; the 4 x 4 kernels' bodies are too large for that to
                // pay, and some RD kernels lose a wave of occupancy to it)
                plain_groups(k0);
            }
        }
    } else {
        // a group of p.L terms spans p.L / KC chunks: one sweep for the exponents, one for the values
        for (uint32_t kg = 0; kg < k; kg += p.L) {
            reset_group();
            for (uint32_t k0 = kg; k0 < kg + p.L; k0 += KC) {
                commit(1);
                prefetch(k0 + KC < kg + p.L ? k0 + KC : kg);            // next chunk of this sweep, or back to the group's start
                pass1(0);
            }
            int emax[R][C]; uint32_t tagged = 0;
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int c = 0; c < C; ++c) exponents(r, c, emax[r][c], tagged);
            for (uint32_t k0 = kg; k0 < kg + p.L; k0 += KC) {
                commit(2);
                if (k0 + KC < k) prefetch(k0 + KC);                     // runs on into the next group's first chunk
                pass2(0, emax);
            }
            end_of_group(kg, emax, tagged);
        }
    }

    // a NaN accumulator propagates through the groups with whatever payload the hardware
    // gives it; the model's NaN encoding is applied once here
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int c = 0; c < C; ++c)
            if ((d[r][c] & 0x7FFFFFFFu) > 0x7F800000u) d[r][c] = nan_bits;
    auto put = [&](int r, int c) {
        const uint64_t o = d_off + (uint64_t)(TI * r) * n + TJ * c;
        if (fl & FL_ACC16) reinterpret_cast<uint16_t *>(D)[o] = (uint16_t)(d[r][c] == nan_bits ? p.nan16 : float_bits_to_half_bits(d[r][c]));
        else D[o] = d[r][c];
    };
    if constexpr (EDGES) {
        if (ragged) {
            if (live) {
                set_outputs(wg_index);                            // (the places again, rather than kept across the loops)
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c)
                        if (i_base + TI * r < m && j_base + TJ * c < n) put(r, c);
            }
            return;
        }
    }
    if (live) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c) put(r, c);
    }
}

// (On 32 x 32 x 8 tiles with groups of 4 or 8 the kernels of every accumulation mode but the first need 132 to 134 vector
// registers for binary32 values, a few over the budget of four waves per SIMD: those are compiled for four waves outright,
// +4 to 10 %.  The BF16 kernels, at 137 to 140, lose by it.)
template <int TM, int R, int C, int KC, int LT, int CMODE, int VM>
constexpr int tiled_min_waves()
{
    return (TM == 32 && R == 4 && C == 2 && KC == 8 && LT != 0 && CMODE != MMAEMU_C_IN_GROUP && VM == 0) ? 4 : 1;
}

template <int TM, int TN, int R, int C, int KC, int LT, int CMODE, int NF, int VM_>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(tiled_min_waves<TM, R, C, KC, LT, CMODE, VM_>())))
emulate_tiled_kernel(TiledArgs ta_, const void *__restrict__ A, const void *__restrict__ B, const uint32_t *Cm,
                     uint32_t *D, uint32_t m, uint32_t n, uint32_t k, uint64_t nitems, uint32_t bm_count,
                     uint32_t bn_count, uint32_t xcd_remap)
{
    tiled_body<TM, TN, R, C, KC, LT, CMODE, NF, VM_>(ta_, A, B, Cm, D, m, n, k, nitems, bm_count, bn_count, xcd_remap, blockIdx.x);
}

// ---- host side ---------------------------------------------------------------------------

template <int TM, int TN, int R, int C, int KC, int LT, int CMODE, int NF, int VM>
static mmaemu_status launch_cfg(const TiledArgs &ta, const void *A, const void *B, const void *Cm, void *D, uint32_t m,
                                uint32_t n, uint32_t k, uint64_t batch, hipStream_t s)
{
    constexpr int SLOTS = 256 / ((TM / R) * (TN / C));
    const uint32_t bm = (m + TM - 1) / TM, bn = (n + TN - 1) / TN;          // (edge blocks: see launch_tiled_shape)
    const uint64_t nitems = batch * bm * bn;
    const uint64_t blocks = (nitems + SLOTS - 1) / SLOTS;
    if (blocks > 0x7FFFFFFFull) { set_error("emulate_mma: too many blocks"); return MMAEMU_ERR_SHAPE; }
    const uint32_t remap = (blocks % 8 == 0 && blocks >= 64) ? 1u : 0u;
    hipLaunchKernelGGL((emulate_tiled_kernel<TM, TN, R, C, KC, LT, CMODE, NF, VM>), dim3((uint32_t)blocks), dim3(256), 0, s,
                       ta, A, B, (const uint32_t *)Cm, (uint32_t *)D, m, n, k, nitems, bm, bn, remap);
    MMAEMU_HIP(hipGetLastError());
    set_last_kernel("tiled %dx%d r%dx%d kc=%d L=%d c_mode=%d fold=%d vm=%d", TM, TN, R, C, KC, LT ? LT : (int)ta.p.L, CMODE,
                    NF, VM);
    return MMAEMU_OK;
}

// choose the fold period: the largest of {whole group, 4, 1} whose 32-bit partial sums cannot overflow
template <int TM, int TN, int R, int C, int KC, int LT, int CMODE, int VM>
static mmaemu_status launch_fold(const TiledArgs &ta, const void *A, const void *B, const void *Cm, void *D, uint32_t m,
                                 uint32_t n, uint32_t k, uint64_t batch, hipStream_t s)
{
    if constexpr (VM == 2) {
        return launch_cfg<TM, TN, R, C, KC, LT, CMODE, 0, VM>(ta, A, B, Cm, D, m, n, k, batch, s);   // terms summed in binary64
    } else if constexpr (CMODE == CM_RD_EVEN_ODD || CMODE == CM_RD_HALVES || CMODE == CM_RD_QUARTERS) {
        return launch_cfg<TM, TN, R, C, KC, LT, CMODE, 0, VM>(ta, A, B, Cm, D, m, n, k, batch, s);   // (the caller checked the 32-bit sums)
    } else {
        constexpr int GL = LT ? LT : KC;
        const uint64_t term = 1ull << (ta.p.F + 2);             // |aligned term| < 2^(F+2)
        if (GL * term <= (1ull << 31)) return launch_cfg<TM, TN, R, C, KC, LT, CMODE, 0, VM>(ta, A, B, Cm, D, m, n, k, batch, s);
        if (4 * term <= (1ull << 31)) return launch_cfg<TM, TN, R, C, KC, LT, CMODE, 4, VM>(ta, A, B, Cm, D, m, n, k, batch, s);
        return launch_cfg<TM, TN, R, C, KC, LT, CMODE, 1, VM>(ta, A, B, Cm, D, m, n, k, batch, s);
    }
}

template <int TM, int TN, int R, int C, int KC, int CMODE, int VM>
static mmaemu_status launch_L(const TiledArgs &ta, const void *A, const void *B, const void *Cm, void *D, uint32_t m,
                              uint32_t n, uint32_t k, uint64_t batch, hipStream_t s, bool &handled, bool edges = false)
{
    handled = true;
    const uint32_t L = ta.p.L;
    if constexpr (CMODE == CM_RD_EVEN_ODD || CMODE == CM_RD_HALVES || CMODE == CM_RD_QUARTERS) {
        // split groups: fixed lengths only, and half a group's aligned terms must fit one 32-bit sum
        if ((uint64_t)(L / 2) << (ta.p.F + 2) <= (1ull << 31)) {
            if constexpr (CMODE != CM_RD_QUARTERS) {
                if (L == 8) return launch_fold<TM, TN, R, C, KC, 8, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s);
            }
            if constexpr (KC >= 16) {
                if (L == 16) return launch_fold<TM, TN, R, C, KC, 16, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s);
            }
            if constexpr (KC >= 32) {
                if (L == 32) return launch_fold<TM, TN, R, C, KC, 32, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s);
            }
        }
        handled = false;
        return MMAEMU_OK;
    } else {
    if (L == 4) return launch_fold<TM, TN, R, C, KC, 4, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s);
    if (L == 8) return launch_fold<TM, TN, R, C, KC, 8, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s);
    if constexpr (KC >= 16) {
        if (L == 16) return launch_fold<TM, TN, R, C, KC, 16, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s);
    }
    if constexpr (KC >= 32) {
        if (L == 32) return launch_fold<TM, TN, R, C, KC, 32, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s);
    }
    if constexpr (VM != 3) {        // (a scaled group lies inside one chunk; so must the groups of a problem with edge blocks)
        if (L % KC == 0 && !edges) return launch_fold<TM, TN, R, C, KC, 0, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s);
    }
    handled = false;
    return MMAEMU_OK;
    }
}

template <int CMODE, int VM>
mmaemu_status launch_tiled_shape(const TiledArgs &ta, const void *A, const void *B, const void *Cm, void *D, uint32_t m,
                                 uint32_t n, uint32_t k, uint64_t batch, hipStream_t s, bool &handled)
{
    handled = false;
    const uint64_t outputs = batch * m * n;
    // Whole small tiles of a batch.  16 x 16 tiles take 2 x 2 register blocks: at about 100 vector registers such a kernel
    // runs four or five waves per SIMD, which on tiles this small is worth more than the halved LDS traffic of 4 x 4
    // blocks at two waves (measured 15 to 30 % on 16x16x16 / 16x16x32 tiles; 32x32x8 tiles are 4 to 10 % faster with 4 x 4).
    // Half and quarter groups keep a second set of sums and maxima per output: no 4 x 4 blocks for them anywhere.
    constexpr bool BIG_BLOCKS_OK = CMODE != CM_RD_HALVES && CMODE != CM_RD_QUARTERS;
    if constexpr (CMODE == CM_RD_QUARTERS) {
        // (groups of 32 on 16 x 16 tiles: staged 32 k at a time)
        if (m == 16 && n == 16 && k % 32 == 0 && ta.p.L == 32) return launch_L<16, 16, 2, 2, 32, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s, handled);
    }
    if (m == 16 && n == 16 && k % 16 == 0) return launch_L<16, 16, 2, 2, 16, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s, handled);
    if constexpr (VM == 4) {
        // (the TF32 instructions' own shape, 16 x 16 x 8)
        if (m == 16 && n == 16 && k % 8 == 0) return launch_L<16, 16, 2, 2, 8, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s, handled);
    }
    if (m == 32 && n == 32 && k % 8 == 0 && k % 32 != 0)
        return launch_L<32, 32, 4, 2, 8, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s, handled);
    // blocks of a larger problem: 4x4 register blocks once there are enough outputs to fill
    // the chip with them (256 CUs x 4 SIMDs x 2 waves x 64 lanes x 16), 2x2 blocks otherwise
    if (BIG_BLOCKS_OK && m % 64 == 0 && n % 64 == 0 && k % 32 == 0 && outputs >= (1ull << 21))
        return launch_L<64, 64, 4, 4, 32, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s, handled);
    if (m % 32 == 0 && n % 32 == 0 && k % 32 == 0)
        return launch_L<32, 32, 2, 2, 32, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s, handled);
    if (m % 32 == 0 && n % 32 == 0 && k % 8 == 0)
        return launch_L<32, 32, 4, 2, 8, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s, handled);
    if (m % 16 == 0 && n % 16 == 0 && k % 16 == 0) return launch_L<16, 16, 2, 2, 16, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s, handled);
    // The shapes of the four-product instructions (32x32x4 and 16x16x4 per block, k = 4 or an odd multiple of it, groups
    // of four): one quad of k per row and pass.
    if constexpr ((CMODE == MMAEMU_C_IN_GROUP || CMODE == MMAEMU_C_AFTER_RD) && (VM == 0 || VM == 1)) {
        if (k % 4 == 0 && ta.p.L == 4 && ((m == 32 && n == 32) || (m == 16 && n == 16))) {
            handled = true;
            if (m == 32) return launch_fold<32, 32, 4, 2, 4, 4, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s);
            return launch_fold<16, 16, 2, 2, 4, 4, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s);
        }
    }
    // Ragged m or n: 32 x 32 blocks whose edge blocks repeat the last row and store only what lies inside (groups of 4
    // to 32 terms, which lie inside a staged chunk; not the block-scaled kernels).  Tiles of 17 to 31 rows and columns
    // fill at least 28 % of their one block, which still beats one thread per output several times over (20 x 20 tiles:
    // x 5); narrower ones stay with the general kernel: padded to 32 x 32 they would mostly compute nothing.
    if constexpr (VM != 3) {
        if (m > 16 && n > 16 && k % 32 == 0) return launch_L<32, 32, 2, 2, 32, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s, handled, true);
        if (m > 16 && n > 16 && k % 8 == 0) return launch_L<32, 32, 4, 2, 8, CMODE, VM>(ta, A, B, Cm, D, m, n, k, batch, s, handled, true);
    }
    return MMAEMU_OK;
}

// explicit instantiations live in emulate_tiled_c<CMODE>v<VM>.hip (one translation unit each)
#define MMAEMU_TILED_SIG(CM, VM)                                                                                        \
    mmaemu_status launch_tiled_shape<CM, VM>(const TiledArgs &, const void *, const void *, const void *, void *, uint32_t, \
                                             uint32_t, uint32_t, uint64_t, hipStream_t, bool &)
extern template MMAEMU_TILED_SIG(MMAEMU_C_IN_GROUP, 0);
extern template MMAEMU_TILED_SIG(MMAEMU_C_IN_GROUP, 1);
extern template MMAEMU_TILED_SIG(MMAEMU_C_IN_GROUP, 2);
extern template MMAEMU_TILED_SIG(MMAEMU_C_AFTER_EXACT, 0);
extern template MMAEMU_TILED_SIG(MMAEMU_C_AFTER_EXACT, 1);
extern template MMAEMU_TILED_SIG(MMAEMU_C_AFTER_EXACT, 2);
extern template MMAEMU_TILED_SIG(MMAEMU_C_AFTER_RD, 0);
extern template MMAEMU_TILED_SIG(MMAEMU_C_AFTER_RD, 1);
extern template MMAEMU_TILED_SIG(MMAEMU_C_AFTER_RD, 2);
extern template MMAEMU_TILED_SIG(CM_RD_EVEN_ODD, 0);
extern template MMAEMU_TILED_SIG(CM_RD_HALVES, 0);
extern template MMAEMU_TILED_SIG(MMAEMU_C_IN_GROUP, 3);
extern template MMAEMU_TILED_SIG(MMAEMU_C_AFTER_EXACT, 3);
extern template MMAEMU_TILED_SIG(MMAEMU_C_AFTER_RD, 3);
extern template MMAEMU_TILED_SIG(CM_RD_EVEN_ODD, 3);
extern template MMAEMU_TILED_SIG(CM_RD_HALVES, 3);
extern template MMAEMU_TILED_SIG(CM_RD_QUARTERS, 0);
extern template MMAEMU_TILED_SIG(CM_RD_QUARTERS, 3);
extern template MMAEMU_TILED_SIG(MMAEMU_C_IN_GROUP, 4);
extern template MMAEMU_TILED_SIG(MMAEMU_C_AFTER_EXACT, 4);
extern template MMAEMU_TILED_SIG(MMAEMU_C_AFTER_RD, 4);

} // namespace mmaemu
