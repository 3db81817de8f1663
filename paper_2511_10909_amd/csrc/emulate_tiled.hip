// Tiled emulation kernels: the fast path of mmaemu_emulate_mma.
//
// What is computed is the chained FDPA model (paper Algorithm "Phi_FDPA") around the
// truncated fused dot-product-add (Algorithm "T-FDPA"); how it is computed is specific
// to CDNA4:
//
//   * A workgroup of 256 threads owns a block of D (one 64x64 block of a large problem,
//     or several whole 16x16 / 32x32 tiles of a batch); each thread owns a 4x4 register
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
//
// Elements whose value leaves the range in which the binary32 product is exact and
// normal (|x| outside [2^-31, 2^32), only possible for BF16), and NaN/infinity, are
// tagged with an exponent sentinel; a group that meets one is recomputed by the integer
// routine of the general kernel from the raw operands in global memory.
#include "fdpa_int.hpp"

namespace mmaemu {

constexpr uint32_t SENTINEL = 0x7000u;      // exponent tag of an element the fast path cannot take

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

template <int T>
__device__ __forceinline__ void decode_elem(uint32_t bits, uint32_t ftz_in, float &val, uint32_t &ex)
{
    using F = Fmt<T>;
    constexpr uint32_t EMASK = (1u << F::EB) - 1u, MMASK = (1u << F::MB) - 1u;
    const uint32_t E = (bits >> F::MB) & EMASK;
    uint32_t M = bits & MMASK, sign = (bits >> (F::W - 1)) & 1u;
    const bool special = F::IEEE ? (E == EMASK) : (E == EMASK && M == MMASK);
    if (ftz_in && E == 0) { M = 0; sign = 0; }                 // FlushSubnormal: -> +0.0
    const uint32_t sig = E ? (M | (1u << F::MB)) : M;
    ex = (E ? E : 1u) - 1u;
    const float mag = ldexpf((float)sig, (int)ex + 1 - F::BIAS - F::MB);   // exact
    const uint32_t vb = __float_as_uint(mag);
    const uint32_t E32 = vb >> 23;
    const bool wild = sig != 0 && (E32 < 96u || E32 > 158u);
    val = __uint_as_float(vb | (sign << 31));
    if (special || wild) { ex = SENTINEL; val = 0.0f; }
}

// four consecutive k elements of one row: raw little-endian bytes in `raw` (low 4*size bytes used)
template <int T>
__device__ __forceinline__ void decode4(uint2 raw, uint32_t ftz_in, float4 &v, uint2 &e)
{
    uint32_t b[4];
    if (Fmt<T>::W == 8) {
        b[0] = raw.x & 0xFFu; b[1] = (raw.x >> 8) & 0xFFu; b[2] = (raw.x >> 16) & 0xFFu; b[3] = raw.x >> 24;
    } else {
        b[0] = raw.x & 0xFFFFu; b[1] = raw.x >> 16; b[2] = raw.y & 0xFFFFu; b[3] = raw.y >> 16;
    }
    float f[4]; uint32_t x[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) decode_elem<T>(b[q], ftz_in, f[q], x[q]);
    v = make_float4(f[0], f[1], f[2], f[3]);
    e = make_uint2(x[0] | (x[1] << 16), x[2] | (x[3] << 16));
}

// Stage ROWS rows x KC k-elements (k contiguous in global memory) of `nslots` matrices.
//   src(slot,row) = base + (slot_row0[slot] + row) * k + k0      (in elements)
template <int T, int ROWS, int KC, int SLOTS, int VS, int ES>
__device__ __forceinline__ void stage_panel(const void *base, const uint64_t (&row0)[SLOTS], uint32_t k, uint32_t k0,
                                            uint32_t ftz_in, float *lv, uint32_t *le)
{
    constexpr int QUADS = SLOTS * ROWS * (KC / 4);
    using elem = typename Fmt<T>::elem;
    for (int q = threadIdx.x; q < QUADS; q += 256) {
        const int kq = q % (KC / 4), row = (q / (KC / 4)) % ROWS, slot = q / ((KC / 4) * ROWS);
        const elem *src = reinterpret_cast<const elem *>(base) + (row0[slot] + row) * (uint64_t)k + k0 + 4 * kq;
        uint2 raw;
        if (Fmt<T>::W == 8) { raw.x = *reinterpret_cast<const uint32_t *>(src); raw.y = 0; }
        else raw = *reinterpret_cast<const uint2 *>(src);
        float4 v; uint2 e;
        decode4<T>(raw, ftz_in, v, e);
        *reinterpret_cast<float4 *>(lv + (slot * ROWS + row) * VS + 4 * kq) = v;
        *reinterpret_cast<uint2 *>(le + (slot * ROWS + row) * ES + 2 * kq) = e;
    }
}

template <int ROWS, int KC, int SLOTS, int VS, int ES>
__device__ __forceinline__ void stage_any(uint32_t t, const void *base, const uint64_t (&row0)[SLOTS], uint32_t k,
                                          uint32_t k0, uint32_t ftz_in, float *lv, uint32_t *le)
{
    switch (t) {   // uniform
    case MMAEMU_FP8_E4M3: stage_panel<MMAEMU_FP8_E4M3, ROWS, KC, SLOTS, VS, ES>(base, row0, k, k0, ftz_in, lv, le); break;
    case MMAEMU_FP8_E5M2: stage_panel<MMAEMU_FP8_E5M2, ROWS, KC, SLOTS, VS, ES>(base, row0, k, k0, ftz_in, lv, le); break;
    case MMAEMU_FP16: stage_panel<MMAEMU_FP16, ROWS, KC, SLOTS, VS, ES>(base, row0, k, k0, ftz_in, lv, le); break;
    default: stage_panel<MMAEMU_BF16, ROWS, KC, SLOTS, VS, ES>(base, row0, k, k0, ftz_in, lv, le); break;
    }
}

// ---- per-group arithmetic ---------------------------------------------------------------

struct TiledArgs {
    ModelArgs p;
    uint32_t ta, tb;
    int32_t ebase;       // Exp = e' + ebase for a product: 2 - bias_a - bias_b
    uint32_t n32;        // terms that may be summed in 32 bits before folding (power of two)
    int32_t gap_lo;      // C_AFTER_EXACT: lowest (last place of c) - (unit of T) for which binary64 holds the sum
};

// rho of S * 2^unit (S an exactly represented integer in binary64)
__device__ __forceinline__ uint32_t convert_out(const ModelArgs &p, double S, int unit)
{
    const double v = ldexp(S, unit);                       // exact: no bits can fall below 2^-1074
    float f = (float)v;                                    // RNE, gradual underflow, overflow -> inf
    uint32_t d = __float_as_uint(f);
    if (p.out_round == MMAEMU_ROUND_RZ) {
        const double back = (double)f;
        if ((back < 0 ? -back : back) > (v < 0 ? -v : v)) d -= 1u;   // rounded away from zero: one step back
    }
    if (p.ftz_out && (d & 0x7F800000u) == 0) d &= 0x80000000u;
    return d;
}

// ---- the kernel -------------------------------------------------------------------------
// TM x TN: block of D per slot; SLOTS slots (independent tiles) per workgroup;
// KC: k elements staged at a time; LT: group length if it divides KC, 0 if the group
// spans whole chunks (L a multiple of KC, any length).
template <int TM, int TN, int KC, int LT, int CMODE>
__global__ void __launch_bounds__(256)
emulate_tiled_kernel(TiledArgs ta_, const void *__restrict__ A, const void *__restrict__ B, const uint32_t *C,
                     uint32_t *D, uint32_t m, uint32_t n, uint32_t k, uint64_t nitems, uint32_t bm_count,
                     uint32_t bn_count)
{
    constexpr int TI = TM / 4, TJ = TN / 4, TPS = TI * TJ, SLOTS = 256 / TPS;
    constexpr int VS = KC + 4;                       // LDS row strides (dwords), padded against bank conflicts
    constexpr int ES = KC / 2 + (KC == 16 ? 2 : 4);
    __shared__ __attribute__((aligned(16))) float Av[SLOTS * TM * VS];
    __shared__ __attribute__((aligned(16))) float Bv[SLOTS * TN * VS];
    __shared__ __attribute__((aligned(16))) uint32_t Ae[SLOTS * TM * ES];
    __shared__ __attribute__((aligned(16))) uint32_t Be[SLOTS * TN * ES];

    const ModelArgs &p = ta_.p;
    const int F = p.F;
    const uint32_t tid = threadIdx.x, slot = tid / TPS, ti = (tid % TPS) / TJ, tj = tid % TJ;

    // items handled by this workgroup: item = (tile, block row, block column)
    uint64_t arow0[SLOTS], brow0[SLOTS];
    const uint64_t item0 = (uint64_t)blockIdx.x * SLOTS;
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        uint64_t it = item0 + s;
        if (it >= nitems) it = nitems - 1;                      // surplus slots redo the last item, results discarded
        const uint64_t tile = it / ((uint64_t)bm_count * bn_count);
        const uint32_t rem = (uint32_t)(it % ((uint64_t)bm_count * bn_count));
        arow0[s] = tile * m + (uint64_t)(rem / bn_count) * TM;
        brow0[s] = tile * n + (uint64_t)(rem % bn_count) * TN;
    }
    const bool live = item0 + slot < nitems;
    uint64_t my_it = item0 + slot;
    if (my_it >= nitems) my_it = nitems - 1;
    const uint64_t my_tile = my_it / ((uint64_t)bm_count * bn_count);
    const uint32_t my_rem = (uint32_t)(my_it % ((uint64_t)bm_count * bn_count));
    const uint32_t i_base = (my_rem / bn_count) * TM + ti, j_base = (my_rem % bn_count) * TN + tj;

    uint32_t d[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c)
            d[r][c] = C[(my_tile * m + i_base + TI * r) * (uint64_t)n + j_base + TJ * c];

    const float *av = Av + (slot * TM + ti) * VS;
    const float *bv = Bv + (slot * TN + tj) * VS;
    const uint32_t *ae = Ae + (slot * TM + ti) * ES;
    const uint32_t *be = Be + (slot * TN + tj) * ES;
    const uint32_t esize_a = ta_.ta <= MMAEMU_FP8_E5M2 ? 1u : 2u, esize_b = ta_.tb <= MMAEMU_FP8_E5M2 ? 1u : 2u;

    const uint32_t Lrt = p.L;                                   // run-time group length (== LT when LT != 0)
    constexpr int GL = LT ? LT : KC;                            // terms handled per inner step
    uint32_t m2[4][4];                                          // packed running maxima of e'
    double Sd[4][4];

    auto run_group_pass1 = [&](int g) {
#pragma unroll
        for (int q = 0; q < GL / 2; ++q) {
            uint32_t ea[4], eb[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) ea[r] = ae[TI * r * ES + g * (GL / 2) + q];
#pragma unroll
            for (int c = 0; c < 4; ++c) eb[c] = be[TJ * c * ES + g * (GL / 2) + q];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) m2[r][c] = pk_max_u16(m2[r][c], pk_add_u16(ea[r], eb[c]));
        }
    };

    // pass 2 over GL terms with per-element scale; S32 folded into Sd every n32 terms
    auto run_group_pass2 = [&](int g, const float (&scale)[4][4]) {
        int32_t S32[4][4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c) S32[r][c] = 0;
#pragma unroll
        for (int q = 0; q < GL; ++q) {
            float a[4], b[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) a[r] = av[TI * r * VS + g * GL + q];
#pragma unroll
            for (int c = 0; c < 4; ++c) b[c] = bv[TJ * c * VS + g * GL + q];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) S32[r][c] += (int32_t)((a[r] * b[c]) * scale[r][c]);
            if (((q + 1) & (int)(ta_.n32 - 1)) == 0 || q == GL - 1) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int c = 0; c < 4; ++c) { Sd[r][c] += (double)S32[r][c]; S32[r][c] = 0; }
            }
        }
    };

    // exponent bookkeeping at the end of pass 1 of a whole group; returns false if the
    // element must take the integer route
    auto finish_pass1 = [&](int r, int c, int &emax, float &scale) -> bool {
        uint32_t e = m2[r][c];
        uint32_t em = (e & 0xFFFFu) > (e >> 16) ? (e & 0xFFFFu) : (e >> 16);
        if (em >= SENTINEL) return false;
        emax = (int)em + ta_.ebase;
        const uint32_t cb = d[r][c];
        if ((cb & 0x7F800000u) == 0x7F800000u) return false;          // NaN / infinite accumulator
        if (CMODE == MMAEMU_C_IN_GROUP) {
            const uint32_t Ec = (cb >> 23) & 0xFFu;                    // (a flushed subnormal keeps Exp = -126)
            const int ec = (int)(Ec ? Ec : 1u) - 127;
            emax = ec > emax ? ec : emax;
        }
        int se = F - emax + 127;                                       // biased exponent of 2^(F - e_max)
        se = se < 1 ? 1 : (se > 254 ? 254 : se);                       // clamps never change a truncated term
        scale = __uint_as_float((uint32_t)se << 23);
        return true;
    };

    auto finish_group = [&](int r, int c, int emax) {
        const int unit = emax - F;
        uint32_t cb = d[r][c];
        if (p.ftz_in && (cb & 0x7F800000u) == 0) cb = 0;               // FlushSubnormal on C (and on a chained d)
        const float cf = __uint_as_float(cb);
        if (CMODE == MMAEMU_C_IN_GROUP) {
            // accumulator aligned and truncated like any other term
            const double tc = trunc(ldexp((double)cf, -unit));
            d[r][c] = convert_out(p, Sd[r][c] + tc, unit);
        } else {
            // d = rho(T 2^unit + c) with the sum exact: binary64 holds it exactly when both
            // terms fit 53 bits together; |T| < 2^31 + folds (< 2^42), c has 24 bits
            const double T = Sd[r][c];
            const uint32_t Ec = (cb >> 23) & 0xFFu;
            const int lsb_c = (int)(Ec ? Ec : 1u) - 150;
            const int gap = lsb_c - unit;
            const bool c_zero = (cb & 0x7FFFFFFFu) == 0;
            if (T == 0.0 || c_zero || (gap >= ta_.gap_lo && gap <= 28)) {
                const double v = ldexp(T, unit) + (double)cf;
                float f = (float)v;
                uint32_t o = __float_as_uint(f);
                if (v == 0.0) o = 0u;                                    // exact zero -> +0.0
                else {
                    if (p.out_round == MMAEMU_ROUND_RZ) {
                        const double back = (double)f;
                        if ((back < 0 ? -back : back) > (v < 0 ? -v : v)) o -= 1u;
                    }
                    if (p.ftz_out && (o & 0x7F800000u) == 0) o &= 0x80000000u;
                }
                d[r][c] = o;
            } else {
                const uint32_t neg = T < 0;
                const uint64_t mag = (uint64_t)(neg ? -T : T);
                const uint32_t csig = (cb & 0x7FFFFFu) | (Ec ? 0x800000u : 0u);
                uint32_t o = add_exact_round(neg, mag, unit, cb >> 31, (uint64_t)csig, lsb_c, p.out_round);
                if (p.ftz_out && (o & 0x7F800000u) == 0) o &= 0x80000000u;
                d[r][c] = o;
            }
        }
    };

    auto slow_group = [&](int r, int c, uint32_t kg) {
        const uint64_t arow = my_tile * m + i_base + TI * r;
        const uint64_t brow = (my_tile * n + j_base + TJ * c);
        const uint8_t *a = reinterpret_cast<const uint8_t *>(A) + (arow * k + kg) * esize_a;
        const uint8_t *b = reinterpret_cast<const uint8_t *>(B) + (brow * k + kg) * esize_b;
        d[r][c] = fdpa_group_raw(p, ta_.ta, ta_.tb, a, b, Lrt, d[r][c]);
    };

    if (LT != 0) {
        for (uint32_t k0 = 0; k0 < k; k0 += KC) {
            __syncthreads();
            stage_any<TM, KC, SLOTS, VS, ES>(ta_.ta, A, arow0, k, k0, p.ftz_in, Av, Ae);
            stage_any<TN, KC, SLOTS, VS, ES>(ta_.tb, B, brow0, k, k0, p.ftz_in, Bv, Be);
            __syncthreads();
#pragma unroll 1
            for (int g = 0; g < KC / GL; ++g) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int c = 0; c < 4; ++c) { m2[r][c] = 0; Sd[r][c] = 0.0; }
                run_group_pass1(g);
                float scale[4][4]; int emax[4][4]; uint32_t slow = 0;
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        scale[r][c] = 0.0f; emax[r][c] = 0;
                        if (!finish_pass1(r, c, emax[r][c], scale[r][c])) slow |= 1u << (4 * r + c);
                    }
                run_group_pass2(g, scale);
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        if (slow & (1u << (4 * r + c))) slow_group(r, c, k0 + g * GL);
                        else finish_group(r, c, emax[r][c]);
                    }
            }
        }
    } else {
        // group = Lrt terms spanning Lrt / KC chunks: sweep the group's chunks twice
        for (uint32_t kg = 0; kg < k; kg += Lrt) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) { m2[r][c] = 0; Sd[r][c] = 0.0; }
            for (uint32_t k0 = kg; k0 < kg + Lrt; k0 += KC) {
                __syncthreads();
                stage_any<TM, KC, SLOTS, VS, ES>(ta_.ta, A, arow0, k, k0, p.ftz_in, Av, Ae);
                stage_any<TN, KC, SLOTS, VS, ES>(ta_.tb, B, brow0, k, k0, p.ftz_in, Bv, Be);
                __syncthreads();
                run_group_pass1(0);
            }
            float scale[4][4]; int emax[4][4]; uint32_t slow = 0;
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    scale[r][c] = 0.0f; emax[r][c] = 0;
                    if (!finish_pass1(r, c, emax[r][c], scale[r][c])) slow |= 1u << (4 * r + c);
                }
            for (uint32_t k0 = kg; k0 < kg + Lrt; k0 += KC) {
                __syncthreads();
                stage_any<TM, KC, SLOTS, VS, ES>(ta_.ta, A, arow0, k, k0, p.ftz_in, Av, Ae);
                stage_any<TN, KC, SLOTS, VS, ES>(ta_.tb, B, brow0, k, k0, p.ftz_in, Bv, Be);
                __syncthreads();
                run_group_pass2(0, scale);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (slow & (1u << (4 * r + c))) slow_group(r, c, kg);
                    else finish_group(r, c, emax[r][c]);
                }
        }
    }

    if (live) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c)
                D[(my_tile * m + i_base + TI * r) * (uint64_t)n + j_base + TJ * c] = d[r][c];
    }
}

// ---- host side ---------------------------------------------------------------------------

template <int TM, int TN, int KC, int LT, int CMODE>
static mmaemu_status launch_cfg(const TiledArgs &ta, const void *A, const void *B, const void *C, void *D, uint32_t m,
                                uint32_t n, uint32_t k, uint64_t batch, hipStream_t s)
{
    constexpr int SLOTS = 256 / ((TM / 4) * (TN / 4));
    const uint32_t bm = m / TM, bn = n / TN;
    const uint64_t nitems = batch * bm * bn;
    const uint64_t blocks = (nitems + SLOTS - 1) / SLOTS;
    if (blocks > 0x7FFFFFFFull) { set_error("emulate_mma: too many blocks"); return MMAEMU_ERR_SHAPE; }
    hipLaunchKernelGGL((emulate_tiled_kernel<TM, TN, KC, LT, CMODE>), dim3((uint32_t)blocks), dim3(256), 0, s, ta, A, B,
                       (const uint32_t *)C, (uint32_t *)D, m, n, k, nitems, bm, bn);
    MMAEMU_HIP(hipGetLastError());
    set_last_kernel("tiled %dx%d kc=%d L=%d c_mode=%d", TM, TN, KC, LT ? LT : (int)ta.p.L, CMODE);
    return MMAEMU_OK;
}

template <int TM, int TN, int KC, int CMODE>
static mmaemu_status launch_L(const TiledArgs &ta, const void *A, const void *B, const void *C, void *D, uint32_t m,
                              uint32_t n, uint32_t k, uint64_t batch, hipStream_t s, bool &handled)
{
    handled = true;
    const uint32_t L = ta.p.L;
    if (L == 4 && KC % 4 == 0) return launch_cfg<TM, TN, KC, 4, CMODE>(ta, A, B, C, D, m, n, k, batch, s);
    if (L == 8 && KC % 8 == 0) return launch_cfg<TM, TN, KC, 8, CMODE>(ta, A, B, C, D, m, n, k, batch, s);
    if constexpr (KC >= 16) {
        if (L == 16 && KC % 16 == 0) return launch_cfg<TM, TN, KC, 16, CMODE>(ta, A, B, C, D, m, n, k, batch, s);
    }
    if constexpr (KC >= 32) {
        if (L == 32 && KC % 32 == 0) return launch_cfg<TM, TN, KC, 32, CMODE>(ta, A, B, C, D, m, n, k, batch, s);
    }
    if (L % KC == 0) return launch_cfg<TM, TN, KC, 0, CMODE>(ta, A, B, C, D, m, n, k, batch, s);
    handled = false;
    return MMAEMU_OK;
}

template <int CMODE>
static mmaemu_status launch_shape(const TiledArgs &ta, const void *A, const void *B, const void *C, void *D, uint32_t m,
                                  uint32_t n, uint32_t k, uint64_t batch, hipStream_t s, bool &handled)
{
    handled = false;
    if (m == 16 && n == 16 && k % 16 == 0)
        return launch_L<16, 16, 16, CMODE>(ta, A, B, C, D, m, n, k, batch, s, handled);
    if (m == 32 && n == 32 && k % 8 == 0 && k <= 16)
        return launch_L<32, 32, 8, CMODE>(ta, A, B, C, D, m, n, k, batch, s, handled);
    if (m % 64 == 0 && n % 64 == 0 && k % 32 == 0)
        return launch_L<64, 64, 32, CMODE>(ta, A, B, C, D, m, n, k, batch, s, handled);
    if (m % 32 == 0 && n % 32 == 0 && k % 8 == 0)
        return launch_L<32, 32, 8, CMODE>(ta, A, B, C, D, m, n, k, batch, s, handled);
    if (m % 16 == 0 && n % 16 == 0 && k % 16 == 0)
        return launch_L<16, 16, 16, CMODE>(ta, A, B, C, D, m, n, k, batch, s, handled);
    return MMAEMU_OK;
}

mmaemu_status launch_emulate(const ModelArgs &p, const void *A, const void *B, const void *C, void *D,
                             uint32_t m, uint32_t n, uint32_t k, uint64_t batch, uint32_t ta, uint32_t tb,
                             hipStream_t s)
{
    // the tiled kernels take F <= 29 (an aligned term must fit a 32-bit integer), loads of
    // four consecutive k elements (alignment of A and B to 4 elements is implied by k % 4 == 0
    // and base alignment, checked here), and sums below 2^53
    const bool aligned = ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 7) == 0;
    if (p.F <= 29 && aligned && (uint64_t)p.L <= (1ull << (50 - p.F))) {
        TiledArgs t;
        t.p = p;
        t.ta = ta;
        t.tb = tb;
        t.ebase = 2 - fmt_info(ta).bias - fmt_info(tb).bias;
        uint32_t n32 = 1;
        while (n32 < 1024 && (uint64_t)(2 * n32) << (p.F + 2) <= (1ull << 31)) n32 *= 2;
        t.n32 = n32;
        uint32_t lg = 0;
        while ((1ull << lg) < p.L) ++lg;
        const int tbits = p.F + 2 + (int)lg;                 // |T| < 2^tbits
        t.gap_lo = tbits >= 52 ? 0 : -(52 - tbits);
        bool handled = false;
        mmaemu_status st = p.c_mode == MMAEMU_C_IN_GROUP
                               ? launch_shape<MMAEMU_C_IN_GROUP>(t, A, B, C, D, m, n, k, batch, s, handled)
                               : launch_shape<MMAEMU_C_AFTER_EXACT>(t, A, B, C, D, m, n, k, batch, s, handled);
        if (handled) return st;
    }
    return launch_emulate_generic(p, A, B, C, D, m, n, k, batch, ta, tb, s);
}

} // namespace mmaemu
