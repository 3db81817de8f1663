// The closed-loop scan in one launch (Sec. 3.1 Step 4: many candidate parameter sets over the same random tiles, each
// compared bit by bit with a reference, Eq. 2): up to MULTI_MAX models of one family and of *any* group length, internal
// width and fold period share the staged operands of a pass.  Families (one kernel instantiation each): T-FDPA with the
// accumulator inside the sum; TR-FDPA (the accumulator added after the products' sum, with the two round-downs and the
// variation switches); TR-FDPA on groups split in halves or quarters; GTR-FDPA (the even / odd split).  What follows
// describes the first; the others differ in what a group's maximum covers and in the group epilogue.
//
// Staging and decoding A and B, loading C and the reference and forming the exponent maxima cost about as much as
// running one model, so that part is paid once per pass for all the models of a launch:
//   * a workgroup pass stages four 16x16x16 or 16x16x32 tiles (one 32x32x8 or 32x32x16 tile), the whole k at once, as the
//     single-model kernels of emulate_tiled.hpp do (same LDS layout and helpers);
//   * pass 1 runs once at the finest granularity, a quarter group of four products: the packed 16-bit maximum of each
//     quarter is kept in LDS, two quarters per dword and thread;
//   * the model loop reads per model six scalars from the kernel-argument segment (F, switches, output mask, NaN
//     pattern, L, arithmetic kind); a group's maximum is the maximum of its quarters; pass 2 is a run-time loop over
//     the group in steps of four k (one 128-bit LDS read per row and step);
//   * arithmetic kinds: 0, the whole group summed in 32 bits; 1, folded into binary64 every four terms; 2, every term;
//     3, F of 30 and more: terms truncated and summed in binary64 (values widened on load where the chunk is held in
//     binary32);
//   * group epilogue: the binary64 route of the single-model kernels, or (kind 0, every output of the wavefront with a
//     normal result and no tagged element) a 32-bit route: the accumulator aligned like a product, the sum an integer,
//     rho one int -> float conversion under the wavefront's rounding mode and an exact scaling;
//   * every output is compared with the reference in registers; a differing output does one LDS atomic on a histogram
//     bucket, the largest distance and first index are reduced over the wavefront by row shifts; a persistent workgroup
//     writes its non-zero counters out once, at its end (a global atomic on a shared cache line costs about as much as a
//     thousand instructions of a wave).
// Models that flush subnormal inputs come last in a launch (the staged values are flushed in place once).
#include "emulate_tiled.hpp"

namespace mmaemu {

struct ScanArgs {
    uint32_t ta, tb;
    int32_t ebase;                     // Exp = e' + ebase for a product
    uint32_t count;                    // models in this launch, 1 .. MULTI_MAX
    uint32_t ref_is_first;             // no reference array: the first model's outputs are the reference
    const uint32_t *dref;              // reference outputs [batch][m][n], or null
    uint32_t *dout;                    // null, or every model's outputs: model i at dout + slot[i] * out_stride
    uint64_t out_stride, index_base;
    uint64_t *stats;                   // the caller's mmaemu_stats array as 64-bit words
    uint32_t zbias;                    // ZBIAS when zero terms stay out of the exponent maxima (TR-FDPA sets with that switch), else 0
    uint32_t slot[MULTI_MAX];
    struct Hot { int32_t F; uint32_t flags, out_mask, nan_bits, L, kind; int32_t F2, Fc, drop, Fm; uint32_t parts, twin; } hot[MULTI_MAX];
};

__device__ __forceinline__ ScanArgs::Hot scan_hot(uint32_t mi)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef const __attribute__((address_space(4))) ScanArgs *KArgs;
    KArgs sa = (KArgs)__builtin_amdgcn_kernarg_segment_ptr();
    ScanArgs::Hot h;
    h.F = sa->hot[mi].F; h.flags = sa->hot[mi].flags; h.out_mask = sa->hot[mi].out_mask; h.nan_bits = sa->hot[mi].nan_bits;
    h.L = sa->hot[mi].L; h.kind = sa->hot[mi].kind;
    h.F2 = sa->hot[mi].F2; h.Fc = sa->hot[mi].Fc; h.drop = sa->hot[mi].drop; h.Fm = sa->hot[mi].Fm; h.parts = sa->hot[mi].parts; h.twin = sa->hot[mi].twin;
    return h;
#else
    return ScanArgs::Hot{};
#endif
}

// TM x TM x KC tiles (16 x 16 x 16, 16 x 16 x 32, 32 x 32 x 8 or 32 x 32 x 16: the whole k of a tile is staged at once), 2 x 2
// outputs per thread; ADAPT: BF16 operands, whose staged chunk is
// held in binary64 when any element lies outside [2^-31, 2^32).
// (Four waves per SIMD are asked for outright where the LDS allows four workgroups per CU: left alone the compiler settles
// at about 150 vector registers and three waves; the handful of registers that go to scratch instead cost less than the
// fourth wave brings: +6 % on both workloads.  Five waves were slower.  The 16 x 16 x 32 instantiations hold two or three
// workgroups per CU and are compiled for that many waves.)
// Algorithm "TR-FDPA", steps 3 and 4, and the variations of it that the model switches name, in binary64 (every quantity
// is an integer of fewer than 53 bits times a power of two, hence exact): T counts units of 2^(em - F) (have_T: a product
// took part), cb is the accumulator; returns the exact value whose conversion is the group's result.
__device__ __forceinline__ double scan_rd_value(double T, bool have_T, int em, int F, uint32_t cb, int F2, int Fc, int drop, uint32_t fl)
{
    const int Fmax = F2 > Fc ? F2 : Fc;
    const uint32_t Ec = (cb >> 23) & 0xFFu;
    const int ec = (int)(Ec ? Ec : 1u) - 127;
    const int E = have_T ? (ec > em ? ec : em) : ec;                      // the accumulator always takes part
    if (have_T && drop && E - em >= drop) have_T = false;                 // the product sum lies too far below: it drops out
    if (!have_T) T = 0.0;
    const double sc_exact = ldexp((double)__uint_as_float(cb), Fc - E);
    double sc = (fl & FL_RD_AS_RZ) ? __builtin_trunc(sc_exact) : __builtin_floor(sc_exact);     // RD_Fc(c at E), units of 2^(E - Fc)
    if ((fl & FL_SPECIAL_TRUNC) && ec < E - Fc - 1 && Ec != 0xFFu) sc = 0.0;                   // (an infinite or NaN accumulator stays)
    if (!(fl & FL_F2_LEADING)) {
        const double T_exact = ldexp(T, (em - F) - (E - F2));
        const double T2 = (fl & FL_RD_AS_RZ) ? __builtin_trunc(T_exact) : __builtin_floor(T_exact);   // RD_F2(T at E)
        return ldexp(ldexp(T2, Fmax - F2) + ldexp(sc, Fmax - Fc), E - Fmax);
    }
    // F2 counted from the leading bit of the exact two-term sum, held as s + err (Knuth's TwoSum; |err| is below half a
    // last place of s, far under the unit that is kept)
    const double a = ldexp(T, em - F), b = ldexp(sc, E - Fc);
    const double sm = a + b, bb = sm - a;
    const double err = (a - (sm - bb)) + (b - bb);
    const long long sbits = __double_as_longlong(sm);
    int lead = (int)((sbits >> 52) & 0x7FF) - 1023;
    const bool toward_zero = (err != 0.0) && ((err < 0.0) != (sm < 0.0));
    if ((sbits & 0xFFFFFFFFFFFFFll) == 0 && toward_zero) lead -= 1;        // just inside the binade below
    lead = lead < -126 ? -126 : lead;                                       // binary32's smallest normal exponent
    const int unit = lead - F2;
    double q = __builtin_floor(ldexp(sm, -unit));
    if (err < 0.0 && ldexp(q, unit) == sm) q -= 1.0;                        // s on the grid, the exact sum just below it
    return sm == 0.0 ? 0.0 : ldexp(q, unit);
}

// LDS of one workgroup: staged values and exponents, the kept quarter maxima, the statistics
template <int TM, int KC, bool ADAPT, int FAM>
constexpr int scan_lds_bytes()
{
    constexpr int SLOTS = 256 / ((TM / 2) * (TM / 2));
    constexpr int VS = KC + 4, VSD = KC + 2, ES = KC / 2 + (KC == 8 ? 4 : 2);
    constexpr int KEPT = FAM == 3 ? KC / 4 : (KC / 4 + 1) / 2;            // dwords of kept maxima per output
    return 2 * SLOTS * TM * (ADAPT ? VSD * 8 : VS * 4) + 2 * SLOTS * TM * ES * 4 + KEPT * 4 * 256 * 4 + (int)sizeof(MultiLds);
}
// workgroups (of four waves, one per SIMD) that a CU's 160 KB of LDS hold, four at most: the waves per SIMD to compile for
template <int TM, int KC, bool ADAPT, int FAM>
constexpr int scan_waves()
{
    constexpr int by_lds = (160 * 1024) / scan_lds_bytes<TM, KC, ADAPT, FAM>();
    return by_lds >= 4 ? 4 : by_lds;
}

// FAM 0: T-FDPA, the accumulator a term of the sum; FAM 1: TR-FDPA (unsplit groups), the accumulator added after the
// products' sum with the two round-downs; FAM 2: GTR-FDPA's merge of sub-group sums with the sub-groups being the two
// halves or the four quarters of a group (binary32 values only: FP8 / FP16 operands, a sub-group's sum in 32 bits); FAM 3:
// GTR-FDPA as printed, the sub-groups being the even and the odd products.
// TWIN (FAM 0, tiles of one group): a model marked `twin` is followed by one that differs from it only in the output
// conversion (rounding, E8M13, output flush, NaN pattern); the two share the group's maximum and sum, and only the end of
// the group and the statistics run twice.
template <int TM, int KC, bool ADAPT, int FAM, bool TWIN>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(scan_waves<TM, KC, ADAPT, FAM>(), scan_waves<TM, KC, ADAPT, FAM>())))
emulate_scan_kernel(ScanArgs sa_, const void *__restrict__ A, const void *__restrict__ B, const uint32_t *Cm, uint64_t nitems, uint32_t nblocks)
{
    constexpr int R = 2, C = 2, TN = TM;
    constexpr int TI = TM / R, TJ = TN / C, TPS = TI * TJ, SLOTS = 256 / TPS;
    static_assert(TPS * SLOTS == 256, "thread layout");
    constexpr int VS = KC + 4, VSD = KC + 2, ES = KC / 2 + (KC == 8 ? 4 : 2);
    constexpr int NQ4 = KC / 4;                                   // quarter groups per row
    constexpr int NK2 = (NQ4 + 1) / 2;                            // dwords of kept maxima per output
    constexpr int VBYTES = SLOTS * TM * (ADAPT ? VSD * 8 : VS * 4);
    constexpr int EBYTES = SLOTS * TM * ES * 4;
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * VBYTES + 2 * EBYTES];
    __shared__ uint32_t m2k[FAM == 3 ? NQ4 : NK2][R * C][256];            // (FAM 3: a quarter's even and odd maximum, one dword)
    __shared__ MultiLds ml;
    constexpr int HC = HIST_COPIES;
    const uint32_t tid = threadIdx.x;
    for (uint32_t i = tid; i < MULTI_MAX * 34 * HC; i += 256) (&ml.hist[0][0][0])[i] = 0;
    if (tid < MULTI_MAX) { ml.naneq[tid] = 0; ml.maxd[tid] = 0; ml.first[tid] = ~0ull; }
    // (the first staging's barriers come before any thread counts anything)

    unsigned char *Av_raw = smem, *Bv_raw = smem + VBYTES;
    uint32_t *Ae = reinterpret_cast<uint32_t *>(smem + 2 * VBYTES);
    uint32_t *Be = reinterpret_cast<uint32_t *>(smem + 2 * VBYTES + EBYTES);
    const ScanArgs *sa = reinterpret_cast<const ScanArgs *>(opaque_kernarg_ptr());
    const uint32_t slot = tid / TPS, ti = (tid % TPS) / TJ, tj = tid % TJ;
    const uint32_t ta = sa_.ta, tb = sa_.tb;
    const int ebase = sa_.ebase;
    const uint32_t esa = (ta <= MMAEMU_FP8_E5M2 || ta >= MMAEMU_FP6_E2M3) ? 1u : 2u;
    const uint32_t esb = (tb <= MMAEMU_FP8_E5M2 || tb >= MMAEMU_FP6_E2M3) ? 1u : 2u;
    const float *av = reinterpret_cast<const float *>(Av_raw) + (slot * TM + ti) * VS;
    const float *bv = reinterpret_cast<const float *>(Bv_raw) + (slot * TN + tj) * VS;
    const double *avd = reinterpret_cast<const double *>(Av_raw) + (slot * TM + ti) * VSD;
    const double *bvd = reinterpret_cast<const double *>(Bv_raw) + (slot * TN + tj) * VSD;
    const uint32_t *ae = Ae + (slot * TM + ti) * ES;
    const uint32_t *be = Be + (slot * TN + tj) * ES;
    const uint32_t count = sa_.count, ref_first = sa_.ref_is_first;
    const bool dumping = sa_.dout != nullptr;
    const uint32_t *dref = sa->dref;

    constexpr int NQ = (SLOTS * TM * (KC / 4) + 255) / 256;
    // AHEAD (the 32 x 32 tiles of FP8 / FP16 operands, whose kernels have registers to spare under the four-wave budget):
    // a pass's global loads (operand quads, accumulator inputs, reference) are issued one pass ahead, right after the
    // previous pass has been staged, so that they arrive while its models run.
    constexpr bool AHEAD = TM == 32 && !ADAPT && FAM == 0;
    constexpr int NA = AHEAD ? NQ : 1, RA = AHEAD ? R : 1, CA = AHEAD ? C : 1;
    uint2 nraw_a[NA], nraw_b[NA];
    uint32_t nc0[RA][CA], nref[RA][CA];
    auto fetch_pass = [&](uint32_t wg) {
        if constexpr (AHEAD) {
            const uint64_t it0 = (uint64_t)wg * SLOTS;
            StagePlan<NQ> pa, pb;
            make_plan<TM, KC, SLOTS, VS, ES, true, NQ>(pa, A, esa, it0, nitems, 1u, 1u, TM, KC);
            make_plan<TN, KC, SLOTS, VS, ES, false, NQ>(pb, B, esb, it0, nitems, 1u, 1u, TN, KC);
            load_panel<NQ>(esa, pa, 0, nraw_a);
            load_panel<NQ>(esb, pb, 0, nraw_b);
            const uint64_t tile = it0 + slot < nitems ? it0 + slot : nitems - 1;
            const uint64_t off = (tile * TM + ti) * (uint64_t)TN + tj;
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    const uint64_t o = off + (uint64_t)(TI * r) * TN + TJ * c;
                    nc0[r][c] = Cm[o];
                    nref[r][c] = ref_first ? 0u : dref[o];
                }
        }
    };
    if (AHEAD && blockIdx.x < nblocks) fetch_pass(blockIdx.x);
    for (uint32_t pass_wg = blockIdx.x; pass_wg < nblocks; pass_wg += gridDim.x) {
        // ---- this pass's tiles: staging plans, outputs, operands in flight ----
        const uint64_t item0 = (uint64_t)pass_wg * SLOTS;
        StagePlan<NQ> plan_a, plan_b;
        make_plan<TM, KC, SLOTS, VS, ES, true, NQ>(plan_a, A, esa, item0, nitems, 1u, 1u, TM, KC);
        make_plan<TN, KC, SLOTS, VS, ES, false, NQ>(plan_b, B, esb, item0, nitems, 1u, 1u, TN, KC);
        uint2 raw_a[NQ], raw_b[NQ];
        if constexpr (AHEAD) {
#pragma unroll
            for (int q = 0; q < NQ; ++q) { raw_a[q] = nraw_a[q]; raw_b[q] = nraw_b[q]; }
        } else {
            load_panel<NQ>(esa, plan_a, 0, raw_a);
            load_panel<NQ>(esb, plan_b, 0, raw_b);
        }
        const bool live = item0 + slot < nitems;
        const uint64_t my_tile = live ? item0 + slot : nitems - 1;
        const uint64_t d_off = (my_tile * TM + ti) * (uint64_t)TN + tj;             // + TI * r * TN + TJ * c
        uint32_t c0[R][C], ref[R][C];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < C; ++c) {
                if constexpr (AHEAD) {
                    c0[r][c] = nc0[r][c];
                    ref[r][c] = nref[r][c];
                } else {
                    const uint64_t o = d_off + (uint64_t)(TI * r) * TN + TJ * c;
                    c0[r][c] = Cm[o];
                    ref[r][c] = ref_first ? 0u : dref[o];
                }
            }
        // ---- decode and stage (as the first model wants them) ----
        bool chunk_is_double = false;
        int staged;
        {
            const uint32_t ftz0 = scan_hot(0).flags & FL_FTZ_IN;
            staged = ftz0 ? 1 : 0;
            float fa[NQ][4], fb[NQ][4];
            uint2 xa[NQ], xb[NQ];
            const uint32_t zbias = FAM != 0 ? sa_.zbias : 0u;
            bool wild = decode_any<NQ>(ta, raw_a, ftz0, zbias, fa, xa);
            wild |= decode_any<NQ>(tb, raw_b, ftz0, zbias, fb, xb);
            if (ADAPT) chunk_is_double = __syncthreads_or(wild) != 0;         // (also protects the previous pass's readers)
            else __syncthreads();
            store_panel<NQ, VS, VSD>(plan_a, fa, xa, Av_raw, Ae, chunk_is_double, 3);
            store_panel<NQ, VS, VSD>(plan_b, fb, xb, Bv_raw, Be, chunk_is_double, 3);
            __syncthreads();
        }
        if (AHEAD && pass_wg + gridDim.x < nblocks) fetch_pass(pass_wg + gridDim.x);
        // ---- pass 1, once: the maximum of e'_a + e'_b over each quarter group, two quarters per kept dword ----
#pragma unroll
        for (int q = 0; q < NQ4; ++q) {
            uint2 ea[R], eb[C];
#pragma unroll
            for (int r = 0; r < R; ++r) ea[r] = *reinterpret_cast<const uint2 *>(ae + TI * r * ES + 2 * q);
#pragma unroll
            for (int c = 0; c < C; ++c) eb[c] = *reinterpret_cast<const uint2 *>(be + TJ * c * ES + 2 * q);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    const uint32_t x = pk_max_u16(pk_add_u16(ea[r].x, eb[c].x), pk_add_u16(ea[r].y, eb[c].y));
                    const uint32_t lo = x & 0xFFFFu, hi = x >> 16;
                    const uint32_t mx = lo > hi ? lo : hi;
                    // (each thread its own words: no barrier needed)
                    if constexpr (FAM == 3) m2k[q][r * C + c][tid] = x;           // low half: the even k, high half: the odd k
                    else if (q % 2 == 0) m2k[q / 2][r * C + c][tid] = mx;
                    else m2k[q / 2][r * C + c][tid] |= mx << 16;
                }
        }

        // ---- the models ----
#pragma unroll 1
        for (uint32_t mi = 0; mi < count; ++mi) {
            const ScanArgs::Hot hot = scan_hot(mi);
            const int F = hot.F;
            const uint32_t fl = hot.flags, L = hot.L, kind = hot.kind;
            typename std::conditional<TWIN, uint32_t, const uint32_t>::type out_mask = hot.out_mask, nan_bits = hot.nan_bits;
            typename std::conditional<TWIN, uint32_t, const uint32_t>::type fe = fl;   // the switches the end of a group reads (a twin brings its own)
            const bool twin = TWIN && hot.twin != 0;
            uint32_t dfirst[TWIN ? R : 1][TWIN ? C : 1];      // the first model's outputs of a pair of twins
            const uint32_t nan_first = hot.nan_bits;
            // rho = RZ-FP32: the short route's int -> float conversion truncates under the binary32 rounding mode "toward
            // zero" (every other binary32 operation of the loop is exact in either mode, and the binary64 route checks the
            // direction of its own conversion)
            if constexpr (FAM == 0) set_f32_round_toward_zero((fl & FL_RZ) != 0);
            (void)kind;
            if ((fl & FL_FTZ_IN) && !staged) {
                // FlushSubnormal on the staged values, in place (exponents do not change: a subnormal keeps Exp = 1 - bias)
                __syncthreads();
                const float min_a = min_normal_of(ta), min_b = min_normal_of(tb);
                if (chunk_is_double) {
                    double *va = reinterpret_cast<double *>(Av_raw), *vb = reinterpret_cast<double *>(Bv_raw);
                    _Pragma("unroll 1") for (uint32_t i = tid; i < SLOTS * TM * VSD; i += 256) if (__builtin_fabs(va[i]) < (double)min_a) va[i] = 0.0;
                    _Pragma("unroll 1") for (uint32_t i = tid; i < SLOTS * TN * VSD; i += 256) if (__builtin_fabs(vb[i]) < (double)min_b) vb[i] = 0.0;
                } else {
                    float *va = reinterpret_cast<float *>(Av_raw), *vb = reinterpret_cast<float *>(Bv_raw);
                    _Pragma("unroll 1") for (uint32_t i = tid; i < SLOTS * TM * VS; i += 256) if (__builtin_fabsf(va[i]) < min_a) va[i] = 0.0f;
                    _Pragma("unroll 1") for (uint32_t i = tid; i < SLOTS * TN * VS; i += 256) if (__builtin_fabsf(vb[i]) < min_b) vb[i] = 0.0f;
                }
                __syncthreads();
                staged = 1;
            }
            uint32_t d[R][C];
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int c = 0; c < C; ++c) d[r][c] = c0[r][c];
            bool slow_seen = false;                           // some group left the short route (a NaN may have come out of it)
            // The groups of one model, specialised on the group length GL and the arithmetic kind so that the loops
            // unroll and the LDS addresses of a group are immediate offsets.
            auto run_groups = [&](auto gl_c, auto kind_c) {
                constexpr int GL = decltype(gl_c)::value, KIND = decltype(kind_c)::value;
                constexpr int U2 = (GL / 4 <= 2) ? 2 : 1;             // (a whole group of 16 in flight costs a wave of occupancy)
                if constexpr (GL <= KC && FAM <= 1) {
                const bool fits = KIND == 0 && ((uint64_t)(GL + 1) << (F + 2)) <= (1ull << 31) && F >= 1;
#pragma unroll 1
                for (int g = 0; g < KC / GL; ++g) {
                    const uint32_t kg = g * GL;
                    // e_max of the group: its quarters' maxima, then the accumulator
                    int emax[R][C];
                    uint32_t tagged = 0, tg[R][C];
                    bool have[R][C];                          // (FAM 1) a product took part
                    auto group_max = [&](int r, int c) -> uint32_t {
                        if constexpr (GL == 4) {
                            return (m2k[g / 2][r * C + c][tid] >> (16 * (g & 1))) & 0xFFFFu;
                        } else {
                            uint32_t x = m2k[g * (GL / 8)][r * C + c][tid];
#pragma unroll
                            for (int i = 1; i < GL / 8; ++i) x = pk_max_u16(x, m2k[g * (GL / 8) + i][r * C + c][tid]);
                            const uint32_t lo = x & 0xFFFFu, hi = x >> 16;
                            return lo > hi ? lo : hi;
                        }
                    };
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) {
                            uint32_t e = group_max(r, c);
                            const int em = (int)e + ebase;
                            have[r][c] = true;
                            if constexpr (FAM == 1) {
                                // (zero terms kept out of the maxima: a product with a zero factor has an exponent sum below 2 ZBIAS)
                                have[r][c] = !(fl & FL_SKIP_ZERO) || e >= 2 * ZBIAS;
                                // a BF16 product may reach 2^128, which this family counts as an infinity: tagged, and settled
                                // from the staged values (such a chunk is held in binary64, where products are exact)
                                if (ADAPT && em >= 127 && !(e & 0xC000u)) e |= 0x8000u;
                                tg[r][c] = e & 0xC000u;
                                tagged |= e;
                                emax[r][c] = em;
                                continue;
                            }
                            tg[r][c] = e & 0xC000u;
                            tagged |= e;
                            uint32_t dd = d[r][c];
                            if ((fl & FL_FTZ_IN) && (dd & 0x7F800000u) == 0) { dd = 0; d[r][c] = 0; }     // FlushSubnormal on the accumulator
                            const uint32_t Ec = (dd >> 23) & 0xFFu;                                        // (a flushed subnormal keeps Exp = -126)
                            const int ec = (int)(Ec ? Ec : 1u) - 127;
                            emax[r][c] = ec > em ? ec : em;
                        }
                    tagged &= 0xC000u;
                    // ---- pass 2 ----
                    int32_t S32[R][C];
                    double Sd[R][C];
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) { S32[r][c] = 0; Sd[r][c] = 0.0; }
                    auto fold = [&]() {
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int c = 0; c < C; ++c) { Sd[r][c] += (double)S32[r][c]; S32[r][c] = 0; }
                    };
                    float fscale[R][C];                           // 2^(F - e_max) in binary32, where pass 2 runs in binary32
                    if ((ADAPT && chunk_is_double) || KIND == 3) {
                        // binary64: exact product, exact scaling; the float -> int conversion truncates, or (KIND 3: F of 30
                        // and more) v_trunc_f64 and a binary64 sum, exact below 2^53
                        double scale[R][C];
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int c = 0; c < C; ++c) scale[r][c] = __hiloint2double((F - emax[r][c] + 1023) << 20, 0);   // 2^(F - e_max), always normal
#pragma unroll 1
                        for (int q = 0; q < GL; q += 2) {
                            double a[R][2], b[C][2];
                            if (ADAPT && chunk_is_double) {
#pragma unroll
                                for (int r = 0; r < R; ++r) { const double2 v = *reinterpret_cast<const double2 *>(avd + TI * r * VSD + kg + q); a[r][0] = v.x; a[r][1] = v.y; }
#pragma unroll
                                for (int c = 0; c < C; ++c) { const double2 v = *reinterpret_cast<const double2 *>(bvd + TJ * c * VSD + kg + q); b[c][0] = v.x; b[c][1] = v.y; }
                            } else {
#pragma unroll
                                for (int r = 0; r < R; ++r) { const float2 v = *reinterpret_cast<const float2 *>(av + TI * r * VS + kg + q); a[r][0] = (double)v.x; a[r][1] = (double)v.y; }
#pragma unroll
                                for (int c = 0; c < C; ++c) { const float2 v = *reinterpret_cast<const float2 *>(bv + TJ * c * VS + kg + q); b[c][0] = (double)v.x; b[c][1] = (double)v.y; }
                            }
#pragma unroll
                            for (int w = 0; w < 2; ++w) {
#pragma unroll
                                for (int r = 0; r < R; ++r)
#pragma unroll
                                    for (int c = 0; c < C; ++c) {
                                        const double t = (a[r][w] * b[c][w]) * scale[r][c];
                                        if constexpr (KIND == 3) Sd[r][c] += __builtin_trunc(t);
                                        else S32[r][c] += (int32_t)t;
                                    }
                                if constexpr (KIND == 2) fold();
                            }
                            if constexpr (KIND == 1) { if ((q & 2) != 0) fold(); }
                        }
                    } else {
                        // binary32 values: the product is exact, the scaling aligns it, the conversion truncates toward zero
                        float (&scale)[R][C] = fscale;
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int c = 0; c < C; ++c) {
                                int se = F + 127 - emax[r][c];                         // biased exponent of 2^(F - e_max)
                                se = se < 1 ? 1 : (se > 254 ? 254 : se);               // the clamps never change a truncated term
                                scale[r][c] = __uint_as_float((uint32_t)se << 23);
                            }
#pragma unroll U2
                        for (int q = 0; q < GL; q += 4) {
                            float a[R][4], b[C][4];
#pragma unroll
                            for (int r = 0; r < R; ++r) {
                                const float4 v = *reinterpret_cast<const float4 *>(av + TI * r * VS + kg + q);
                                a[r][0] = v.x; a[r][1] = v.y; a[r][2] = v.z; a[r][3] = v.w;
                            }
#pragma unroll
                            for (int c = 0; c < C; ++c) {
                                const float4 v = *reinterpret_cast<const float4 *>(bv + TJ * c * VS + kg + q);
                                b[c][0] = v.x; b[c][1] = v.y; b[c][2] = v.z; b[c][3] = v.w;
                            }
#pragma unroll
                            for (int w = 0; w < 4; ++w) {
#pragma unroll
                                for (int r = 0; r < R; ++r)
#pragma unroll
                                    for (int c = 0; c < C; ++c) S32[r][c] += (int32_t)((a[r][w] * b[c][w]) * scale[r][c]);
                                if constexpr (KIND == 2) fold();
                            }
                            if constexpr (KIND == 1) fold();
                        }
                    }

                    // ---- end of the group ----
                    // Short route: when the GL truncated products and the truncated accumulator together fit 32 bits, the
                    // accumulator is aligned like a product, the whole sum is a 32-bit integer, and rho is the int -> float
                    // conversion followed by an exact scaling -- as long as the result cannot be subnormal and nothing is
                    // tagged: e_max - F >= -126 and e_max <= 127 for every output of the wavefront.
                    uint32_t dkeep[TWIN ? R : 1][TWIN ? C : 1];
                    if constexpr (TWIN) {
                        if (twin) {
#pragma unroll
                            for (int r = 0; r < R; ++r)
#pragma unroll
                                for (int c = 0; c < C; ++c) dkeep[r][c] = d[r][c];
                        }
                    }
                    constexpr int TWINS = TWIN ? 2 : 1;
#pragma unroll 1
                    for (int tw = 0; tw < TWINS && (tw == 0 || twin); ++tw) {
                    if constexpr (TWIN) {
                        if (tw == 1) {
                            // the twin: the first model's outputs aside, the accumulator back, the twin's output conversion
                            const ScanArgs::Hot h2 = scan_hot(mi + 1);
#pragma unroll
                            for (int r = 0; r < R; ++r)
#pragma unroll
                                for (int c = 0; c < C; ++c) { dfirst[r][c] = d[r][c]; d[r][c] = dkeep[r][c]; }
                            if constexpr (TWIN) {
                                fe = h2.flags;
                                out_mask = h2.out_mask;
                                nan_bits = h2.nan_bits;
                            }
                            set_f32_round_toward_zero((fe & FL_RZ) != 0);
                        }
                    }
                    bool done = false;
                    if constexpr (KIND == 0 && FAM == 0) {
                        if (fits) {
                            uint32_t worst = tagged ? 0xFFFFFFFFu : 0u;
#pragma unroll
                            for (int r = 0; r < R; ++r)
#pragma unroll
                                for (int c = 0; c < C; ++c) {
                                    const uint32_t u = (uint32_t)(emax[r][c] - (F - 126));          // 0 .. 253 - F on this route
                                    worst = u > worst ? u : worst;
                                }
                            if (__all(worst <= (uint32_t)(253 - F))) {
#pragma unroll
                                for (int r = 0; r < R; ++r)
#pragma unroll
                                    for (int c = 0; c < C; ++c) {
                                        // 2^(F - e_max), a normal number on this route (so pass 2's clamps left it alone)
                                        // (the BF16 kernels form it again: kept across their binary64 branch it costs registers)
                                        const float scale = ADAPT ? __uint_as_float((uint32_t)(F + 127 - emax[r][c]) << 23) : fscale[r][c];
                                        const int32_t S = S32[r][c] + (int32_t)(__uint_as_float(d[r][c]) * scale);
                                        const float f = (float)S;                                  // (truncates under RZ)
                                        uint32_t o = __float_as_uint(ldexpf(f, emax[r][c] - F));
                                        if ((fe & FL_RZ)) {
                                            if ((o & 0x7FFFFFFFu) == 0x7F800000u) o -= 1u;         // overflow: the largest finite number
                                            o &= out_mask;
                                        }
                                        d[r][c] = o;
                                    }
                                done = true;
                            }
                        }
                    }
                    if (!done) {
                        slow_seen = true;
                        uint32_t dn[R][C];
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int c = 0; c < C; ++c) {
                                const double T = Sd[r][c] + (double)S32[r][c];
                                double v;
                                if constexpr (FAM == 0) {
                                    const int unit = emax[r][c] - F;
                                    // the accumulator, aligned and truncated like every other term
                                    const double tc = __builtin_trunc(ldexp((double)__uint_as_float(d[r][c]), -unit));
                                    v = ldexp(T + tc, unit);                                   // exact: integers below 2^53
                                } else {
                                    if ((fl & FL_FTZ_IN) && (d[r][c] & 0x7F800000u) == 0) d[r][c] = 0;         // FlushSubnormal on the accumulator
                                    v = scan_rd_value(T, have[r][c], emax[r][c], F, d[r][c], hot.F2, hot.Fc, hot.drop, fl);
                                }
                                uint32_t o = __float_as_uint((float)v);
                                if ((fe & FL_RZ)) {
                                    const double back = (double)__uint_as_float(o);
                                    if (__builtin_fabs(back) > __builtin_fabs(v)) o -= 1u;     // rounded away from zero: step back
                                    o &= out_mask;                                             // RZ-E8M13 cuts further, still toward zero
                                }
                                if ((fe & FL_FTZ_OUT) && (o & 0x7F800000u) == 0) o &= 0x80000000u;
                                if (FAM == 1 && (fl & FL_ZERO_POSITIVE) && (o & 0x7FFFFFFFu) == 0) o = 0u;
                                dn[r][c] = o;
                            }
                        if (tagged) {
                            // NaN and infinite operands (Sec. 4.2): classes and signs from the staged values
                            const bool dbl = ADAPT && chunk_is_double;
                            const void *pa = dbl ? static_cast<const void *>(avd + kg) : static_cast<const void *>(av + kg);
                            const void *pb = dbl ? static_cast<const void *>(bvd + kg) : static_cast<const void *>(bv + kg);
                            // (FAM 1: under the product-overflow rule a finite product of 2^128 or more counts as an infinity;
                            // a group tagged for its large maximum alone in which no product gets there keeps the value above)
                            const uint2 sp = special_products<R, C, TI * VS, TJ * VS, TI * VSD, TJ * VSD, GL>(pa, pb, (dbl ? 1u : 0u) | (FAM == 1 ? 2u : 0u));
#pragma unroll
                            for (int r = 0; r < R; ++r)
#pragma unroll
                                for (int c = 0; c < C; ++c)
                                    if (tg[r][c]) {
                                        const uint32_t i = r * C + c, cb = d[r][c];
                                        bool nn = (sp.x >> i) & 1u, pp = (sp.y >> i) & 1u, mm = (sp.y >> (16 + i)) & 1u;
                                        if ((cb & 0x7FFFFFFFu) > 0x7F800000u) nn = true;                       // the accumulator joins
                                        else if ((cb & 0x7FFFFFFFu) == 0x7F800000u) { if (cb >> 31) mm = true; else pp = true; }
                                        if (nn || (pp && mm)) dn[r][c] = nan_bits;
                                        else if (pp || mm) dn[r][c] = pp ? 0x7F800000u : 0xFF800000u;
                                    }
                        }
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int c = 0; c < C; ++c) d[r][c] = dn[r][c];
                    }
                    }
                }
                }
            };
            auto by_kind = [&](auto gl_c) {
                if (kind == 0) run_groups(gl_c, std::integral_constant<int, 0>{});
                else if (kind == 1) run_groups(gl_c, std::integral_constant<int, 1>{});
                else if (kind == 2) run_groups(gl_c, std::integral_constant<int, 2>{});
                else run_groups(gl_c, std::integral_constant<int, 3>{});
            };
            // End of a split group: T, the merged sum of the sub-groups in units of 2^(em - F_m) (hv: some product took
            // part); then as TR-FDPA with F_m in the place of F, rho, and Sec. 4.2's special values from the staged values
            // of the whole group of GLT terms at kg.
            auto finish_merged = [&](auto glt_c, uint32_t kg, const double (&T)[R][C], const bool (&hv)[R][C], const int (&em)[R][C],
                                     const uint32_t (&tg)[R][C], uint32_t tagged) {
                constexpr int GLT = decltype(glt_c)::value;
                slow_seen = true;
                uint32_t dn[R][C];
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        if ((fl & FL_FTZ_IN) && (d[r][c] & 0x7F800000u) == 0) d[r][c] = 0;                 // FlushSubnormal on the accumulator
                        const double v = scan_rd_value(T[r][c], hv[r][c], em[r][c], hot.Fm, d[r][c], hot.F2, hot.Fc, hot.drop, fl);
                        uint32_t o = __float_as_uint((float)v);
                        if ((fl & FL_RZ)) {
                            const double back = (double)__uint_as_float(o);
                            if (__builtin_fabs(back) > __builtin_fabs(v)) o -= 1u;             // rounded away from zero: step back
                            o &= out_mask;
                        }
                        if ((fl & FL_FTZ_OUT) && (o & 0x7F800000u) == 0) o &= 0x80000000u;
                        if ((fl & FL_ZERO_POSITIVE) && (o & 0x7FFFFFFFu) == 0) o = 0u;
                        dn[r][c] = o;
                    }
                if (tagged) {
                    const uint2 sp = special_products<R, C, TI * VS, TJ * VS, TI * VSD, TJ * VSD, GLT>(av + kg, bv + kg, 2u);
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c)
                            if (tg[r][c]) {
                                const uint32_t i = r * C + c, cb = d[r][c];
                                bool nn = (sp.x >> i) & 1u, pp = (sp.y >> i) & 1u, mm = (sp.y >> (16 + i)) & 1u;
                                if ((cb & 0x7FFFFFFFu) > 0x7F800000u) nn = true;                           // the accumulator joins
                                else if ((cb & 0x7FFFFFFFu) == 0x7F800000u) { if (cb >> 31) mm = true; else pp = true; }
                                if (nn || (pp && mm)) dn[r][c] = nan_bits;
                                else if (pp || mm) dn[r][c] = pp ? 0x7F800000u : 0xFF800000u;
                            }
                }
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c) d[r][c] = dn[r][c];
            };
            // Split groups (Algorithm "GTR-FDPA", steps 3 to 5, with consecutive sub-groups): every sub-group of SL terms is
            // summed at its own maximum; the sums are rounded down to F_m bits at the largest maximum of the sub-groups
            // that hold a product and added; then as TR-FDPA with F_m in the place of F.
            auto run_split = [&](auto sl_c, auto ns_c) {
                constexpr int SL = decltype(sl_c)::value, NS = decltype(ns_c)::value, GLT = SL * NS;
                constexpr int US = (SL / 4 <= 2) ? 2 : 1;
                if constexpr (GLT <= KC && !ADAPT && FAM == 2) {
#pragma unroll 1
                for (int g = 0; g < KC / GLT; ++g) {
                    const uint32_t kg = g * GLT;
                    // the packed maximum of sub-group sg of the staged tile (SL terms), from the kept quarter maxima
                    auto sub_max = [&](int sg, int r, int c) -> uint32_t {
                        if constexpr (SL == 4) {
                            return (m2k[sg / 2][r * C + c][tid] >> (16 * (sg & 1))) & 0xFFFFu;
                        } else {
                            uint32_t x = m2k[sg * (SL / 8)][r * C + c][tid];
#pragma unroll
                            for (int i = 1; i < SL / 8; ++i) x = pk_max_u16(x, m2k[sg * (SL / 8) + i][r * C + c][tid]);
                            const uint32_t lo = x & 0xFFFFu, hi = x >> 16;
                            return lo > hi ? lo : hi;
                        }
                    };
                    int em[R][C];
                    uint32_t tg[R][C], have[R][C], tagged = 0;
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) {
                            tg[r][c] = 0;
                            have[r][c] = 0;
                            int best = 0, first = 0;
#pragma unroll
                            for (int q = 0; q < NS; ++q) {
                                const uint32_t e = sub_max(g * NS + q, r, c);
                                tg[r][c] |= e & 0xC000u;
                                tagged |= e;
                                const int eq = (int)e + ebase;
                                if (q == 0) first = eq;
                                if (!(fl & FL_SKIP_ZERO) || e >= 2 * ZBIAS) {
                                    best = (!have[r][c] || eq > best) ? eq : best;
                                    have[r][c] |= 1u << q;
                                }
                            }
                            em[r][c] = have[r][c] ? best : first;
                        }
                    tagged &= 0xC000u;
                    double Tm[R][C];
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) Tm[r][c] = 0.0;
                    // (one sub-group at a time, its maximum read again: four sets of maxima and sums in flight cost registers)
#pragma unroll 1
                    for (int q = 0; q < NS; ++q) {
                        int32_t S32[R][C];
                        int eq[R][C];
                        float scale[R][C];
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int c = 0; c < C; ++c) {
                                S32[r][c] = 0;
                                eq[r][c] = (int)sub_max(g * NS + q, r, c) + ebase;
                                int se = F + 127 - eq[r][c];                           // biased exponent of 2^(F - e_max)
                                se = se < 1 ? 1 : (se > 254 ? 254 : se);               // the clamps never change a truncated term
                                scale[r][c] = __uint_as_float((uint32_t)se << 23);
                            }
#pragma unroll US
                        for (int t = 0; t < SL; t += 4) {
                            float a[R][4], b[C][4];
#pragma unroll
                            for (int r = 0; r < R; ++r) {
                                const float4 v = *reinterpret_cast<const float4 *>(av + TI * r * VS + kg + q * SL + t);
                                a[r][0] = v.x; a[r][1] = v.y; a[r][2] = v.z; a[r][3] = v.w;
                            }
#pragma unroll
                            for (int c = 0; c < C; ++c) {
                                const float4 v = *reinterpret_cast<const float4 *>(bv + TJ * c * VS + kg + q * SL + t);
                                b[c][0] = v.x; b[c][1] = v.y; b[c][2] = v.z; b[c][3] = v.w;
                            }
#pragma unroll
                            for (int w = 0; w < 4; ++w)
#pragma unroll
                                for (int r = 0; r < R; ++r)
#pragma unroll
                                    for (int c = 0; c < C; ++c) S32[r][c] += (int32_t)((a[r][w] * b[c][w]) * scale[r][c]);
                        }
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int c = 0; c < C; ++c)
                                if ((have[r][c] >> q) & 1u) Tm[r][c] += __builtin_floor(ldexp((double)S32[r][c], (eq[r][c] - F) - (em[r][c] - hot.Fm)));
                    }
                    bool hv[R][C];
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) hv[r][c] = have[r][c] != 0;
                    finish_merged(std::integral_constant<int, GLT>{}, kg, Tm, hv, em, tg, tagged);
                }
                }
            };
            // Algorithm "GTR-FDPA": the even and the odd products of a group are aligned at their own maxima (which pass 1's
            // packed arithmetic keeps apart: even k in the low halves) and summed apart; then merged as above.
            auto run_even_odd = [&](auto gl_c) {
                constexpr int GL = decltype(gl_c)::value;
                constexpr int UE = (GL / 4 <= 2) ? 2 : 1;
                if constexpr (GL <= KC && !ADAPT && FAM == 3) {
#pragma unroll 1
                for (int g = 0; g < KC / GL; ++g) {
                    const uint32_t kg = g * GL;
                    int ee[R][C], eo[R][C];
                    uint32_t tg[R][C], tagged = 0;
                    bool he[R][C], ho[R][C];
                    float scale_e[R][C], scale_o[R][C];
                    int32_t Se[R][C], So[R][C];
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) {
                            uint32_t x = m2k[g * (GL / 4)][r * C + c][tid];
#pragma unroll
                            for (int i = 1; i < GL / 4; ++i) x = pk_max_u16(x, m2k[g * (GL / 4) + i][r * C + c][tid]);
                            const uint32_t lo = x & 0xFFFFu, hi = x >> 16;
                            tg[r][c] = x & SENTINEL_MASK;
                            tagged |= x;
                            ee[r][c] = (int)lo + ebase;
                            eo[r][c] = (int)hi + ebase;
                            he[r][c] = !(fl & FL_SKIP_ZERO) || lo >= 2 * ZBIAS;
                            ho[r][c] = !(fl & FL_SKIP_ZERO) || hi >= 2 * ZBIAS;
                            int se = F + 127 - ee[r][c], so = F + 127 - eo[r][c];
                            se = se < 1 ? 1 : (se > 254 ? 254 : se);                  // the clamps never change a truncated term
                            so = so < 1 ? 1 : (so > 254 ? 254 : so);
                            scale_e[r][c] = __uint_as_float((uint32_t)se << 23);
                            scale_o[r][c] = __uint_as_float((uint32_t)so << 23);
                            Se[r][c] = 0;
                            So[r][c] = 0;
                        }
                    tagged &= SENTINEL_MASK;
#pragma unroll UE
                    for (int t = 0; t < GL; t += 4) {
                        float a[R][4], b[C][4];
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            const float4 v = *reinterpret_cast<const float4 *>(av + TI * r * VS + kg + t);
                            a[r][0] = v.x; a[r][1] = v.y; a[r][2] = v.z; a[r][3] = v.w;
                        }
#pragma unroll
                        for (int c = 0; c < C; ++c) {
                            const float4 v = *reinterpret_cast<const float4 *>(bv + TJ * c * VS + kg + t);
                            b[c][0] = v.x; b[c][1] = v.y; b[c][2] = v.z; b[c][3] = v.w;
                        }
#pragma unroll
                        for (int w = 0; w < 4; ++w)
#pragma unroll
                            for (int r = 0; r < R; ++r)
#pragma unroll
                                for (int c = 0; c < C; ++c) {
                                    if (w & 1) So[r][c] += (int32_t)((a[r][w] * b[c][w]) * scale_o[r][c]);
                                    else Se[r][c] += (int32_t)((a[r][w] * b[c][w]) * scale_e[r][c]);
                                }
                    }
                    double T[R][C];
                    int em[R][C];
                    bool hv[R][C];
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int c = 0; c < C; ++c) {
                            const bool h0 = he[r][c], h1 = ho[r][c];
                            em[r][c] = (h0 && h1) ? (ee[r][c] > eo[r][c] ? ee[r][c] : eo[r][c]) : (h0 ? ee[r][c] : eo[r][c]);
                            T[r][c] = 0.0;
                            if (h0) T[r][c] += __builtin_floor(ldexp((double)Se[r][c], (ee[r][c] - F) - (em[r][c] - hot.Fm)));
                            if (h1) T[r][c] += __builtin_floor(ldexp((double)So[r][c], (eo[r][c] - F) - (em[r][c] - hot.Fm)));
                            hv[r][c] = h0 || h1;
                        }
                    finish_merged(gl_c, kg, T, hv, em, tg, tagged);
                }
                }
            };
            if constexpr (FAM == 3) {
                if (L == 4) run_even_odd(std::integral_constant<int, 4>{});
                else if (L == 8) run_even_odd(std::integral_constant<int, 8>{});
                else if (L == 16) run_even_odd(std::integral_constant<int, 16>{});
                else run_even_odd(std::integral_constant<int, 32>{});
            } else if constexpr (FAM == 2) {
                const uint32_t parts = hot.parts, SLr = L / parts;              // sub-groups of a group, terms of a sub-group
                if (parts == 2) {
                    if (SLr == 4) run_split(std::integral_constant<int, 4>{}, std::integral_constant<int, 2>{});
                    else if (SLr == 8) run_split(std::integral_constant<int, 8>{}, std::integral_constant<int, 2>{});
                    else run_split(std::integral_constant<int, 16>{}, std::integral_constant<int, 2>{});
                } else {
                    if (SLr == 4) run_split(std::integral_constant<int, 4>{}, std::integral_constant<int, 4>{});
                    else run_split(std::integral_constant<int, 8>{}, std::integral_constant<int, 4>{});
                }
            } else {
            if (L == 4) by_kind(std::integral_constant<int, 4>{});
            else if (L == 8) by_kind(std::integral_constant<int, 8>{});
            else if (L == 16) by_kind(std::integral_constant<int, 16>{});
            else by_kind(std::integral_constant<int, 32>{});                 // (no code where KC is below 32)
            }

            // ---- this model's outputs against the reference ----
            // Per output that differs: one LDS atomic on its histogram bucket (bucket 0 of the LDS copy counts pairs that
            // differ at distance 0: zeros of both signs, NaNs of two patterns), so the number of mismatches is the
            // histogram's sum; the largest distance and the first index are reduced over the wavefront with row shifts,
            // and lane 63 puts them into LDS.
            // (a pair of twins: the first model's outputs were set aside; then the twin's, in the next place of the arrays)
            constexpr int ACCOUNTS = TWIN ? 2 : 1;
#pragma unroll 1
            for (int acc = 0; acc < ACCOUNTS && (acc == 0 || twin); ++acc) {
            const bool set_aside = TWIN && twin && acc == 0;
            if (TWIN && acc == 1) ++mi;
            uint32_t maxd = 0;
            uint32_t first_off = 0xFFFFFFFFu;
            if (live) {
                uint32_t *dout = nullptr;
                uint64_t dump_off = 0;
                if (dumping) { dout = sa->dout; dump_off = (uint64_t)sa->slot[mi] * sa->out_stride; }       // (uniform)
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        uint32_t x = set_aside ? dfirst[TWIN ? r : 0][TWIN ? c : 0] : d[r][c];
                        if (slow_seen && (x & 0x7FFFFFFFu) > 0x7F800000u) x = set_aside ? nan_first : nan_bits;          // (the short route produces no NaN)
                        const uint64_t o = d_off + (uint64_t)(TI * r) * TN + TJ * c;
                        if (dumping) dout[dump_off + o] = x;
                        if (ref_first && mi == 0) ref[r][c] = x;
                        const uint32_t y = ref[r][c];
                        if (x != y) {
                            const uint32_t off = (uint32_t)((TI * r) * TN + TJ * c);
                            first_off = off < first_off ? off : first_off;
                            const uint32_t ax = x & 0x7FFFFFFFu, ay = y & 0x7FFFFFFFu;
                            const bool nx = ax > 0x7F800000u, ny = ay > 0x7F800000u;
                            uint32_t bucket;
                            if (nx || ny) {
                                bucket = (nx && ny) ? 0u : 33u;
                                if (nx && ny) atomicAdd(&ml.naneq[mi], 1u);                      // (rare)
                            } else {
                                // distance of the ordered keys (sign-magnitude patterns read as signed integers): below 2^32
                                const int32_t sx = (int32_t)x >> 31, sy = (int32_t)y >> 31;                    // 0 or -1
                                const int32_t kx = ((int32_t)ax ^ sx) - sx, ky = ((int32_t)ay ^ sy) - sy;       // -|x| for a negative x
                                const uint32_t dist = kx >= ky ? (uint32_t)kx - (uint32_t)ky : (uint32_t)ky - (uint32_t)kx;
                                maxd = dist > maxd ? dist : maxd;
                                bucket = 32u - (uint32_t)__clz((int)dist);                                      // (__clz(0) = 32)
                            }
                            atomicAdd(&ml.hist[mi][bucket][tid & (HC - 1)], 1u);
                        }
                    }
            }
            // (offsets relative to the first output of this pass of the workgroup: 32 bits do for the reduction)
            const uint32_t rel = first_off == 0xFFFFFFFFu ? 0xFFFFFFFFu : (uint32_t)(d_off - item0 * (uint64_t)(TM * TN)) + first_off;
            const uint32_t wmin = wave_reduce_to_lane63<false>(rel), wmax = wave_reduce_to_lane63<true>(maxd);
            if ((tid & 63u) == 63u && wmin != 0xFFFFFFFFu) {
                atomicMin(&ml.first[mi], (unsigned long long)(sa->index_base + item0 * (uint64_t)(TM * TN) + wmin));
                if (wmax) atomicMax(&ml.maxd[mi], wmax);
            }
            }
        }
        set_f32_round_toward_zero(false);
    }
    __syncthreads();
    // one global atomic per non-zero counter per workgroup; n_compared and bucket 0 are known up front: workgroup 0 adds
    // the whole count once, every workgroup takes its non-zero buckets back out of bucket 0
    unsigned long long *gst = reinterpret_cast<unsigned long long *>(sa->stats);
    for (uint32_t i = tid; i < count * 34u; i += 256) {
        const uint32_t mi = i / 34u, b = i - mi * 34u;
        unsigned long long *g = gst + (uint64_t)sa->slot[mi] * STATS_WORDS;
        if (b == 0) {
            uint32_t nonzero = 0, mism = 0;
            for (int bb = 1; bb < 34; ++bb)
                for (int cpy = 0; cpy < HC; ++cpy) nonzero += ml.hist[mi][bb][cpy];
            for (int cpy = 0; cpy < HC; ++cpy) mism += ml.hist[mi][0][cpy];         // differing patterns at distance 0
            mism += nonzero;
            const unsigned long long total = (unsigned long long)nitems * (TM * TN);
            if (blockIdx.x == 0) { atomicAdd(&g[0], total); atomicAdd(&g[5], total); }
            if (nonzero) atomicAdd(&g[5], 0ull - (unsigned long long)nonzero);
            if (mism) {
                atomicAdd(&g[1], (unsigned long long)mism);
                atomicMin(&g[3], ml.first[mi]);
            }
            if (ml.naneq[mi]) atomicAdd(&g[2], (unsigned long long)ml.naneq[mi]);
            if (ml.maxd[mi]) atomicMax(&g[4], (unsigned long long)ml.maxd[mi]);
        } else {
            uint32_t t = 0;
            for (int cpy = 0; cpy < HC; ++cpy) t += ml.hist[mi][b][cpy];
            if (t) atomicAdd(&g[5 + b], (unsigned long long)t);
        }
    }
}

template <int TM, int KC, bool ADAPT, int FAM, bool TWIN = false>
static mmaemu_status launch_scan_cfg(const ScanArgs &sa, const void *A, const void *B, const uint32_t *C, uint64_t batch, hipStream_t s)
{
    constexpr int SLOTS = 256 / ((TM / 2) * (TM / 2));
    const uint64_t blocks = (batch + SLOTS - 1) / SLOTS;
    if (blocks > 0x7FFFFFFFull) { set_error("emulate_compare_many: too many blocks"); return MMAEMU_ERR_SHAPE; }
    if (blocks == 0) return MMAEMU_OK;
    // Persistent workgroups: every workgroup ends with a few dozen global atomics on the same few cache lines.  Long
    // launches take 2048 workgroups (the dispatcher balances a grid beyond the resident set); short ones as many as the
    // device holds at once, and of those just enough that all make the same number of passes.
    uint32_t grid = 2048u;
    if (blocks < 8u * 2048u) {
        static uint32_t resident[16] = {};
        int dev = 0;
        MMAEMU_HIP(hipGetDevice(&dev));
        uint32_t &res = resident[dev & 15];
        if (!res) {
            int per_cu = 0, cus = 0;
            MMAEMU_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, emulate_scan_kernel<TM, KC, ADAPT, FAM, TWIN>, 256, 0));
            MMAEMU_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
            res = (uint32_t)(per_cu > 0 ? per_cu : 1) * (uint32_t)(cus > 0 ? cus : 1);
        }
        const uint64_t passes = (blocks + res - 1) / res;
        grid = (uint32_t)((blocks + passes - 1) / passes);
    }
    hipLaunchKernelGGL((emulate_scan_kernel<TM, KC, ADAPT, FAM, TWIN>), dim3(grid), dim3(256), 0, s, sa, A, B, C, batch, (uint32_t)blocks);
    MMAEMU_HIP(hipGetLastError());
    set_last_kernel("multi x%u tiled %dx%d r2x2 kc=%d any L vm=%d%s", sa.count, TM, TM, KC, ADAPT ? 1 : 0, FAM == 1 ? " rd" : (FAM == 2 ? " rd split" : (FAM == 3 ? " rd even/odd" : (TWIN ? ", twins share sums" : ""))));
    return MMAEMU_OK;
}

// Whether the kernel takes a model, the model's arithmetic kind, and the class of models it can share a launch with:
// 0, T-FDPA with the accumulator inside the sum; 1, TR-FDPA (unsplit groups, any of the variation switches); 2 and 3,
// TR-FDPA sets that keep zero terms out of the exponent maxima (the staged exponents then differ), without and with
// FlushSubnormal on the inputs (which decides what a zero is); 4 to 6, the same three for groups split in halves or
// quarters; 7 to 9, for the even / odd split.  Whole 16x16x16, 16x16x32, 32x32x8 or 32x32x16 tiles of
// FP8 / FP16 / BF16 / FP6 / FP4 operands, group length 4, 8, 16 or 32, F up to 40.
bool scan_takes(const ModelArgs &p, uint32_t ta, uint32_t tb, uint32_t m, uint32_t n, uint32_t k, const void *A, const void *B, uint32_t &kind,
                uint32_t &cls)
{
    const bool bf16 = ta == MMAEMU_BF16 || tb == MMAEMU_BF16;
    if (p.flags & (FL_ACC16 | FL_NAN_PROPAGATE)) return false;
    if (p.c_mode == MMAEMU_C_IN_GROUP) {
        if (p.skip_zero_terms || p.zero_result_positive) return false;
        cls = 0;
    } else if (p.c_mode == MMAEMU_C_AFTER_RD && p.split == MMAEMU_SPLIT_NONE) {
        // (BF16 products of 2^128 and more that keep their values need the general kernel's integer range; the truncating
        // variant of the round-downs exists for the plain F2 rule)
        if ((p.wide_products && bf16) || (p.rd_toward_zero && p.f2_at_leading_bit)) return false;
        cls = p.skip_zero_terms ? (p.ftz_in ? 3u : 2u) : 1u;
    } else if (p.c_mode == MMAEMU_C_AFTER_RD && (p.split == MMAEMU_SPLIT_HALVES || p.split == MMAEMU_SPLIT_QUARTERS)) {
        // halves or quarters of at least four terms, each summed in 32 bits, from binary32 values
        const uint32_t parts = p.split == MMAEMU_SPLIT_HALVES ? 2u : 4u;
        if (bf16 || p.rd_toward_zero || p.F >= 30 || p.L < 4 * parts || ((uint64_t)(p.L / parts) << (p.F + 2)) > (1ull << 31)) return false;
        cls = 4u + (p.skip_zero_terms ? (p.ftz_in ? 2u : 1u) : 0u);
    } else if (p.c_mode == MMAEMU_C_AFTER_RD && p.split == MMAEMU_SPLIT_EVEN_ODD) {
        // the even and the odd products of a group (Algorithm "GTR-FDPA"), each summed in 32 bits, from binary32 values
        if (bf16 || p.rd_toward_zero || p.F >= 30 || ((uint64_t)(p.L / 2) << (p.F + 2)) > (1ull << 31)) return false;
        cls = 7u + (p.skip_zero_terms ? (p.ftz_in ? 2u : 1u) : 0u);
    } else {
        return false;
    }
    if (!((m == 16 && n == 16 && (k == 16 || k == 32)) || (m == 32 && n == 32 && (k == 8 || k == 16)))) return false;
    if (ta == MMAEMU_FP32 || tb == MMAEMU_FP32 || ta == MMAEMU_TF32 || tb == MMAEMU_TF32) return false;
    if ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 7) return false;
    if (p.F > 40) return false;
    if (!(p.L == 4 || p.L == 8 || p.L == 16 || p.L == 32) || p.L > k) return false;
    const uint64_t term = 1ull << (p.F + 2);                // |aligned term| < 2^(F+2)
    kind = p.F >= 30 ? 3u : ((uint64_t)p.L * term <= (1ull << 31) ? 0u : (4 * term <= (1ull << 31) ? 1u : 2u));
    return true;
}

// tiles of one group whose launch holds twins (models that differ only in the output conversion)
static mmaemu_status launch_scan_twins(const ScanArgs &sa, const void *A, const void *B, const uint32_t *Cm, uint32_t m, uint32_t n, uint32_t k,
                                       uint64_t batch, bool adapt, hipStream_t s)
{
    if (m == 16 && n == 16 && k == 16) return adapt ? launch_scan_cfg<16, 16, true, 0, true>(sa, A, B, Cm, batch, s) : launch_scan_cfg<16, 16, false, 0, true>(sa, A, B, Cm, batch, s);
    if (m == 32 && n == 32 && k == 8) return adapt ? launch_scan_cfg<32, 8, true, 0, true>(sa, A, B, Cm, batch, s) : launch_scan_cfg<32, 8, false, 0, true>(sa, A, B, Cm, batch, s);
    if (m == 16 && n == 16 && k == 32) return adapt ? launch_scan_cfg<16, 32, true, 0, true>(sa, A, B, Cm, batch, s) : launch_scan_cfg<16, 32, false, 0, true>(sa, A, B, Cm, batch, s);
    if (m == 32 && n == 32 && k == 16) return adapt ? launch_scan_cfg<32, 16, true, 0, true>(sa, A, B, Cm, batch, s) : launch_scan_cfg<32, 16, false, 0, true>(sa, A, B, Cm, batch, s);
    set_error("emulate_compare_many: no kernel for this shape");
    return MMAEMU_ERR_UNSUPPORTED;
}

template <int FAM>
static mmaemu_status launch_scan_shape(const ScanArgs &sa, const void *A, const void *B, const uint32_t *Cm, uint32_t m, uint32_t n, uint32_t k,
                                       uint64_t batch, bool adapt, hipStream_t s)
{
    if constexpr (FAM >= 2) {                    // (binary32 values only)
        if (m == 16 && n == 16 && k == 16) return launch_scan_cfg<16, 16, false, FAM>(sa, A, B, Cm, batch, s);
        if (m == 32 && n == 32 && k == 8) return launch_scan_cfg<32, 8, false, FAM>(sa, A, B, Cm, batch, s);
        if (m == 16 && n == 16 && k == 32) return launch_scan_cfg<16, 32, false, FAM>(sa, A, B, Cm, batch, s);
        if (m == 32 && n == 32 && k == 16) return launch_scan_cfg<32, 16, false, FAM>(sa, A, B, Cm, batch, s);
    } else {
    if (m == 16 && n == 16 && k == 16) return adapt ? launch_scan_cfg<16, 16, true, FAM>(sa, A, B, Cm, batch, s) : launch_scan_cfg<16, 16, false, FAM>(sa, A, B, Cm, batch, s);
    if (m == 32 && n == 32 && k == 8) return adapt ? launch_scan_cfg<32, 8, true, FAM>(sa, A, B, Cm, batch, s) : launch_scan_cfg<32, 8, false, FAM>(sa, A, B, Cm, batch, s);
    if (m == 16 && n == 16 && k == 32) return adapt ? launch_scan_cfg<16, 32, true, FAM>(sa, A, B, Cm, batch, s) : launch_scan_cfg<16, 32, false, FAM>(sa, A, B, Cm, batch, s);
    if (m == 32 && n == 32 && k == 16) return adapt ? launch_scan_cfg<32, 16, true, FAM>(sa, A, B, Cm, batch, s) : launch_scan_cfg<32, 16, false, FAM>(sa, A, B, Cm, batch, s);
    }
    set_error("emulate_compare_many: no kernel for this shape");
    return MMAEMU_ERR_UNSUPPORTED;
}

mmaemu_status launch_scan(const MultiLaunch &ml, const void *A, const void *B, const void *C, uint32_t m, uint32_t n, uint32_t k,
                          uint64_t batch, uint32_t ta, uint32_t tb, hipStream_t s)
{
    ScanArgs sa = {};
    sa.ta = ta;
    sa.tb = tb;
    sa.zbias = (ml.cls >= 1 && (ml.cls - 1) % 3 != 0) ? ZBIAS : 0u;
    sa.ebase = 2 - fmt_info(ta).bias - fmt_info(tb).bias - 2 * (int)sa.zbias;
    sa.count = ml.count;
    sa.ref_is_first = ml.ref_is_first ? 1u : 0u;
    sa.dref = ml.dref;
    sa.dout = ml.dout;
    sa.out_stride = ml.out_stride;
    sa.index_base = ml.index_base;
    sa.stats = reinterpret_cast<uint64_t *>(ml.stats);
    // Order within the launch.  T-FDPA models on tiles of one group (L = k) that differ only in the output conversion
    // (rounding, E8M13, output flush, NaN pattern) are twins: the second is moved next to the first (never across the
    // line between sets that flush their inputs and sets that do not: twins agree on that), and the kernel computes
    // their common maximum and sum once.
    uint32_t order[MULTI_MAX], n_order = 0;
    bool placed[MULTI_MAX] = {}, twin_of_next[MULTI_MAX] = {};
    bool any_twin = false;
    const uint32_t conversion_only = FL_RZ | FL_FTZ_OUT;
    for (uint32_t i = 0; i < ml.count; ++i) {
        if (placed[i]) continue;
        placed[i] = true;
        order[n_order++] = i;
        const ModelArgs &p = ml.models[i];
        if (ml.cls != 0 || p.L != k) continue;
        for (uint32_t j = i + 1; j < ml.count; ++j) {
            const ModelArgs &q = ml.models[j];
            if (placed[j] || q.L != p.L || q.F != p.F || ml.kind[j] != ml.kind[i] || ((q.flags ^ p.flags) & ~conversion_only) != 0) continue;
            placed[j] = true;
            twin_of_next[n_order - 1] = true;
            order[n_order++] = j;
            any_twin = true;
            break;
        }
    }
    for (uint32_t q = 0; q < ml.count; ++q) {
        const uint32_t i = order[q];
        const ModelArgs &p = ml.models[i];
        sa.slot[q] = ml.slot[i];
        sa.hot[q] = ScanArgs::Hot{p.F, p.flags, p.out_mask, p.nan_bits, p.L, ml.kind[i], p.F2, p.Fc, p.sum_drop_distance, p.Fm,
                                  p.split == MMAEMU_SPLIT_QUARTERS ? 4u : 2u, twin_of_next[q] ? 1u : 0u};
    }
    const bool adapt = ta == MMAEMU_BF16 || tb == MMAEMU_BF16;
    const uint32_t *Cm = static_cast<const uint32_t *>(C);
    if (ml.cls == 0 && any_twin) return launch_scan_twins(sa, A, B, Cm, m, n, k, batch, adapt, s);
    if (ml.cls == 0) return launch_scan_shape<0>(sa, A, B, Cm, m, n, k, batch, adapt, s);
    if (ml.cls <= 3) return launch_scan_shape<1>(sa, A, B, Cm, m, n, k, batch, adapt, s);
    if (ml.cls <= 6) return launch_scan_shape<2>(sa, A, B, Cm, m, n, k, batch, false, s);
    return launch_scan_shape<3>(sa, A, B, Cm, m, n, k, batch, false, s);
}

} // namespace mmaemu
