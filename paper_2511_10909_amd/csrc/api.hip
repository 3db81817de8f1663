// C-ABI entry points of libmmaemu: argument validation, error reporting, dispatch.
// All validation happens here, on the host, before any kernel is enqueued.
#include "common.hpp"

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

struct mmaemu_model {
    uint32_t magic;
    mmaemu_model_params params;
};

namespace mmaemu {

static constexpr uint32_t MODEL_MAGIC = 0x4D4D4145u;   // "MMAE"
static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

static thread_local char g_kernel[128] = "";

void set_last_kernel(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_kernel, sizeof(g_kernel), fmt, ap);
    va_end(ap);
}

mmaemu_status hip_fail(hipError_t e, const char *what)
{
    set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
    return MMAEMU_ERR_HIP;
}

static bool is_ab_type(uint32_t t) { return t <= MMAEMU_FP32 || is_narrow_type(t) || t == MMAEMU_TF32; }
static bool is_word_type(uint32_t t) { return t == MMAEMU_TF32 || t == MMAEMU_FP32; }      // operands held in 32-bit words

static uint32_t ceil_log2(uint32_t x)
{
    uint32_t l = 0;
    while ((1ull << l) < x) ++l;
    return l;
}

} // namespace mmaemu

using namespace mmaemu;

extern "C" {

const char *mmaemu_status_string(mmaemu_status s)
{
    switch (s) {
    case MMAEMU_OK: return "ok";
    case MMAEMU_ERR_INVALID_ARG: return "invalid argument";
    case MMAEMU_ERR_UNSUPPORTED: return "unsupported";
    case MMAEMU_ERR_SHAPE: return "bad shape";
    case MMAEMU_ERR_HIP: return "HIP runtime error";
    case MMAEMU_ERR_NOMEM: return "out of memory";
    }
    return "unknown status";
}

const char *mmaemu_last_error(void) { return g_err; }

const char *mmaemu_last_kernel(void) { return g_kernel; }

uint32_t mmaemu_version(void) { return 100; }

mmaemu_status mmaemu_model_create(const mmaemu_model_params *p, mmaemu_model **out)
{
    if (!p || !out) { set_error("model_create: NULL argument"); return MMAEMU_ERR_INVALID_ARG; }
    *out = nullptr;
    if (p->struct_size != sizeof(mmaemu_model_params)) {
        set_error("model_create: struct_size %u, expected %zu", p->struct_size, sizeof(mmaemu_model_params));
        return MMAEMU_ERR_INVALID_ARG;
    }
    if (p->c_mode > MMAEMU_C_EXACT || p->out_round > MMAEMU_ROUND_RZ || p->ftz_in > 1 || p->ftz_out > 1) {
        set_error("model_create: enum field out of range");
        return MMAEMU_ERR_INVALID_ARG;
    }
    if (p->family > MMAEMU_FAMILY_FMA) { set_error("model_create: family out of range"); return MMAEMU_ERR_INVALID_ARG; }
    if (p->nan_propagate > 1) { set_error("model_create: nan_propagate must be 0 or 1"); return MMAEMU_ERR_INVALID_ARG; }
    if (p->nan_propagate && p->family != MMAEMU_FAMILY_FDPA && p->family != MMAEMU_FAMILY_FMA) {
        set_error("model_create: nan_propagate belongs to the FDPA and FMA families");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (p->family != MMAEMU_FAMILY_GST_FDPA && (p->gst_group || p->scale_format)) {
        set_error("model_create: gst_group and scale_format belong to the GST-FDPA family");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (p->family == MMAEMU_FAMILY_GST_FDPA) {
        if (p->scale_format > MMAEMU_SCALE_FORMAT_UE4M3) { set_error("model_create: scale_format out of range"); return MMAEMU_ERR_INVALID_ARG; }
        if (p->gst_group == 0 || p->gst_group > 64 || (p->group_len && (p->group_len % p->gst_group || p->group_len / p->gst_group > 64))) {
            set_error("model_create: GST-FDPA needs 1 <= gst_group <= 64 dividing group_len, at most 64 groups per operation");
            return MMAEMU_ERR_UNSUPPORTED;
        }
        if (p->c_mode || p->frac_bits2 || p->out_mant_bits != 23 || p->ftz_in || p->ftz_out || p->split || p->acc_special_truncation ||
            p->frac_bits_merge || p->frac_bits_acc || p->f2_at_leading_bit || p->skip_zero_terms || p->zero_result_positive ||
            p->sum_drop_distance || p->wide_products) {
            set_error("model_create: the GST-FDPA family takes group_len, gst_group, frac_bits, out_round, nan_bits and scale_format only");
            return MMAEMU_ERR_UNSUPPORTED;
        }
    }
    if (p->family == MMAEMU_FAMILY_FTZ_ADDMUL) {
        if (p->group_len != 2 && p->group_len != 4) {
            set_error("model_create: the FTZ-AddMul family needs group_len (P) = 2 or 4");
            return MMAEMU_ERR_UNSUPPORTED;
        }
        if (p->align_round || p->c_mode || p->frac_bits2 || p->out_round || p->out_mant_bits != 23 || p->ftz_in || p->ftz_out ||
            p->split || p->acc_special_truncation || p->frac_bits_merge || p->frac_bits_acc || p->f2_at_leading_bit ||
            p->skip_zero_terms || p->zero_result_positive || p->sum_drop_distance || p->wide_products) {
            set_error("model_create: the FTZ-AddMul family takes group_len and nan_bits only");
            return MMAEMU_ERR_UNSUPPORTED;
        }
    }
    if (p->family == MMAEMU_FAMILY_FMA) {
        if (p->group_len > 1 || p->align_round || p->c_mode || p->frac_bits2 || p->out_round || p->out_mant_bits != 23 || p->ftz_in ||
            p->ftz_out || p->split || p->acc_special_truncation || p->frac_bits_merge || p->frac_bits_acc || p->f2_at_leading_bit ||
            p->skip_zero_terms || p->zero_result_positive || p->sum_drop_distance || p->wide_products) {
            set_error("model_create: the FMA family takes nan_bits and nan_propagate only (group_len 0 or 1)");
            return MMAEMU_ERR_UNSUPPORTED;
        }
    }
    if (p->align_round != MMAEMU_ALIGN_RZ) { set_error("model_create: only RZ alignment is supported"); return MMAEMU_ERR_UNSUPPORTED; }
    if (p->out_mant_bits != 23 && !(p->out_mant_bits == 13 && p->out_round == MMAEMU_ROUND_RZ)) {
        set_error("model_create: out_mant_bits must be 23 (FP32), or 13 with out_round = RZ (RZ-E8M13)");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    const bool rd_mode = p->c_mode == MMAEMU_C_AFTER_RD || p->c_mode == MMAEMU_C_AFTER_RD_EVEN_ODD;
    if (!rd_mode && p->frac_bits2 != 0) {
        set_error("model_create: frac_bits2 is used by the C_AFTER_RD modes only and must be 0 otherwise");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (rd_mode && (p->frac_bits2 > 48 || p->frac_bits_merge > 48 || p->frac_bits_acc > 48)) {
        set_error("model_create: frac_bits2 / frac_bits_merge / frac_bits_acc above 48");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (p->rd_toward_zero > 1 || (p->rd_toward_zero && (!rd_mode || p->family != MMAEMU_FAMILY_FDPA))) {
        set_error("model_create: rd_toward_zero (0 / 1) belongs to the C_AFTER_RD modes of the FDPA family");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (p->split > MMAEMU_SPLIT_QUARTERS || p->acc_special_truncation > 1 || p->f2_at_leading_bit > 1 ||
        p->skip_zero_terms > 1 || p->zero_result_positive > 1 || p->wide_products > 1) {
        set_error("model_create: enum field out of range");
        return MMAEMU_ERR_INVALID_ARG;
    }
    if (p->c_mode != MMAEMU_C_AFTER_RD &&
        (p->split || p->acc_special_truncation || p->frac_bits_merge || p->frac_bits_acc || p->f2_at_leading_bit ||
         p->sum_drop_distance || p->wide_products)) {
        set_error("model_create: split, acc_special_truncation, frac_bits_merge, frac_bits_acc, f2_at_leading_bit, "
                  "sum_drop_distance and wide_products belong to c_mode C_AFTER_RD");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (p->frac_bits_merge && p->split == MMAEMU_SPLIT_NONE) {
        set_error("model_create: frac_bits_merge needs a split");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (p->frac_bits > (rd_mode ? 40u : 48u)) {
        set_error("model_create: frac_bits %u > %u", p->frac_bits, rd_mode ? 40u : 48u);
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (p->group_len > (1u << 20)) { set_error("model_create: group_len %u > 2^20", p->group_len); return MMAEMU_ERR_UNSUPPORTED; }
    mmaemu_model *m = new (std::nothrow) mmaemu_model;
    if (!m) { set_error("model_create: allocation failed"); return MMAEMU_ERR_NOMEM; }
    m->magic = MODEL_MAGIC;
    m->params = *p;
    *out = m;
    return MMAEMU_OK;
}

mmaemu_status mmaemu_model_destroy(mmaemu_model *m)
{
    if (!m) return MMAEMU_OK;
    if (m->magic != MODEL_MAGIC) { set_error("model_destroy: not a model handle"); return MMAEMU_ERR_INVALID_ARG; }
    m->magic = 0;
    delete m;
    return MMAEMU_OK;
}

mmaemu_status mmaemu_model_get_params(const mmaemu_model *m, mmaemu_model_params *out)
{
    if (!m || !out || m->magic != MODEL_MAGIC) { set_error("model_get_params: bad argument"); return MMAEMU_ERR_INVALID_ARG; }
    *out = m->params;
    return MMAEMU_OK;
}

// The FDPA family's parameters as the kernels take them, for a problem with k products per output (checks that depend
// on k and on the accumulator's type included).
static mmaemu_status fdpa_model_args(const mmaemu_model_params &mp, uint32_t k, bool acc16, ModelArgs &ma)
{
    const uint32_t L = (mp.group_len == 0 || mp.group_len > k) ? k : mp.group_len;
    if (k % L) { set_error("emulate_mma: k=%u is not a multiple of the group length L=%u", k, L); return MMAEMU_ERR_SHAPE; }
    if (mp.c_mode == MMAEMU_C_IN_GROUP && mp.frac_bits + 3 + ceil_log2(L) > 63) {      // the fused sum is a 64-bit integer
        set_error("emulate_mma: C_IN_GROUP needs frac_bits + 3 + ceil(log2 L) <= 63");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (mp.c_mode == MMAEMU_C_AFTER_EXACT && mp.frac_bits + 2 + ceil_log2(L) > 56) {
        set_error("emulate_mma: C_AFTER_EXACT needs frac_bits + 2 + ceil(log2 L) <= 56");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    const bool rd_mode = mp.c_mode == MMAEMU_C_AFTER_RD || mp.c_mode == MMAEMU_C_AFTER_RD_EVEN_ODD;
    const uint32_t split = mp.c_mode == MMAEMU_C_AFTER_RD_EVEN_ODD ? (uint32_t)MMAEMU_SPLIT_EVEN_ODD : mp.split;
    if (rd_mode) {
        uint32_t fmax = mp.frac_bits > mp.frac_bits2 ? mp.frac_bits : mp.frac_bits2;
        if (mp.frac_bits_merge > fmax) fmax = mp.frac_bits_merge;
        if (mp.frac_bits_acc > fmax) fmax = mp.frac_bits_acc;
        if (fmax + 3 + ceil_log2(L) > 53) {
            set_error("emulate_mma: the C_AFTER_RD modes need max(F, F2, F_m, F_c) + 3 + ceil(log2 L) <= 53");
            return MMAEMU_ERR_UNSUPPORTED;
        }
        if ((split != MMAEMU_SPLIT_NONE && (L & 1u)) || (split == MMAEMU_SPLIT_QUARTERS && (L & 3u))) {
            set_error("emulate_mma: a split group needs an even group length, quarters a multiple of 4 (L=%u)", L);
            return MMAEMU_ERR_SHAPE;
        }
    }
    ma.L = L;
    ma.F = (int32_t)mp.frac_bits;
    ma.F2 = (int32_t)mp.frac_bits2;
    ma.c_mode = rd_mode ? (uint32_t)MMAEMU_C_AFTER_RD : mp.c_mode;
    ma.split = split;
    ma.acc_special_truncation = mp.c_mode == MMAEMU_C_AFTER_RD_EVEN_ODD ? 1u : mp.acc_special_truncation;
    ma.Fm = (int32_t)(mp.frac_bits_merge ? mp.frac_bits_merge : mp.frac_bits);
    ma.Fc = (int32_t)(mp.frac_bits_acc ? mp.frac_bits_acc : mp.frac_bits);
    ma.f2_at_leading_bit = mp.f2_at_leading_bit;
    ma.skip_zero_terms = mp.skip_zero_terms;
    ma.zero_result_positive = mp.zero_result_positive;
    ma.wide_products = mp.wide_products;
    ma.sum_drop_distance = (int32_t)(mp.sum_drop_distance > 100000u ? 100000u : mp.sum_drop_distance);
    ma.rd_toward_zero = mp.rd_toward_zero;
    ma.out_round = mp.out_round;
    ma.out_mask = mp.out_mant_bits == 13 ? 0xFFFFFC00u : 0xFFFFFFFFu;
    ma.ftz_in = mp.ftz_in;
    ma.ftz_out = mp.ftz_out;
    ma.nan_bits = mp.nan_bits;
    ma.nan16 = mp.nan_bits & 0xFFFFu;
    if (acc16) ma.nan_bits = 0x7FC00000u;             // inside the kernels the accumulator is a binary32 pattern
    ma.flags = (acc16 ? FL_ACC16 : 0u) | (ma.out_round == MMAEMU_ROUND_RZ ? FL_RZ : 0u) | (ma.ftz_out ? FL_FTZ_OUT : 0u) | (ma.zero_result_positive ? FL_ZERO_POSITIVE : 0u) |
               (ma.ftz_in ? FL_FTZ_IN : 0u) | (ma.acc_special_truncation ? FL_SPECIAL_TRUNC : 0u) | (ma.f2_at_leading_bit ? FL_F2_LEADING : 0u) |
               (ma.skip_zero_terms ? FL_SKIP_ZERO : 0u) | (ma.wide_products ? FL_WIDE_PRODUCTS : 0u) | (mp.nan_propagate ? FL_NAN_PROPAGATE : 0u) |
               (mp.rd_toward_zero ? FL_RD_AS_RZ : 0u);
    return MMAEMU_OK;
}

static mmaemu_status emulate_impl(const mmaemu_model *model, const void *A, const void *B, const void *C, void *D,
                                  const uint8_t *SA, const uint8_t *SB, uint32_t block,
                                  uint32_t m, uint32_t n, uint32_t k, uint64_t batch, mmaemu_dtypes dt,
                                  void *hip_stream)
{
    if (!model || model->magic != MODEL_MAGIC) { set_error("emulate_mma: bad model handle"); return MMAEMU_ERR_INVALID_ARG; }
    if (m == 0 || n == 0 || k == 0) { set_error("emulate_mma: zero dimension (m=%u n=%u k=%u)", m, n, k); return MMAEMU_ERR_SHAPE; }
    if (k > (1u << 20)) { set_error("emulate_mma: k=%u > 2^20", k); return MMAEMU_ERR_SHAPE; }
    if (dt.a == MMAEMU_FP64 || dt.b == MMAEMU_FP64 || dt.c == MMAEMU_FP64 || dt.d == MMAEMU_FP64) {
        // binary64 is the other format Algorithms "FMA" / "Phi_FMA" name: that family only, all four arrays binary64
        const mmaemu_model_params &mq = model->params;
        if (mq.family != MMAEMU_FAMILY_FMA || dt.a != MMAEMU_FP64 || dt.b != MMAEMU_FP64 || dt.c != MMAEMU_FP64 || dt.d != MMAEMU_FP64 || SA) {
            set_error("emulate_mma: FP64 arrays go with the FMA family, all four of them FP64, unscaled");
            return MMAEMU_ERR_UNSUPPORTED;
        }
        const uint64_t mn_ = (uint64_t)m * n;
        if (batch && (mn_ > (1ull << 40) || batch > (1ull << 62) / mn_ || batch * mn_ > (1ull << 48))) { set_error("emulate_mma: problem too large"); return MMAEMU_ERR_SHAPE; }
        if (batch == 0) return MMAEMU_OK;
        if (!A || !B || !C || !D) { set_error("emulate_mma: NULL device pointer"); return MMAEMU_ERR_INVALID_ARG; }
        if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C | (uintptr_t)D) & 7) { set_error("emulate_mma: pointers must be aligned to their element size"); return MMAEMU_ERR_INVALID_ARG; }
        return launch_emulate_fma64(A, B, C, D, m, n, k, batch, mq.nan_bits, mq.nan_propagate != 0, (hipStream_t)hip_stream);
    }
    if (dt.a > MMAEMU_TF32 || dt.b > MMAEMU_TF32 || dt.c > MMAEMU_FP32 || dt.d > MMAEMU_FP32) {
        set_error("emulate_mma: dtype out of range");
        return MMAEMU_ERR_INVALID_ARG;
    }
    const bool acc16 = dt.c == MMAEMU_FP16 && dt.d == MMAEMU_FP16;
    if (!is_ab_type(dt.a) || !is_ab_type(dt.b) || !((dt.c == MMAEMU_FP32 && dt.d == MMAEMU_FP32) || acc16)) {
        set_error("emulate_mma: supported types are a, b in {E4M3, E5M2, FP16, BF16, FP32, E2M3, E3M2, E2M1, TF32} and c = d = FP32 or c = d = FP16");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if ((is_word_type(dt.a) || is_word_type(dt.b)) && dt.a != dt.b) {
        set_error("emulate_mma: TF32 operands pair with TF32 operands only, FP32 with FP32");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if ((is_narrow_type(dt.a) && !is_byte_type(dt.b)) || (is_narrow_type(dt.b) && !is_byte_type(dt.a))) {
        set_error("emulate_mma: FP6 / FP4 operands pair with FP6, FP4 and FP8 operands only");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    const mmaemu_model_params &mp = model->params;
    if (mp.nan_propagate && !(dt.a == MMAEMU_FP32 && dt.b == MMAEMU_FP32 && dt.c == MMAEMU_FP32)) {
        set_error("emulate_mma: nan_propagate is defined for FP32 operands and accumulators");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (acc16 && (mp.family != MMAEMU_FAMILY_FDPA || mp.c_mode > MMAEMU_C_AFTER_EXACT || mp.out_mant_bits != 23)) {
        set_error("emulate_mma: FP16 accumulators go with c_mode C_IN_GROUP or C_AFTER_EXACT and the plain conversion");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    const uintptr_t ab_mask = (uintptr_t)(fmt_info(dt.a).width / 8 - 1) | (uintptr_t)(fmt_info(dt.b).width / 8 - 1);
    if ((((uintptr_t)A | (uintptr_t)B) & ab_mask) || (((uintptr_t)C | (uintptr_t)D) & (acc16 ? 1u : 3u))) {
        set_error("emulate_mma: pointers must be aligned to their element size");
        return MMAEMU_ERR_INVALID_ARG;
    }
    if (mp.family == MMAEMU_FAMILY_FDPA && mp.c_mode == MMAEMU_C_EXACT && (SA || acc16)) {
        set_error("emulate_mma: C_EXACT (E-FDPA) takes unscaled operands and FP32 accumulators");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (SA && mp.family == MMAEMU_FAMILY_FTZ_ADDMUL) { set_error("emulate_mma_scaled: block scales belong to the FDPA families"); return MMAEMU_ERR_UNSUPPORTED; }
    if (mp.family == MMAEMU_FAMILY_GST_FDPA) {
        if (batch == 0) return MMAEMU_OK;
        if (!SA) { set_error("emulate_mma: the GST-FDPA family needs scale factors (mmaemu_emulate_mma_scaled)"); return MMAEMU_ERR_UNSUPPORTED; }
        if (dt.a != MMAEMU_FP4_E2M1 || dt.b != MMAEMU_FP4_E2M1 || acc16) { set_error("emulate_mma: GST-FDPA takes FP4 operands and FP32 accumulators"); return MMAEMU_ERR_UNSUPPORTED; }
        const uint32_t Lg = (mp.group_len == 0 || mp.group_len > k) ? k : mp.group_len;
        if (k % Lg || Lg % block || block % mp.gst_group || Lg / mp.gst_group > 64) {
            set_error("emulate_mma: GST-FDPA needs k %% L = 0, L %% block = 0, block %% G = 0 and L / G <= 64 (k=%u L=%u block=%u G=%u)", k, Lg, block, mp.gst_group);
            return MMAEMU_ERR_SHAPE;
        }
        const uint64_t mn_ = (uint64_t)m * n;
        if (batch && (mn_ > (1ull << 40) || batch > (1ull << 62) / mn_ || batch * mn_ > (1ull << 48))) { set_error("emulate_mma: problem too large"); return MMAEMU_ERR_SHAPE; }
        if (batch == 0) return MMAEMU_OK;
        if (!A || !B || !C || !D) { set_error("emulate_mma: NULL device pointer"); return MMAEMU_ERR_INVALID_ARG; }
        const GstArgs ga = {Lg, mp.gst_group, block, mp.frac_bits, mp.out_round, mp.scale_format, mp.nan_bits};
        return launch_emulate_gst(ga, A, B, C, D, SA, SB, m, n, k, batch, (hipStream_t)hip_stream);
    }
    if (mp.family == MMAEMU_FAMILY_FMA) {
        if (SA) { set_error("emulate_mma_scaled: block scales belong to the FDPA families"); return MMAEMU_ERR_UNSUPPORTED; }
        if (dt.a != MMAEMU_FP32 || dt.b != MMAEMU_FP32 || dt.c != MMAEMU_FP32 || dt.d != MMAEMU_FP32) {
            set_error("emulate_mma: the FMA family takes FP32 operands and accumulators");
            return MMAEMU_ERR_UNSUPPORTED;
        }
        const uint64_t mn_ = (uint64_t)m * n;
        if (batch && (mn_ > (1ull << 40) || batch > (1ull << 62) / mn_ || batch * mn_ > (1ull << 48))) {
            set_error("emulate_mma: problem too large");
            return MMAEMU_ERR_SHAPE;
        }
        if (batch == 0) return MMAEMU_OK;
        if (!A || !B || !C || !D) { set_error("emulate_mma: NULL device pointer"); return MMAEMU_ERR_INVALID_ARG; }
        return launch_emulate_fma(A, B, C, D, m, n, k, batch, mp.nan_bits, mp.nan_propagate != 0, (hipStream_t)hip_stream);
    }
    if (mp.family == MMAEMU_FAMILY_FTZ_ADDMUL && (is_narrow_type(dt.a) || is_narrow_type(dt.b) || is_word_type(dt.a))) {
        set_error("emulate_mma: the FTZ-AddMul family takes FP8, FP16 and BF16 operands");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (mp.family == MMAEMU_FAMILY_FTZ_ADDMUL) {
        if (k % mp.group_len) { set_error("emulate_mma: k=%u is not a multiple of P=%u", k, mp.group_len); return MMAEMU_ERR_SHAPE; }
        const uint64_t mn_ = (uint64_t)m * n;
        if (batch && (mn_ > (1ull << 40) || batch > (1ull << 62) / mn_ || batch * mn_ > (1ull << 48))) {
            set_error("emulate_mma: problem too large");
            return MMAEMU_ERR_SHAPE;
        }
        if (batch == 0) return MMAEMU_OK;
        if (!A || !B || !C || !D) { set_error("emulate_mma: NULL device pointer"); return MMAEMU_ERR_INVALID_ARG; }
        ModelArgs am = {};
        am.L = mp.group_len;
        am.nan_bits = mp.nan_bits;
        return launch_emulate_addmul(am, A, B, C, D, m, n, k, batch, dt.a, dt.b, (hipStream_t)hip_stream);
    }
    ModelArgs ma;
    {
        const mmaemu_status st = fdpa_model_args(mp, k, acc16, ma);
        if (st != MMAEMU_OK) return st;
    }
    const uint64_t mn = (uint64_t)m * n;
    if (batch && (mn > (1ull << 40) || batch > (1ull << 62) / mn || batch * mn > (1ull << 48) ||
                  batch * (uint64_t)(m > n ? m : n) > (1ull << 62) / k)) {
        set_error("emulate_mma: problem too large");
        return MMAEMU_ERR_SHAPE;
    }
    if (batch == 0) return MMAEMU_OK;
    if (!A || !B || !C || !D) { set_error("emulate_mma: NULL device pointer"); return MMAEMU_ERR_INVALID_ARG; }
    return launch_emulate(ma, A, B, C, D, m, n, k, batch, dt.a, dt.b, (hipStream_t)hip_stream, SA, SB, block);
}

mmaemu_status mmaemu_emulate_mma(const mmaemu_model *model, const void *A, const void *B, const void *C, void *D,
                                 uint32_t m, uint32_t n, uint32_t k, uint64_t batch, mmaemu_dtypes dt,
                                 void *hip_stream)
{
    return emulate_impl(model, A, B, C, D, nullptr, nullptr, 1, m, n, k, batch, dt, hip_stream);
}

mmaemu_status mmaemu_emulate_mma_scaled(const mmaemu_model *model, const void *A, const void *B, const void *C, void *D,
                                        const void *SA, const void *SB, uint32_t block, uint32_t m, uint32_t n, uint32_t k,
                                        uint64_t batch, mmaemu_dtypes dt, void *hip_stream)
{
    if (block == 0 || k % block) { set_error("emulate_mma_scaled: k=%u is not a multiple of the scale block %u", k, block); return MMAEMU_ERR_SHAPE; }
    if (batch && (!SA || !SB)) { set_error("emulate_mma_scaled: NULL scale pointer"); return MMAEMU_ERR_INVALID_ARG; }
    if (batch == 0) return emulate_impl(model, A, B, C, D, nullptr, nullptr, 1, m, n, k, batch, dt, hip_stream);
    return emulate_impl(model, A, B, C, D, (const uint8_t *)SA, (const uint8_t *)SB, block, m, n, k, batch, dt, hip_stream);
}

// whether the multi-model kernel takes a model (then with its arithmetic kind there)
static mmaemu_status many_class(const mmaemu_model_params &mp, const void *A, const void *B, uint32_t m, uint32_t n, uint32_t k,
                                mmaemu_dtypes dt, ModelArgs &p, bool &fused, uint32_t &kind, uint32_t &cls)
{
    fused = false;
    kind = 0;
    cls = 0;
    if (mp.family == MMAEMU_FAMILY_FDPA && is_ab_type(dt.a) && is_ab_type(dt.b)) {
        const mmaemu_status st = fdpa_model_args(mp, k, false, p);
        if (st != MMAEMU_OK) return st;
        fused = scan_takes(p, dt.a, dt.b, m, n, k, A, B, kind, cls);
    }
    return MMAEMU_OK;
}

mmaemu_status mmaemu_compare_many_classes(const mmaemu_model *const *models, uint32_t n_models, uint32_t m, uint32_t n,
                                          uint32_t k, mmaemu_dtypes dt, int32_t *class_of_model)
{
    if (!models || !class_of_model || n_models == 0 || n_models > MMAEMU_COMPARE_MANY_MAX) {
        set_error("compare_many_classes: 1 to %u models and an output array", (unsigned)MMAEMU_COMPARE_MANY_MAX);
        return MMAEMU_ERR_INVALID_ARG;
    }
    if (m == 0 || n == 0 || k == 0) { set_error("compare_many_classes: zero dimension"); return MMAEMU_ERR_SHAPE; }
    if (dt.a > MMAEMU_TF32 || dt.b > MMAEMU_TF32) { set_error("compare_many_classes: dtype out of range"); return MMAEMU_ERR_INVALID_ARG; }
    for (uint32_t i = 0; i < n_models; ++i) {
        if (!models[i] || models[i]->magic != MODEL_MAGIC) { set_error("compare_many_classes: bad model handle at %u", i); return MMAEMU_ERR_INVALID_ARG; }
        ModelArgs p;
        bool fused;
        uint32_t kind, cls;
        const mmaemu_status st = many_class(models[i]->params, nullptr, nullptr, m, n, k, dt, p, fused, kind, cls);
        if (st != MMAEMU_OK) return st;
        class_of_model[i] = fused ? (int32_t)cls : -1;          // (within a class the kernel takes any mix of group lengths and widths)
    }
    return MMAEMU_OK;
}

mmaemu_status mmaemu_emulate_compare_many(const mmaemu_model *const *models, uint32_t n_models, const void *A, const void *B,
                                          const void *C, const void *Dref, void *D_out, uint32_t m, uint32_t n, uint32_t k,
                                          uint64_t batch, mmaemu_dtypes dt, uint64_t index_base, mmaemu_stats *dev_stats,
                                          void *hip_stream)
{
    if (!models || n_models == 0 || n_models > MMAEMU_COMPARE_MANY_MAX) {
        set_error("emulate_compare_many: 1 to %u models", (unsigned)MMAEMU_COMPARE_MANY_MAX);
        return MMAEMU_ERR_INVALID_ARG;
    }
    for (uint32_t i = 0; i < n_models; ++i)
        if (!models[i] || models[i]->magic != MODEL_MAGIC) { set_error("emulate_compare_many: bad model handle at %u", i); return MMAEMU_ERR_INVALID_ARG; }
    if (!dev_stats) { set_error("emulate_compare_many: NULL statistics array"); return MMAEMU_ERR_INVALID_ARG; }
    if (m == 0 || n == 0 || k == 0) { set_error("emulate_compare_many: zero dimension (m=%u n=%u k=%u)", m, n, k); return MMAEMU_ERR_SHAPE; }
    if (dt.c != MMAEMU_FP32 || dt.d != MMAEMU_FP32) { set_error("emulate_compare_many: FP32 accumulators and outputs"); return MMAEMU_ERR_UNSUPPORTED; }
    if (dt.a > MMAEMU_TF32 || dt.b > MMAEMU_TF32) { set_error("emulate_compare_many: dtype out of range"); return MMAEMU_ERR_INVALID_ARG; }
    const uint64_t mn = (uint64_t)m * n;
    if (batch && (mn > (1ull << 40) || batch > (1ull << 48) / mn)) { set_error("emulate_compare_many: problem too large"); return MMAEMU_ERR_SHAPE; }
    if (batch == 0) return MMAEMU_OK;
    if (!A || !B || !C) { set_error("emulate_compare_many: NULL device pointer"); return MMAEMU_ERR_INVALID_ARG; }
    if (((uintptr_t)C | (uintptr_t)Dref | (uintptr_t)D_out | (uintptr_t)dev_stats) & 3u) {
        set_error("emulate_compare_many: C, Dref, D_out and the statistics must be 4-byte aligned");
        return MMAEMU_ERR_INVALID_ARG;
    }
    const uint64_t count = batch * mn;
    hipStream_t s = (hipStream_t)hip_stream;
    uint32_t *dout = static_cast<uint32_t *>(D_out);

    // which models the multi-model kernels take, and in which variant
    struct Item { ModelArgs p; bool fused, done; uint32_t kind, cls; };
    Item items[MMAEMU_COMPARE_MANY_MAX];
    bool all_one = n_models <= (uint32_t)MULTI_MAX;
    for (uint32_t i = 0; i < n_models; ++i) {
        Item &it = items[i];
        it.fused = false;
        it.done = false;
        it.kind = 0;
        it.cls = 0;
        const mmaemu_status cst = many_class(models[i]->params, A, B, m, n, k, dt, it.p, it.fused, it.kind, it.cls);
        if (cst != MMAEMU_OK) return cst;
        // (within a launch the models that flush subnormal inputs come last; a leading reference model that flushes
        // can therefore share its launch with flushing models only)
        all_one = all_one && it.fused && it.cls == items[0].cls && !(items[0].p.ftz_in && !it.p.ftz_in);
    }
    bool any_unfused = false;
    for (uint32_t i = 0; i < n_models; ++i) any_unfused = any_unfused || !items[i].fused;
    if (!dout && (any_unfused || (!Dref && !all_one))) {
        set_error("emulate_compare_many: this set of models does not run in one launch (or needs the general kernel): D_out is required");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    const uint32_t *ref = static_cast<const uint32_t *>(Dref);

    // fused launch of `lead` (if not UINT32_MAX: it leads the launch and is the reference) and every model the kernel
    // takes that has not run yet; at most MULTI_MAX per launch, FlushSubnormal sets last so that the staged operands are
    // flushed once at most
    auto run_class = [&](uint32_t lead, bool ref_is_first, uint32_t cls) -> mmaemu_status {
        for (;;) {
            MultiLaunch ml = {};
            ml.cls = cls;
            ml.ref_is_first = ref_is_first;
            ml.dref = ref;
            ml.dout = dout;
            ml.out_stride = count;
            ml.index_base = index_base;
            ml.stats = dev_stats;
            if (ref_is_first) { ml.slot[0] = lead; ml.models[0] = items[lead].p; ml.kind[0] = items[lead].kind; ml.count = 1; items[lead].done = true; }
            for (int pass = (ref_is_first && items[lead].p.ftz_in) ? 1 : 0; pass < 2; ++pass)
                for (uint32_t i = 0; i < n_models && ml.count < (uint32_t)MULTI_MAX; ++i) {
                    Item &it = items[i];
                    if (it.done || !it.fused || it.cls != cls || (int)(it.p.ftz_in != 0) != pass) continue;
                    ml.slot[ml.count] = i;
                    ml.models[ml.count] = it.p;
                    ml.kind[ml.count] = it.kind;
                    ml.count += 1;
                    it.done = true;
                }
            if (ml.count == 0) return MMAEMU_OK;
            const mmaemu_status st = launch_scan(ml, A, B, C, m, n, k, batch, dt.a, dt.b, s);
            if (st != MMAEMU_OK) return st;
            if (ref_is_first) {                    // what is left of the class compares with the first model's stored outputs
                ref_is_first = false;
                ref = dout;                        // (slot 0; null only when nothing is left)
                if (!ref) return MMAEMU_OK;
            }
        }
    };

    if (!ref) {
        // the reference is model 0's output: it runs first
        if (items[0].fused) {
            const mmaemu_status st = run_class(0, true, items[0].cls);
            if (st != MMAEMU_OK) return st;
        } else {
            mmaemu_status st = emulate_impl(models[0], A, B, C, dout, nullptr, nullptr, 1, m, n, k, batch, dt, hip_stream);
            if (st != MMAEMU_OK) return st;
            st = launch_compare(dout, dout, count, index_base, false, dev_stats, s);
            if (st != MMAEMU_OK) return st;
            items[0].done = true;
        }
        ref = dout;
    }
    for (uint32_t i = 0; i < n_models; ++i) {
        if (items[i].done) continue;
        if (items[i].fused) {
            const mmaemu_status st = run_class(UINT32_MAX, false, items[i].cls);
            if (st != MMAEMU_OK) return st;
        } else {
            uint32_t *Di = dout + (uint64_t)i * count;
            mmaemu_status st = emulate_impl(models[i], A, B, C, Di, nullptr, nullptr, 1, m, n, k, batch, dt, hip_stream);
            if (st != MMAEMU_OK) return st;
            st = launch_compare(Di, ref, count, index_base, false, dev_stats + i, s);
            if (st != MMAEMU_OK) return st;
            items[i].done = true;
        }
    }
    return MMAEMU_OK;
}

mmaemu_status mmaemu_stats_reset(mmaemu_stats *st, void *hip_stream)
{
    if (!st) { set_error("stats_reset: NULL"); return MMAEMU_ERR_INVALID_ARG; }
    return launch_stats_reset(st, (hipStream_t)hip_stream);
}

mmaemu_status mmaemu_compare(const void *D0, const void *D1, uint64_t count, uint64_t index_base, mmaemu_dtype d,
                             mmaemu_stats *st, void *hip_stream)
{
    if (d != MMAEMU_FP32 && d != MMAEMU_FP16 && d != MMAEMU_FP64) { set_error("compare: FP32, FP16 or FP64 outputs"); return MMAEMU_ERR_UNSUPPORTED; }
    const uintptr_t amask = d == MMAEMU_FP64 ? 7 : (d == MMAEMU_FP32 ? 3 : 1);
    if (!st) { set_error("compare: NULL stats"); return MMAEMU_ERR_INVALID_ARG; }
    if (count == 0) return MMAEMU_OK;
    if (!D0 || !D1) { set_error("compare: NULL device pointer"); return MMAEMU_ERR_INVALID_ARG; }
    if (((uintptr_t)D0 | (uintptr_t)D1) & amask) { set_error("compare: pointers must be aligned to the element size"); return MMAEMU_ERR_INVALID_ARG; }
    if (count > (1ull << 48)) { set_error("compare: count too large"); return MMAEMU_ERR_SHAPE; }
    if (d == MMAEMU_FP64) return launch_compare64(D0, D1, count, index_base, st, (hipStream_t)hip_stream);
    return launch_compare(D0, D1, count, index_base, d == MMAEMU_FP16, st, (hipStream_t)hip_stream);
}

// argument checks shared by mmaemu_generate and mmaemu_generate_noalloc; *run = false: valid, nothing to do
static mmaemu_status generate_check(const mmaemu_gen_params *g, void *out, mmaemu_dtype dtype, uint64_t ept,
                                    uint64_t first_tile, uint64_t n_tiles, bool *run)
{
    *run = false;
    if (!g) { set_error("generate: NULL params"); return MMAEMU_ERR_INVALID_ARG; }
    if (g->struct_size != sizeof(mmaemu_gen_params)) {
        set_error("generate: struct_size %u, expected %zu", g->struct_size, sizeof(mmaemu_gen_params));
        return MMAEMU_ERR_INVALID_ARG;
    }
    if (dtype == MMAEMU_TF32) { set_error("generate: TF32 streams are FP32 streams (generate MMAEMU_FP32)"); return MMAEMU_ERR_UNSUPPORTED; }
    if (((uint32_t)dtype > MMAEMU_FP4_E2M1 && dtype != MMAEMU_FP64) || g->family > MMAEMU_GEN_SIGNED_ZEROS || g->scale_scope > MMAEMU_SCALE_FACTOR) {
        set_error("generate: enum out of range");
        return MMAEMU_ERR_INVALID_ARG;
    }
    if (dtype == MMAEMU_FP64) {
        // binary64 output: the value families unscaled or times a constant, and the bit families that have a 64-bit reading
        const bool value_family = g->family == MMAEMU_GEN_NORMAL || g->family == MMAEMU_GEN_UNIFORM || g->family == MMAEMU_GEN_NORMAL_OUTLIERS;
        if (g->family == MMAEMU_GEN_CANCELLING || (value_family && (g->scale_scope == MMAEMU_SCALE_TENSOR || g->scale_scope == MMAEMU_SCALE_TILE))) {
            set_error("generate: FP64 output takes no CANCELLING family and no per-tensor / per-tile scaling");
            return MMAEMU_ERR_UNSUPPORTED;
        }
        if (ept == 0) { set_error("generate: elems_per_tile = 0"); return MMAEMU_ERR_SHAPE; }
        if (n_tiles > (1ull << 61) / ept || first_tile > (1ull << 61) / ept || (first_tile + n_tiles) > (1ull << 61) / ept) {
            set_error("generate: element index range too large");
            return MMAEMU_ERR_SHAPE;
        }
        if (g->family == MMAEMU_GEN_UNIFORM_EXP && (g->exp_lo > g->exp_hi || g->exp_hi > 2047u)) {
            set_error("generate: exponent-field range %u..%u outside 0..2047", g->exp_lo, g->exp_hi);
            return MMAEMU_ERR_UNSUPPORTED;
        }
        if (value_family && g->scale_scope != MMAEMU_SCALE_NONE && !(g->scale_target > 0.0)) { set_error("generate: scale_target must be positive"); return MMAEMU_ERR_INVALID_ARG; }
        if (n_tiles == 0) return MMAEMU_OK;
        if (!out) { set_error("generate: NULL output"); return MMAEMU_ERR_INVALID_ARG; }
        if ((uintptr_t)out & 7) { set_error("generate: output not aligned to its element size"); return MMAEMU_ERR_INVALID_ARG; }
        *run = true;
        return MMAEMU_OK;
    }
    if (dtype == MMAEMU_E8M0 && g->family != MMAEMU_GEN_ZERO && g->family != MMAEMU_GEN_RANDOM_BITS &&
        g->family != MMAEMU_GEN_UNIFORM_EXP) {
        set_error("generate: scale codes (E8M0) come from the ZERO, RANDOM_BITS and UNIFORM_EXP families only");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (ept == 0) { set_error("generate: elems_per_tile = 0"); return MMAEMU_ERR_SHAPE; }
    if (n_tiles > (1ull << 62) / ept || first_tile > (1ull << 62) / ept || (first_tile + n_tiles) > (1ull << 62) / ept) {
        set_error("generate: element index range too large");
        return MMAEMU_ERR_SHAPE;
    }
    const FmtInfo f = fmt_info(dtype);
    if (g->family == MMAEMU_GEN_CANCELLING && dtype == MMAEMU_FP32) {
        set_error("generate: CANCELLING is not defined for FP32 output");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (g->family == MMAEMU_GEN_UNIFORM_EXP || g->family == MMAEMU_GEN_CANCELLING) {
        const uint32_t emax_field = (1u << f.ebits) - 1u;
        if (g->exp_lo > g->exp_hi || g->exp_hi > emax_field) {
            set_error("generate: exponent-field range %u..%u outside 0..%u", g->exp_lo, g->exp_hi, emax_field);
            return MMAEMU_ERR_UNSUPPORTED;
        }
    }
    const bool value_family = g->family == MMAEMU_GEN_NORMAL || g->family == MMAEMU_GEN_UNIFORM || g->family == MMAEMU_GEN_NORMAL_OUTLIERS;
    if (value_family && g->scale_scope != MMAEMU_SCALE_NONE && !(g->scale_target > 0.0)) {
        set_error("generate: scale_target must be positive");
        return MMAEMU_ERR_INVALID_ARG;
    }
    if (n_tiles == 0) return MMAEMU_OK;
    if (!out) { set_error("generate: NULL output"); return MMAEMU_ERR_INVALID_ARG; }
    if ((uintptr_t)out & (uintptr_t)(f.width / 8 - 1)) { set_error("generate: output not aligned to its element size"); return MMAEMU_ERR_INVALID_ARG; }
    *run = true;
    return MMAEMU_OK;
}

mmaemu_status mmaemu_generate(const mmaemu_gen_params *g, void *out, mmaemu_dtype dtype, uint64_t ept,
                              uint64_t first_tile, uint64_t n_tiles, void *workspace, void *hip_stream)
{
    bool run;
    const mmaemu_status st = generate_check(g, out, dtype, ept, first_tile, n_tiles, &run);
    if (st != MMAEMU_OK || !run) return st;
    const bool value_family = g->family == MMAEMU_GEN_NORMAL || g->family == MMAEMU_GEN_UNIFORM || g->family == MMAEMU_GEN_NORMAL_OUTLIERS;
    if (value_family && g->scale_scope == MMAEMU_SCALE_TENSOR) {
        if (!workspace || ((uintptr_t)workspace & 7)) { set_error("generate: SCALE_TENSOR needs an 8-byte aligned workspace"); return MMAEMU_ERR_INVALID_ARG; }
    }
    return launch_generate(*g, out, dtype, ept, first_tile, n_tiles, workspace, (hipStream_t)hip_stream);
}

mmaemu_status mmaemu_generate_noalloc(const mmaemu_gen_params *g, void *out, mmaemu_dtype dtype, uint64_t ept,
                                      uint64_t first_tile, uint64_t n_tiles, void *hip_stream)
{
    bool run;
    const mmaemu_status st = generate_check(g, out, dtype, ept, first_tile, n_tiles, &run);
    if (st != MMAEMU_OK) return st;
    if (ept && n_tiles > MMAEMU_GENERATE_NOALLOC_MAX_ELEMS / ept) {
        set_error("generate_noalloc: %llu tiles of %llu elements exceed the limit of 2^40 elements per call",
                  (unsigned long long)n_tiles, (unsigned long long)ept);
        return MMAEMU_ERR_SHAPE;
    }
    if (!run) return MMAEMU_OK;
    return launch_generate_noalloc(*g, out, dtype, ept, first_tile, n_tiles, (hipStream_t)hip_stream);
}

// the block-scaled instructions: 16x16x128 (25 ids) and 32x32x64 (25 ids)
static bool is_scaled_instr(uint32_t i)
{
    return (i >= MMAEMU_MFMA_SCALE_F32_16X16X128_F8F6F4_BASE && i < MMAEMU_MFMA_F32_32X32X16_F16) ||
           (i >= MMAEMU_MFMA_SCALE_F32_32X32X64_F8F6F4_BASE && i < MMAEMU_MFMA_F32_32X32X4_2B_F16);
}

mmaemu_status mmaemu_mfma_info(mmaemu_mfma_instr instr, uint32_t *m, uint32_t *n, uint32_t *k_native, mmaemu_dtype *a,
                               mmaemu_dtype *b)
{
    if ((uint32_t)instr == MMAEMU_MFMA_F64_16X16X4_F64 || (uint32_t)instr == MMAEMU_MFMA_F64_4X4X4_4B_F64) {
        const uint32_t mm_ = (uint32_t)instr == MMAEMU_MFMA_F64_16X16X4_F64 ? 16u : 4u;
        if (m) *m = mm_;
        if (n) *n = mm_;
        if (k_native) *k_native = 4;
        if (a) *a = MMAEMU_FP64;
        if (b) *b = MMAEMU_FP64;
        return MMAEMU_OK;
    }
    if ((uint32_t)instr >= MMAEMU_MFMA_F32_32X32X4_2B_F16 && (uint32_t)instr <= MMAEMU_MFMA_F32_4X4X1_16B_F32) {     // multi-block forms
        const uint32_t q = (uint32_t)instr - MMAEMU_MFMA_F32_32X32X4_2B_F16, shape = q % 3, type = q / 3;
        const uint32_t mm_ = shape == 0 ? 32u : (shape == 1 ? 16u : 4u);
        if (m) *m = mm_;
        if (n) *n = mm_;
        if (k_native) *k_native = type == 2 ? 1u : 4u;
        if (a) *a = type == 0 ? MMAEMU_FP16 : (type == 1 ? MMAEMU_BF16 : MMAEMU_FP32);
        if (b) *b = type == 0 ? MMAEMU_FP16 : (type == 1 ? MMAEMU_BF16 : MMAEMU_FP32);
        return MMAEMU_OK;
    }
    if ((uint32_t)instr == MMAEMU_MFMA_F32_16X16X4_F32 || (uint32_t)instr == MMAEMU_MFMA_F32_32X32X2_F32) {
        const bool small = (uint32_t)instr == MMAEMU_MFMA_F32_16X16X4_F32;
        if (m) *m = small ? 16 : 32;
        if (n) *n = small ? 16 : 32;
        if (k_native) *k_native = small ? 4 : 2;
        if (a) *a = MMAEMU_FP32;
        if (b) *b = MMAEMU_FP32;
        return MMAEMU_OK;
    }
    if ((uint32_t)instr >= MMAEMU_MFMA_F32_32X32X16_F16 && (uint32_t)instr <= MMAEMU_MFMA_F32_32X32X16_BF8_BF8) {
        static const mmaemu_dtype T2[6][2] = {{MMAEMU_FP16, MMAEMU_FP16}, {MMAEMU_BF16, MMAEMU_BF16}, {MMAEMU_FP8_E4M3, MMAEMU_FP8_E4M3},
                                              {MMAEMU_FP8_E4M3, MMAEMU_FP8_E5M2}, {MMAEMU_FP8_E5M2, MMAEMU_FP8_E4M3}, {MMAEMU_FP8_E5M2, MMAEMU_FP8_E5M2}};
        const uint32_t q = (uint32_t)instr - MMAEMU_MFMA_F32_32X32X16_F16;
        if (m) *m = 32;
        if (n) *n = 32;
        if (k_native) *k_native = 16;
        if (a) *a = T2[q][0];
        if (b) *b = T2[q][1];
        return MMAEMU_OK;
    }
    if (is_scaled_instr((uint32_t)instr)) {
        static const mmaemu_dtype F[5] = {MMAEMU_FP8_E4M3, MMAEMU_FP8_E5M2, MMAEMU_FP6_E2M3, MMAEMU_FP6_E3M2, MMAEMU_FP4_E2M1};
        const bool big = (uint32_t)instr >= MMAEMU_MFMA_SCALE_F32_32X32X64_F8F6F4_BASE;
        const uint32_t q = (uint32_t)instr - (big ? MMAEMU_MFMA_SCALE_F32_32X32X64_F8F6F4_BASE : MMAEMU_MFMA_SCALE_F32_16X16X128_F8F6F4_BASE);
        if (m) *m = big ? 32 : 16;
        if (n) *n = big ? 32 : 16;
        if (k_native) *k_native = big ? 64 : 128;
        if (a) *a = F[q / 5];
        if (b) *b = F[q % 5];
        return MMAEMU_OK;
    }
    static const struct { uint32_t m, n, k; mmaemu_dtype a, b; } T[10] = {
        {16, 16, 16, MMAEMU_FP16, MMAEMU_FP16},         {16, 16, 16, MMAEMU_BF16, MMAEMU_BF16},
        {32, 32, 8, MMAEMU_FP16, MMAEMU_FP16},          {32, 32, 8, MMAEMU_BF16, MMAEMU_BF16},
        {16, 16, 32, MMAEMU_FP16, MMAEMU_FP16},         {16, 16, 32, MMAEMU_BF16, MMAEMU_BF16},
        {16, 16, 32, MMAEMU_FP8_E4M3, MMAEMU_FP8_E4M3}, {16, 16, 32, MMAEMU_FP8_E4M3, MMAEMU_FP8_E5M2},
        {16, 16, 32, MMAEMU_FP8_E5M2, MMAEMU_FP8_E4M3}, {16, 16, 32, MMAEMU_FP8_E5M2, MMAEMU_FP8_E5M2}};
    if ((uint32_t)instr >= MMAEMU_MFMA_COUNT) { set_error("mfma_info: unknown instruction %u", (uint32_t)instr); return MMAEMU_ERR_INVALID_ARG; }
    if (m) *m = T[instr].m;
    if (n) *n = T[instr].n;
    if (k_native) *k_native = T[instr].k;
    if (a) *a = T[instr].a;
    if (b) *b = T[instr].b;
    return MMAEMU_OK;
}

mmaemu_status mmaemu_mfma_probe(mmaemu_mfma_instr instr, const void *A, const void *B, const void *C, void *D, uint32_t k,
                                uint64_t batch, void *hip_stream)
{
    uint32_t m, n, kn;
    mmaemu_dtype ta, tb;
    mmaemu_status st = mmaemu_mfma_info(instr, &m, &n, &kn, &ta, &tb);
    if (st != MMAEMU_OK) return st;
    if (is_scaled_instr((uint32_t)instr)) { set_error("mfma_probe: a block-scaled instruction needs mfma_probe_scaled"); return MMAEMU_ERR_INVALID_ARG; }
    if (k == 0 || k > kn) { set_error("mfma_probe: k=%u outside 1..%u", k, kn); return MMAEMU_ERR_SHAPE; }
    if (batch > (1ull << 40)) { set_error("mfma_probe: batch too large"); return MMAEMU_ERR_SHAPE; }
    if (batch == 0) return MMAEMU_OK;
    if (!A || !B || !C || !D) { set_error("mfma_probe: NULL device pointer"); return MMAEMU_ERR_INVALID_ARG; }
    const bool f64 = ta == MMAEMU_FP64;
    const uintptr_t ab_align = f64 ? 7 : (uintptr_t)(fmt_info(ta).width / 8 - 1);
    if (((uintptr_t)A | (uintptr_t)B) & ab_align || ((uintptr_t)C | (uintptr_t)D) & (f64 ? 7 : 3)) {
        set_error("mfma_probe: misaligned pointer");
        return MMAEMU_ERR_INVALID_ARG;
    }
    return launch_mfma_probe((uint32_t)instr, A, B, C, D, k, batch, (hipStream_t)hip_stream);
}

mmaemu_status mmaemu_mfma_probe_scaled(mmaemu_mfma_instr instr, const void *A, const void *B, const void *C, void *D,
                                       const void *SA, const void *SB, uint32_t k, uint64_t batch, void *hip_stream)
{
    uint32_t m, n, kn;
    mmaemu_status st = mmaemu_mfma_info(instr, &m, &n, &kn, nullptr, nullptr);
    if (st != MMAEMU_OK) return st;
    if (!is_scaled_instr((uint32_t)instr)) { set_error("mfma_probe_scaled: not a block-scaled instruction"); return MMAEMU_ERR_INVALID_ARG; }
    if (k == 0 || k > kn || k % 32) { set_error("mfma_probe_scaled: k=%u must be a multiple of 32 up to %u", k, kn); return MMAEMU_ERR_SHAPE; }
    if (batch > (1ull << 40)) { set_error("mfma_probe_scaled: batch too large"); return MMAEMU_ERR_SHAPE; }
    if (batch == 0) return MMAEMU_OK;
    if (!A || !B || !C || !D || !SA || !SB) { set_error("mfma_probe_scaled: NULL device pointer"); return MMAEMU_ERR_INVALID_ARG; }
    if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C | (uintptr_t)D) & 3) { set_error("mfma_probe_scaled: pointers must be 4-byte aligned"); return MMAEMU_ERR_INVALID_ARG; }
    return launch_mfma_probe_scaled((uint32_t)instr, A, B, C, D, SA, SB, k, batch, (hipStream_t)hip_stream);
}

uint32_t mmaemu_issue_probe_count(void) { return issue_probe_count(); }

const char *mmaemu_issue_probe_name(uint32_t op) { return issue_probe_name(op); }

mmaemu_status mmaemu_issue_probe(uint32_t op, uint32_t iterations, uint32_t workgroups, void *out, void *hip_stream)
{
    if (op >= issue_probe_count()) { set_error("issue_probe: unknown instruction %u", op); return MMAEMU_ERR_INVALID_ARG; }
    if (iterations == 0 || workgroups == 0 || workgroups > (1u << 20)) { set_error("issue_probe: iterations and workgroups (up to 2^20) must be positive"); return MMAEMU_ERR_SHAPE; }
    if (!out || ((uintptr_t)out & 3)) { set_error("issue_probe: out must be 1 KiB of 4-byte aligned device memory"); return MMAEMU_ERR_INVALID_ARG; }
    return launch_issue_probe(op, iterations, workgroups, static_cast<uint32_t *>(out), (hipStream_t)hip_stream);
}

mmaemu_status mmaemu_err_stats_reset(mmaemu_err_stats *st, void *hip_stream)
{
    if (!st) { set_error("err_stats_reset: NULL"); return MMAEMU_ERR_INVALID_ARG; }
    return launch_err_stats_reset(st, (hipStream_t)hip_stream);
}

mmaemu_status mmaemu_exact_dot_sample(const void *A, const void *B, const void *D, uint32_t m, uint32_t n, uint32_t k,
                                      mmaemu_dtypes dt, uint64_t stride, mmaemu_err_stats *st, void *hip_stream)
{
    if (!A || !B || !D || !st) { set_error("exact_dot_sample: NULL pointer"); return MMAEMU_ERR_INVALID_ARG; }
    if (m == 0 || n == 0 || k == 0 || k > (1u << 20) || stride == 0) { set_error("exact_dot_sample: bad shape or stride"); return MMAEMU_ERR_SHAPE; }
    if (dt.a > MMAEMU_FP8_E5M2 || dt.b > MMAEMU_FP8_E5M2 || dt.d != MMAEMU_FP32) {
        set_error("exact_dot_sample: operands must be FP8 and D FP32");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    return launch_exact_dot_sample(A, B, (const uint32_t *)D, m, n, k, dt.a, dt.b, stride, st, (hipStream_t)hip_stream);
}

mmaemu_status mmaemu_deviation_hist_reset(mmaemu_deviation_hist *h, void *hip_stream)
{
    if (!h) { set_error("deviation_hist_reset: NULL"); return MMAEMU_ERR_INVALID_ARG; }
    return launch_deviation_reset(h, (hipStream_t)hip_stream);
}

mmaemu_status mmaemu_deviation_sample(const void *A, const void *B, const void *C, const void *D, uint32_t m, uint32_t n,
                                      uint32_t k, uint64_t batch, mmaemu_dtypes dt, uint64_t stride, int32_t bin_exp,
                                      mmaemu_deviation_hist *h, void *hip_stream)
{
    if (!A || !B || !D || !h) { set_error("deviation_sample: NULL pointer"); return MMAEMU_ERR_INVALID_ARG; }
    if (((uintptr_t)D & 3) || ((uintptr_t)C & 3) || ((uintptr_t)h & 7)) { set_error("deviation_sample: misaligned pointer"); return MMAEMU_ERR_INVALID_ARG; }
    if (m == 0 || n == 0 || k == 0 || k > (1u << 20) || stride == 0) { set_error("deviation_sample: bad shape or stride"); return MMAEMU_ERR_SHAPE; }
    if (batch > (1ull << 62) / ((uint64_t)m * n)) { set_error("deviation_sample: batch * m * n too large"); return MMAEMU_ERR_SHAPE; }
    const bool ab_ok = (is_byte_type(dt.a) || dt.a == MMAEMU_FP16 || dt.a == MMAEMU_BF16) && (is_byte_type(dt.b) || dt.b == MMAEMU_FP16 || dt.b == MMAEMU_BF16);
    if (!ab_ok || dt.c != MMAEMU_FP32 || dt.d != MMAEMU_FP32) {
        set_error("deviation_sample: operands of at most 16 bits, FP32 accumulator and output");
        return MMAEMU_ERR_UNSUPPORTED;
    }
    if (((uintptr_t)A & (is_byte_type(dt.a) ? 0 : 1)) || ((uintptr_t)B & (is_byte_type(dt.b) ? 0 : 1))) { set_error("deviation_sample: misaligned operands"); return MMAEMU_ERR_INVALID_ARG; }
    if (bin_exp < -280 || bin_exp > 250) { set_error("deviation_sample: bin_exp outside -280 .. 250"); return MMAEMU_ERR_INVALID_ARG; }
    if (batch == 0) return MMAEMU_OK;
    return launch_deviation_sample(A, B, (const uint32_t *)C, (const uint32_t *)D, m, n, k, batch, dt.a, dt.b, stride, bin_exp, h,
                                   (hipStream_t)hip_stream);
}

} // extern "C"
