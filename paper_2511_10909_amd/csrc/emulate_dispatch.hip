// Dispatch of the emulation entry point: tiled kernels where shape and parameters allow,
// the general kernel otherwise.
#include "emulate_tiled.hpp"

namespace mmaemu {

template <int VM>
static mmaemu_status launch_vm(const TiledArgs &t, const void *A, const void *B, const void *Cm, void *D, uint32_t m, uint32_t n,
                               uint32_t k, uint64_t batch, hipStream_t s, bool &handled)
{
    if (t.p.c_mode == MMAEMU_C_IN_GROUP) return launch_tiled_shape<MMAEMU_C_IN_GROUP, VM>(t, A, B, Cm, D, m, n, k, batch, s, handled);
    if (t.p.c_mode == MMAEMU_C_AFTER_EXACT) return launch_tiled_shape<MMAEMU_C_AFTER_EXACT, VM>(t, A, B, Cm, D, m, n, k, batch, s, handled);
    if (t.p.split == MMAEMU_SPLIT_NONE) return launch_tiled_shape<MMAEMU_C_AFTER_RD, VM>(t, A, B, Cm, D, m, n, k, batch, s, handled);
    if constexpr (VM == 0 || VM == 3) {
        if (t.p.split == MMAEMU_SPLIT_EVEN_ODD) return launch_tiled_shape<CM_RD_EVEN_ODD, VM>(t, A, B, Cm, D, m, n, k, batch, s, handled);
        if (t.p.split == MMAEMU_SPLIT_HALVES) return launch_tiled_shape<CM_RD_HALVES, VM>(t, A, B, Cm, D, m, n, k, batch, s, handled);
        return launch_tiled_shape<CM_RD_QUARTERS, VM>(t, A, B, Cm, D, m, n, k, batch, s, handled);
    }
    handled = false;        // split groups with BF16 or TF32 operands or wide F: general kernel
    return MMAEMU_OK;
}

mmaemu_status launch_emulate(const ModelArgs &p, const void *A, const void *B, const void *Cm, void *D,
                             uint32_t m, uint32_t n, uint32_t k, uint64_t batch, uint32_t ta, uint32_t tb,
                             hipStream_t s, const uint8_t *SA, const uint8_t *SB, uint32_t block)
{
    // the tiled kernels need 8-byte aligned operand arrays (four consecutive k elements are
    // loaded at once) and group sums below 2^52
    const bool aligned = ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 7) == 0;
    // the RD mode runs tiled with all of its variations; the two other modes only as the paper has them
    // (the tiled kernels tag BF16 and TF32 products of 2^128 and more as infinities: without that rule such products need
    // the general kernel's integer range)
    const bool wide_bf16 = p.wide_products && (ta == MMAEMU_BF16 || tb == MMAEMU_BF16 || ta == MMAEMU_TF32);
    // (rounding toward zero in place of the round-downs: the tiled kernels have it for unsplit groups with the plain F2 rule)
    const bool rz_ok = !p.rd_toward_zero || (p.split == MMAEMU_SPLIT_NONE && !p.f2_at_leading_bit);
    const bool tiled_mode = p.c_mode != MMAEMU_C_EXACT && rz_ok &&
                            ((p.c_mode == MMAEMU_C_AFTER_RD && !wide_bf16) || (p.c_mode != MMAEMU_C_AFTER_RD && !p.skip_zero_terms && !p.zero_result_positive));
    // block scales run tiled when every group lies inside one block (all of its products then share one scale
    // exponent) and the values stay binary32 (FP8 / FP16 operands, F below 30)
    const bool scaled = SA != nullptr;
    const bool tf32 = ta == MMAEMU_TF32;                                  // (pairs with itself only)
    const bool scaled_ok = !scaled || (block % p.L == 0 && ta != MMAEMU_BF16 && tb != MMAEMU_BF16 && !tf32 && p.F < 30);
    // FP32 operands run in the general kernel only, and so does F above 40; TF32 operands (four to a 128-bit load) run
    // tiled with binary32 values, i.e. F below 30, from 16-byte aligned arrays
    const bool aligned16 = ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 15) == 0;
    const bool tiled_types = ta != MMAEMU_FP32 && p.F <= 40 && (!tf32 || (p.F < 30 && aligned16));
    if (tiled_mode && tiled_types && scaled_ok && aligned && (uint64_t)p.L <= (1ull << (50 - p.F))) {
        TiledArgs t;
        t.p = p;
        t.ta = ta;
        t.tb = tb;
        t.sa = SA;
        t.sb = SB;
        t.block = block;
        t.ebase = 2 - fmt_info(ta).bias - fmt_info(tb).bias -
                  ((p.c_mode == MMAEMU_C_AFTER_RD && p.skip_zero_terms) ? 2 * (int)ZBIAS : 0);
        bool handled = false;
        mmaemu_status st;
        if (scaled) st = launch_vm<3>(t, A, B, Cm, D, m, n, k, batch, s, handled);
        else if (tf32) st = launch_vm<4>(t, A, B, Cm, D, m, n, k, batch, s, handled);
        else if (p.F >= 30) st = launch_vm<2>(t, A, B, Cm, D, m, n, k, batch, s, handled);             // wide F: binary64 terms
        else if (ta == MMAEMU_BF16 || tb == MMAEMU_BF16) st = launch_vm<1>(t, A, B, Cm, D, m, n, k, batch, s, handled);
        else st = launch_vm<0>(t, A, B, Cm, D, m, n, k, batch, s, handled);
        if (handled) return st;
    }
    return launch_emulate_generic(p, A, B, Cm, D, m, n, k, batch, ta, tb, s, SA, SB, scaled ? block : 1u);
}

// ---- several models per launch ----------------------------------------------------------------

// Whether the multi-model kernels take this model on this problem, and the kernel variant it needs there (value mode,
// fold period: the same choice launch_fold makes for one model).
bool multi_class(const ModelArgs &p, uint32_t ta, uint32_t tb, uint32_t m, uint32_t n, uint32_t k, const void *A, const void *B,
                 int &vm, int &nf)
{
    if (p.c_mode != MMAEMU_C_IN_GROUP || p.skip_zero_terms || p.zero_result_positive || (p.flags & (FL_ACC16 | FL_NAN_PROPAGATE))) return false;
    if (!((m == 16 && n == 16 && k == 16) || (m == 32 && n == 32 && k == 8))) return false;
    if (ta == MMAEMU_FP32 || tb == MMAEMU_FP32 || ta == MMAEMU_TF32 || tb == MMAEMU_TF32) return false;
    if ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 7) return false;
    if (p.F > 40) return false;
    if (!(p.L == 4 || p.L == 8 || (p.L == 16 && k == 16))) return false;
    vm = p.F >= 30 ? 2 : ((ta == MMAEMU_BF16 || tb == MMAEMU_BF16) ? 1 : 0);
    const uint64_t term = 1ull << (p.F + 2);                // |aligned term| < 2^(F+2)
    nf = vm == 2 ? 0 : ((uint64_t)p.L * term <= (1ull << 31) ? 0 : (4 * term <= (1ull << 31) ? 4 : 1));
    return true;
}

// One launch: the models of `ml` (all of one class as multi_class names it) over the batch's tiles.
mmaemu_status launch_multi(const MultiLaunch &ml, const void *A, const void *B, const void *C, uint32_t m, uint32_t n, uint32_t k,
                           uint64_t batch, uint32_t ta, uint32_t tb, hipStream_t s)
{
    MultiArgs mu = {};
    mu.t.p = ml.models[0];
    mu.t.ta = ta;
    mu.t.tb = tb;
    mu.t.sa = nullptr;
    mu.t.sb = nullptr;
    mu.t.block = 1;
    mu.t.ebase = 2 - fmt_info(ta).bias - fmt_info(tb).bias;
    mu.count = ml.count;
    mu.ref_is_first = ml.ref_is_first ? 1u : 0u;
    mu.dref = ml.dref;
    mu.dout = ml.dout;
    mu.out_stride = ml.out_stride;
    mu.index_base = ml.index_base;
    mu.stats = reinterpret_cast<uint64_t *>(ml.stats);
    for (uint32_t i = 0; i < ml.count; ++i) {
        mu.slot[i] = ml.slot[i];
        mu.models[i] = ml.models[i];
        mu.hot[i] = MultiArgs::Hot{ml.models[i].F, ml.models[i].flags, ml.models[i].out_mask, ml.models[i].nan_bits};
    }
    const MultiCall call = {A, B, static_cast<const uint32_t *>(C), m, n, k, batch};
    bool handled = false;
    mmaemu_status st;
    if (ml.vm == 2) st = launch_multi_shape<2>(mu, call, ml.L, ml.nf, s, handled);
    else if (ml.vm == 1) st = launch_multi_shape<1>(mu, call, ml.L, ml.nf, s, handled);
    else st = launch_multi_shape<0>(mu, call, ml.L, ml.nf, s, handled);
    if (st == MMAEMU_OK && !handled) { set_error("emulate_compare_many: no kernel for this shape"); return MMAEMU_ERR_UNSUPPORTED; }
    return st;
}

} // namespace mmaemu
