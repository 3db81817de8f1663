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
    // Algorithm "E-FDPA" on whole 16 x 16 blocks: operands shared through LDS, the exact sum held in a pair of binary64 numbers
    if (!scaled && efdpa_blocks_take(p, ta, tb, m, n, k)) return launch_emulate_efdpa(p, A, B, Cm, D, m, n, k, batch, ta, tb, s);
    if (!scaled && efdpa_pairs_take(p, Cm, D, k)) return launch_emulate_efdpa_pairs(p, A, B, Cm, D, m, n, k, batch, ta, tb, s);
    return launch_emulate_generic(p, A, B, Cm, D, m, n, k, batch, ta, tb, s, SA, SB, scaled ? block : 1u);
}

} // namespace mmaemu
