/*
 * libmmaemu -- evaluation of parameterised bit-accurate matrix-multiply-accumulate
 * arithmetic models on AMD CDNA4 (gfx950), after "Bit-Accurate Modeling of GPU Matrix
 * Multiply-Accumulate Units" (closed-loop feature probing, CLFP).
 *
 * The library is the data-parallel part of CLFP's randomized validation (paper
 * Sec. 3.1, Step 4): generate random operand tiles on the device, push them through
 * one or more arithmetic-behaviour models Phi (Sec. 4.1.3) and through the native
 * matrix instruction, and count bitwise disagreements (Eq. 2).
 *
 * Conventions, valid for every call unless stated otherwise
 *   - Pointers named A, B, C, D, out, dev_* and workspace are DEVICE pointers owned by
 *     the caller; the library never allocates, frees or retains device memory.
 *     All other pointers are HOST pointers.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).  Work is
 *     enqueued on it and the call returns without synchronising.
 *   - Errors are return codes; nothing aborts or throws.  Arguments are validated on
 *     the host before anything is launched; on error nothing has been enqueued.
 *     mmaemu_last_error() gives a thread-local description of the last failure.
 *   - Matrix layout: a batch of independent tiles, tile-major and K-contiguous for both
 *     multiplicands: A[batch][m][k], B[batch][n][k], C[batch][m][n], D[batch][m][n];
 *     batch = 1 is an ordinary GEMM-shaped problem.  Elements are raw bit patterns:
 *     1 byte (FP8), 2 bytes (FP16, BF16) or 4 bytes (FP32), little endian.
 */
#ifndef MMAEMU_H
#define MMAEMU_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MMAEMU_OK = 0,
    MMAEMU_ERR_INVALID_ARG = 1, /* NULL pointer, bad enum value, bad struct_size */
    MMAEMU_ERR_UNSUPPORTED = 2, /* valid in the paper's terms but outside what the kernels cover */
    MMAEMU_ERR_SHAPE = 3,       /* zero dimension, K not a multiple of L, size over a stated limit */
    MMAEMU_ERR_HIP = 4,         /* a HIP runtime call failed; text in mmaemu_last_error() */
    MMAEMU_ERR_NOMEM = 5
} mmaemu_status;

/* Operand encodings.  FP8 flavours are the OCP ones (E4M3: no infinity, one NaN
 * mantissa, max 448; E5M2: IEEE-like, max 57344).  Decoding follows the paper's
 * "exact unnormalized products" (Sec. 4.1.3, T-FDPA): exponent field 0 means
 * Exp = 1 - bias and no hidden bit, for zeros as well. */
typedef enum {
    MMAEMU_FP8_E4M3 = 0,
    MMAEMU_FP8_E5M2 = 1,
    MMAEMU_FP16 = 2,
    MMAEMU_BF16 = 3,
    MMAEMU_FP32 = 4,
    MMAEMU_E8M0 = 5, /* block-scale codes (Algorithm "ST-FDPA"): one byte, 2^(code - 127), 0xFF = NaN; no sign, no
                        mantissa.  Only mmaemu_generate takes it (families ZERO, RANDOM_BITS, UNIFORM_EXP, where the
                        "exponent field" is the whole code). */
    /* FP6 and FP4 operands (element formats of the OCP microscaling specification; Require lines of Algorithms
     * "T-FDPA" and "ST-FDPA"): every code is a finite number; one code per byte in its low 6 / 4 bits (sign on top),
     * higher bits ignored on input and written as zero by mmaemu_generate. */
    MMAEMU_FP6_E2M3 = 6, /* bias 1, largest 7.5 */
    MMAEMU_FP6_E3M2 = 7, /* bias 3, largest 28 */
    MMAEMU_FP4_E2M1 = 8, /* bias 1, largest 6 */
    /* TF32 operands (Require lines of Algorithms "T-FDPA" and "TR-FDPA"): one binary32 word per element, of which the
     * sign, the 8 exponent bits and the top 10 mantissa bits count; the low 13 bits are ignored on input (a NaN whose
     * payload lies only there reads as an infinity).  Pairs with itself only; mmaemu_generate does not take it
     * (every MMAEMU_FP32 stream is a TF32 stream). */
    MMAEMU_TF32 = 9,
    /* binary64, eight bytes per element: the other format Algorithms "FMA" and "Phi_FMA" are stated for.  Taken by the
     * FMA family (all four arrays FP64), mmaemu_generate, mmaemu_compare and the FP64 MFMA probes. */
    MMAEMU_FP64 = 10
} mmaemu_dtype;

typedef struct {
    uint32_t a, b, c, d; /* mmaemu_dtype values; a, b in {E4M3, E5M2, FP16, BF16, FP32, E2M3, E3M2, E2M1, TF32} (the FP6 /
                            FP4 types pair with each other and with the FP8 types, TF32 and FP32 each with itself; FP32
                            operands and frac_bits above 40 run in the general kernel); c = d = FP32, or c = d = FP16
                            (Algorithm "T-FDPA" with F_C = FP16: the accumulator is decoded as binary16, Exp >= -14,
                            rho is RNE-FP16 of Table "Conversion functions" (RZ likewise), both flushes use 2^-14, the
                            NaN pattern is the low half of nan_bits; c_mode C_IN_GROUP or C_AFTER_EXACT only) */
} mmaemu_dtypes;

enum { MMAEMU_C_IN_GROUP = 0, MMAEMU_C_AFTER_EXACT = 1, MMAEMU_C_AFTER_RD = 2, MMAEMU_C_AFTER_RD_EVEN_ODD = 3, MMAEMU_C_EXACT = 4 };
enum { MMAEMU_ROUND_RNE = 0, MMAEMU_ROUND_RZ = 1 };
enum { MMAEMU_ALIGN_RZ = 0 };
enum { MMAEMU_SPLIT_NONE = 0, MMAEMU_SPLIT_EVEN_ODD = 1, MMAEMU_SPLIT_HALVES = 2, MMAEMU_SPLIT_QUARTERS = 3 };
enum { MMAEMU_FAMILY_FDPA = 0, MMAEMU_FAMILY_FTZ_ADDMUL = 1, MMAEMU_FAMILY_GST_FDPA = 2, MMAEMU_FAMILY_FMA = 3 };
enum { MMAEMU_SCALE_FORMAT_E8M0 = 0, MMAEMU_SCALE_FORMAT_UE4M3 = 1 };

/*
 * One arithmetic-behaviour model: the chained FDPA model (paper Algorithm "Phi_FDPA")
 * around the truncated fused dot-product-add (Algorithm "T-FDPA"):
 *   L = min(K, group_len)            (group_len = 0: fully fused, L = K)
 *   d <- c; for each consecutive group of L products: d <- FDPA(a_group, b_group, d)
 *   FDPA: exact products s_k, e_k = Exp(a_k) + Exp(b_k); e_max over the L products and
 *         the accumulator; each term aligned at e_max and truncated toward zero to
 *         frac_bits (F) fractional bits; exact fixed-point sum; conversion rho.
 * c_mode = MMAEMU_C_AFTER_EXACT keeps the accumulator out of the truncated sum:
 *   T over the L products only (e_max over the products), d = rho(T * 2^e_max + c)
 *   with that two-term sum exact (Algorithm "TR-FDPA" without its two RD roundings).
 * c_mode = MMAEMU_C_AFTER_RD is Algorithm "TR-FDPA": T as above; E = max(e_max, e_c);
 *   T is rounded down (toward minus infinity) to frac_bits2 (F2) and the accumulator to
 *   frac_bits (F) fractional bits at E; d = rho of their sum.  A product of magnitude
 *   2^128 or more counts as an infinity of its sign (Sec. 4.2).
 * c_mode = MMAEMU_C_AFTER_RD_EVEN_ODD is Algorithm "GTR-FDPA": the products of even and
 *   of odd index within a group are fused apart, each at its own maximum exponent; the
 *   two sums are rounded down to F bits at the larger of the two and added; then as
 *   TR-FDPA, except that the accumulator's term is dropped when e_c < E - F - 1.
 *   L must be even.  (Table "TR-FDPA and GTR-FDPA parameter selection": F = 24,
 *   F2 = 31, RNE-FP32, L_max = 8 for 16-bit and 16 for 8-bit inputs.)  It is the same as
 *   C_AFTER_RD with split = MMAEMU_SPLIT_EVEN_ODD and acc_special_truncation = 1.
 * c_mode = MMAEMU_C_EXACT is Algorithm "E-FDPA" (the exact fused dot-product-add of the CDNA1 instructions): the L
 *   products and the accumulator are summed exactly, whatever their exponents, and rho is applied once per group;
 *   frac_bits plays no part.  The sum is held as an unevaluated pair of binary64 numbers while that is exact and in a
 *   640-bit fixed-point number otherwise (in a second launch over the outputs that need it, unless D is C); whole
 *   16 x 16 blocks share their operands through LDS, other shapes run one thread per output.  Every operand type,
 *   unscaled operands, FP32 accumulators.
 * Variations of C_AFTER_RD that the paper does not print (each 0 by default, which gives
 * the paper's algorithms; they were found by running the paper's probing method against
 * the MFMA instructions of gfx950):
 *   split                  sub-groups of a group: none, even / odd products, first / second half, or the four
 *                          consecutive quarters (each fused at its own maximum, all merged at the largest; L % 4 = 0)
 *   acc_special_truncation the special truncation of GTR-FDPA (threshold e_c < E - F_c - 1)
 *   frac_bits_merge (F_m)  fractional bits of the RD roundings that merge the sub-group sums (0: F)
 *   frac_bits_acc (F_c)    fractional bits of the accumulator's RD rounding (0: F)
 *   f2_at_leading_bit      T 2^(e_max - E) + s_c' is formed exactly, then rounded down to F2
 *                          fractional bits counted below its own leading bit instead of below 2^E
 *                          (below 2^-126 when the sum is smaller than that)
 *   sum_drop_distance (n)  counterpart of the special truncation for the product sum:
 *                          T' = 0 when E - e_max >= n (0: never)
 *   wide_products          a product of magnitude 2^128 or more keeps its value (no infinity
 *                          from a single product; overflow happens where a group's sum is
 *                          converted): the block-scaled MFMA of gfx950 behaves so
 * and of every mode:
 *   skip_zero_terms        products with a zero significand take no part in any exponent maximum
 *                          (the accumulator always does; a zero one has the exponent -126)
 *   zero_result_positive   a result that rounds or is flushed to zero is +0.0
 * out_round: rho = RNE-FP32 or RZ-FP32 (Table "Conversion functions"); overflow gives
 *   infinity (RNE) or the largest finite value (RZ); an exact-zero sum gives +0.0.
 *   out_mant_bits = 13 with out_round = RZ is RZ-E8M13 of the same table: binary32 with the
 *   low 10 mantissa bits cut toward zero (D still holds binary32 patterns).
 * ftz_in : subnormal A, B and C inputs are replaced by +0.0 first (Algorithm
 *          "Phi_FTZ-AddMul", FlushSubnormal).
 * ftz_out: after every group's conversion, |d| < 2^-126 becomes zero of the same
 *          sign (Algorithm "FTZ-Add/FTZ-Mul", last line).
 * nan_bits: pattern written for every NaN result (Sec. 4.2; 0x7FFFFFFF on NVIDIA parts).
 *
 * family = MMAEMU_FAMILY_FTZ_ADDMUL selects the other model of the paper, built from binary
 *   operations (Algorithms "FTZ-Add and FTZ-Mul" and "Phi_FTZ-AddMul", Sec. 4.1.1): subnormal
 *   A, B, C inputs become +0.0; every product is RNE-FP32(a b) and every sum RNE-FP32(x + y),
 *   each flushed to a zero of its sign when below 2^-126; every P = group_len (2 or 4)
 *   consecutive products are summed pairwise, and c and the K/P partial sums sequentially.
 *   Only group_len and nan_bits are used; the FDPA fields must hold their defaults
 *   (frac_bits is ignored).  K must be a multiple of P.
 *
 * family = MMAEMU_FAMILY_FMA is Algorithm "Phi_FMA" (Sec. 4.1.2) on FP32 operands and accumulators: d <- c, then
 *   d <- FMA(a_k, b_k, d) for k = 0 .. K - 1 in order, each step the standard fused multiply-add of Algorithm "FMA":
 *   a b + d as if to infinite precision, rounded once to binary32, ties to even; subnormal inputs and results kept;
 *   overflow gives infinity.  The sign of an exact zero is IEEE-754's: +0.0, except that a zero product and a zero
 *   accumulator of the same sign keep that sign.  Special values as in Sec. 4.2 (every NaN result is nan_bits), or with
 *   nan_propagate the payload rule described at that field, applied per step.  With dtypes = (FP64, FP64, FP64, FP64) the
 *   same chain on binary64 (Algorithm "FMA" with F = FP64), the NaN pattern being nan_bits widened as a conversion from
 *   binary32 to binary64 widens a NaN (sign, exponent field all ones, the 23 mantissa bits on top of the 52) and the
 *   quiet bit of the payload rule bit 51.  Uses nan_bits and nan_propagate only;
 *   group_len must be 0 or 1 and every other field must hold its default (frac_bits is ignored).
 *   (The FDPA family with group_len = 1, c_mode = C_AFTER_EXACT and frac_bits wide enough for the whole product, 46
 *   for FP32 operands, computes the same chain except for that sign: there an exact zero is always +0.0.)
 *
 * family = MMAEMU_FAMILY_GST_FDPA is Algorithm "GST-FDPA" (Sec. 4.1.3), through mmaemu_emulate_mma_scaled only, FP4 (E2M1)
 *   operands on both sides: per operation of L = group_len products, every gst_group (G) consecutive products form an
 *   exact dot product p_g; s_g = p_g * SignedSig(alpha) * SignedSig(beta), e_g = Exp(alpha) + Exp(beta) with the
 *   scale factors of the group's block (`block` of the call is K_block, a multiple of G and a divisor of L); the
 *   L / G terms and the accumulator are aligned at their maximum exponent, truncated toward zero to frac_bits
 *   fractional bits and summed; rho as above.  scale_format: E8M0 (significand 1, Exp = code - 127, 0xFF NaN) or
 *   UE4M3, NVFP4's unsigned E4M3 (E4M3 decoding of the low seven bits, 0x7F NaN, the top bit ignored).  A NaN scale
 *   or accumulator gives nan_bits.  Uses group_len, gst_group, frac_bits, out_round, nan_bits, scale_format; every
 *   other field must hold its default.  (Table "GST-FDPA parameter selection": L = 64, G = 16, F = 35, RZ-FP32,
 *   K_block = 32 for MXFP4 and 16 for NVFP4.)  L / G <= 64.
 *
 * Limits: frac_bits <= 40; K <= 2^20; with C_AFTER_EXACT also
 * frac_bits + 2 + ceil(log2 L) <= 56; with the two RD modes frac_bits2, frac_bits_merge
 * and frac_bits_acc <= 48 and max(F, F2, F_m, F_c) + 3 + ceil(log2 L) <= 53.
 */
typedef struct {
    uint32_t struct_size;   /* sizeof(mmaemu_model_params), checked */
    uint32_t group_len;     /* L_max */
    uint32_t frac_bits;     /* F */
    uint32_t align_round;   /* MMAEMU_ALIGN_RZ */
    uint32_t c_mode;
    uint32_t frac_bits2;    /* F2 (the two RD modes); must be 0 in the other modes */
    uint32_t out_round;
    uint32_t out_mant_bits; /* 23 (FP32 output) or 13 (E8M13, RZ only) */
    uint32_t ftz_in, ftz_out;
    uint32_t nan_bits;
    uint32_t split;                  /* MMAEMU_SPLIT_*; C_AFTER_RD only */
    uint32_t acc_special_truncation; /* 0 / 1; C_AFTER_RD only */
    uint32_t frac_bits_merge;        /* F_m; C_AFTER_RD with a split only */
    uint32_t frac_bits_acc;          /* F_c; C_AFTER_RD only */
    uint32_t f2_at_leading_bit;      /* 0 / 1; C_AFTER_RD only */
    uint32_t skip_zero_terms;        /* 0 / 1 */
    uint32_t zero_result_positive;   /* 0 / 1 */
    uint32_t sum_drop_distance;      /* C_AFTER_RD only */
    uint32_t family;                 /* MMAEMU_FAMILY_* */
    uint32_t wide_products;          /* 0 / 1; C_AFTER_RD only */
    uint32_t gst_group;              /* G; MMAEMU_FAMILY_GST_FDPA only */
    uint32_t scale_format;           /* MMAEMU_SCALE_FORMAT_*; MMAEMU_FAMILY_GST_FDPA only */
    uint32_t nan_propagate;          /* 0 / 1.  Variation of the special-value rules (Sec. 4.2) for FP32 operands with an
                                        FP32 accumulator (MMAEMU_FAMILY_FDPA and MMAEMU_FAMILY_FMA; other types:
                                        MMAEMU_ERR_UNSUPPORTED at the call): a NaN result is not the one pattern nan_bits but, in this order of
                                        precedence, the first NaN operand in the order a_0, b_0, a_1, b_1, ... of the
                                        group, made quiet (mantissa bit 22 set, sign and payload kept); else nan_bits
                                        if some product is infinity times zero; else a NaN accumulator, made quiet;
                                        else nan_bits (infinities of both signs).  With group_len = 1 this is a chain
                                        of fused multiply-adds that pass payloads on, which is what the FP32 MFMA
                                        instructions of gfx950 do (they generate 0xFFC00000). */
    uint32_t rd_toward_zero;         /* 0 / 1; C_AFTER_RD modes only.  1: every round-down of the summation's second step
                                        (the product sum at F2 bits, the accumulator at F bits, the merges of a split
                                        group) truncates toward zero instead: the hypothetical instruction of Sec. 6.2.4
                                        whose deviation from the real result is symmetric, against which the bias of the
                                        printed algorithms shows */
} mmaemu_model_params;

typedef struct mmaemu_model mmaemu_model; /* opaque, host memory, owned by the library */

/* Validates *params (host) and creates a model.  *out receives the handle.
 * Errors: INVALID_ARG (NULL, struct_size), UNSUPPORTED (reserved field set, F too large). */
mmaemu_status mmaemu_model_create(const mmaemu_model_params *params, mmaemu_model **out);
/* Frees a model.  NULL is accepted.  No kernel keeps a reference to a model after the
 * enqueueing call has returned. */
mmaemu_status mmaemu_model_destroy(mmaemu_model *model);
mmaemu_status mmaemu_model_get_params(const mmaemu_model *model, mmaemu_model_params *out);

/*
 * D = Phi_model(A, B, C) for `batch` independent m x n x k tiles (paper Eq. 1 / Eq. 3:
 * every d_ij is an independent dot-product-accumulate).  D may alias C; D may not
 * overlap A or B.  Pointers aligned to their element size (the tiled kernels are taken when A and B are
 * 8-byte aligned, 16-byte for TF32).  batch = 0 is a no-op.
 * Errors: SHAPE (m, n or k zero; k > 2^20; k % L != 0; m*n or batch*m*n overflow),
 *         UNSUPPORTED (dtype combination), INVALID_ARG (NULL or misaligned pointer, bad handle), HIP.
 */
mmaemu_status mmaemu_emulate_mma(const mmaemu_model *model, const void *A, const void *B,
                                 const void *C, void *D, uint32_t m, uint32_t n, uint32_t k,
                                 uint64_t batch, mmaemu_dtypes dtypes, void *hip_stream);

/*
 * The same on block-scaled operands (paper Algorithm "ST-FDPA"): SA[batch][m][k / block] and
 * SB[batch][n][k / block] (device, one byte each) hold E8M0 scale factors, value 2^(x - 127), 0xFF = NaN.
 * Every product of block q of a row takes Exp(alpha_q) + Exp(beta_q) on top of its exponent sum, in every
 * accumulation mode of the FDPA family; a NaN scale makes the group's result NaN.  k must be a multiple of
 * block.  (Runs in the tiled kernels when block is a multiple of the group length and the operands are FP8 or
 * FP16, else in the general kernel.)
 * Errors: as mmaemu_emulate_mma; SHAPE (block = 0 or k % block != 0), INVALID_ARG (NULL scales),
 *         UNSUPPORTED (FTZ-AddMul family).
 */
mmaemu_status mmaemu_emulate_mma_scaled(const mmaemu_model *model, const void *A, const void *B,
                                        const void *C, void *D, const void *SA, const void *SB,
                                        uint32_t block, uint32_t m, uint32_t n, uint32_t k,
                                        uint64_t batch, mmaemu_dtypes dtypes, void *hip_stream);

/*
 * Bitwise comparison statistics (paper Eq. 2: Phi(A,B,C) = MMA-Interface(A,B,C) bit for
 * bit; Sec. 3.1 Step 4).  The struct lives in DEVICE memory and is accumulated with
 * atomics, so chunked runs add up.
 *   ulp_hist[0]      ordered-integer distance 0 (equal bits, +0 vs -0, or both NaN)
 *   ulp_hist[i]      distance in [2^(i-1), 2^i), i = 1..32
 *   ulp_hist[33]     exactly one of the two values is NaN
 * Ordered-integer distance: key(b) = b if the sign bit is clear, else -(b & 0x7FFFFFFF);
 * distance = |key(x) - key(y)|.  For FP16 outputs the same on 16-bit patterns (sign bit 0x8000, NaN above 0x7C00;
 * only buckets 0..16 and 33 can fill).  For FP64 outputs the same on 64-bit patterns; ulp_hist[32] then also holds every
 * distance of 2^32 and more, and max_ulp_dist can take all 64 bits.
 */
typedef struct {
    uint64_t n_compared;
    uint64_t n_mismatch_bits;      /* bit patterns differ */
    uint64_t n_mismatch_nan_equiv; /* both NaN, patterns differ (also counted above) */
    uint64_t first_mismatch_index; /* smallest index_base + i with differing bits; UINT64_MAX if none */
    uint64_t max_ulp_dist;         /* over pairs of non-NaN values */
    uint64_t ulp_hist[34];
} mmaemu_stats;

/* Sets *dev_stats to the empty state (all zero, first_mismatch_index = UINT64_MAX). */
mmaemu_status mmaemu_stats_reset(mmaemu_stats *dev_stats, void *hip_stream);
/* Accumulates the comparison of D0[0..count) with D1[0..count): FP32 bit patterns (`d` = MMAEMU_FP32), FP16 bit
 * patterns (`d` = MMAEMU_FP16, the outputs of models run with c = d = FP16) or FP64 bit patterns (`d` = MMAEMU_FP64, the
 * FMA family on binary64); other types: MMAEMU_ERR_UNSUPPORTED.
 * Pointers aligned to the element size.  count = 0 is a no-op. */
mmaemu_status mmaemu_compare(const void *D0, const void *D1, uint64_t count, uint64_t index_base,
                             mmaemu_dtype d, mmaemu_stats *dev_stats, void *hip_stream);

/*
 * The closed loop on several candidate models at once (paper Sec. 3.1 Step 4: a candidate Phi is run on random inputs and
 * compared bit by bit with the interface, Eq. 2; here n_models candidates share one pass over the inputs).  For every
 * model i: D_i = Phi_i(A, B, C) as mmaemu_emulate_mma computes it, compared with the reference as mmaemu_compare does,
 * the result accumulated into dev_stats[i] (device array of n_models structs; first_mismatch_index counts from
 * index_base).  The reference is Dref[batch][m][n] (device, FP32 patterns: typically the native instruction's
 * output), or, when Dref is NULL, the output of models[0] (whose own row then reports no mismatch).
 * D_out: NULL, or device memory for n_models * batch * m * n FP32 patterns; model i's outputs are then also written
 * at D_out + i * batch * m * n.  D_out must not overlap A, B, C or Dref.
 * Models of the FDPA family with frac_bits <= 40 and group length 4, 8, 16 or 32, on 16 x 16 x 16, 16 x 16 x 32,
 * 32 x 32 x 8 or 32 x 32 x 16 tiles with 8-byte aligned A and B of 8- or 16-bit types, run in a kernel that stages and
 * decodes the operands once for up to 16 models (any mix of group lengths and widths) and keeps every output in
 * registers: D reaches memory only on request (on tiles of one group, models that differ only in the output conversion
 * also share the group's sum).  Two families of models run that way, each in launches of its own:
 * c_mode C_IN_GROUP without variation switches (Algorithm "T-FDPA"), and c_mode C_AFTER_RD (Algorithm "TR-FDPA") with
 * any of its variation switches: unsplit groups, groups split in halves or quarters, and the even / odd split of
 * Algorithm "GTR-FDPA" launch apart from each other (split groups on FP8 / FP16 operands only, halves and quarters of
 * at least four terms; sets that keep zero terms out of the maxima launch apart from those that do not, and then also
 * by ftz_in; not: wide_products with BF16 operands).  Any other model runs through
 * mmaemu_emulate_mma and mmaemu_compare and needs D_out, as does a reference taken from models[0] when the models do not
 * all fit one such launch.
 * At most MMAEMU_COMPARE_MANY_MAX models per call.  batch = 0 is a no-op.
 * Errors: as mmaemu_emulate_mma; UNSUPPORTED (FP16 accumulators; D_out needed but NULL), INVALID_ARG (n_models, NULL).
 */
#define MMAEMU_COMPARE_MANY_MAX 64
mmaemu_status mmaemu_emulate_compare_many(const mmaemu_model *const *models, uint32_t n_models, const void *A,
                                          const void *B, const void *C, const void *Dref, void *D_out, uint32_t m,
                                          uint32_t n, uint32_t k, uint64_t batch, mmaemu_dtypes dtypes,
                                          uint64_t index_base, mmaemu_stats *dev_stats, void *hip_stream);

/* Host-side query, for reports and for callers that want one launch per call: class_of_model[i] (host array of
 * n_models) receives a non-negative number that is equal for models which mmaemu_emulate_compare_many runs in common
 * launches on this problem (given 8-byte aligned A and B), or -1 for a model that goes through mmaemu_emulate_mma and
 * mmaemu_compare there. */
mmaemu_status mmaemu_compare_many_classes(const mmaemu_model *const *models, uint32_t n_models, uint32_t m, uint32_t n,
                                          uint32_t k, mmaemu_dtypes dtypes, int32_t *class_of_model);

/*
 * Synthetic operand generation (the input families of Sec. 3.1 Step 4: common
 * distributions and random bit streams).  Counter-based: element g (global index
 * (first_tile + t) * elems_per_tile + e) of operand `operand` owns words
 * g*wpe .. g*wpe + wpe-1 of the stream
 *   word(w) = Philox4x32-10(counter = (lo32(w>>2), hi32(w>>2), operand, 0),
 *                           key = (lo32(seed), hi32(seed)))[w & 3],
 * so any chunk of tiles can be generated independently.  wpe = 2 for FP32 output of
 * UNIFORM_EXP, else 1.
 *   ZERO         all-zero bits
 *   FINITE_BITS  uniform over all finite bit patterns of the format
 *   UNIFORM_EXP  random sign and mantissa; exponent field uniform over exp_lo..exp_hi,
 *                plus the value 0 as one more equally likely choice if exp_zero
 *   RANDOM_BITS  uniform over all bit patterns (NaN and infinities included)
 *   NORMAL       N(0,1) by Box-Muller on word pairs, evaluated in binary64 with a fixed
 *                sequence of +, *, / (bit-reproducible on any IEEE-754 machine),
 *                optionally multiplied by scale_target / max|z| (max over the call's
 *                elements, or per tile), rounded to binary32 then to the output format
 *                (RNE, saturating at the largest finite value)
 *   UNIFORM      uniform on [-1, 1): (word + 0.5) * 2^-31 - 1 in binary64; scaling and casts as NORMAL
 *   NORMAL_OUTLIERS  z + h * 10 * z', with z as NORMAL, z' the same from word stream operand + 256 and
 *                h = 1 where the word of stream operand + 512 is below floor(0.001 * 2^32), else 0
 *                (the DNN-like family N(0,1) + Bernoulli(0.001) N(0,100) of Sec. 3.1 Step 4, variance
 *                100 read as standard deviation 10); scaling and casts as NORMAL
 *   CANCELLING   adversarial sums (Sec. 3.1 Step 4, large condition numbers): an element of even index
 *                is drawn as UNIFORM_EXP; the odd element after it repeats that draw, with the sign
 *                flipped for operand 0 and, for the other operands, the last mantissa bit flipped
 *                where the low 4 bits of the odd element's own word are 0.  With K even and both
 *                operands K-contiguous the products cancel pairwise up to those perturbations.
 *                Not defined for FP32 output.
 *   SIGNED_ZEROS one of eight equally likely values picked by the top three bits of the word: sign = bit 29;
 *                bits 31..30 = 0 or 1: zero, 2: 1.0, 3: the smallest subnormal.  Exact zeros of both signs next to
 *                the values that produce them (sums of zeros, which random streams of wide formats never reach).
 *                Not defined for scale codes.
 */
enum { MMAEMU_GEN_ZERO = 0, MMAEMU_GEN_FINITE_BITS = 1, MMAEMU_GEN_UNIFORM_EXP = 2,
       MMAEMU_GEN_RANDOM_BITS = 3, MMAEMU_GEN_NORMAL = 4, MMAEMU_GEN_UNIFORM = 5,
       MMAEMU_GEN_NORMAL_OUTLIERS = 6, MMAEMU_GEN_CANCELLING = 7, MMAEMU_GEN_SIGNED_ZEROS = 8 };
enum { MMAEMU_SCALE_NONE = 0, MMAEMU_SCALE_TENSOR = 1, MMAEMU_SCALE_TILE = 2,
       MMAEMU_SCALE_FACTOR = 3 /* every value times scale_target itself (Sec. 6.2.4 draws operands from 1000 x N(0,1)) */ };

typedef struct {
    uint32_t struct_size;
    uint32_t family;
    uint64_t seed;
    uint32_t operand;        /* 0 = A, 1 = B, 2 = C: selects the word stream */
    uint32_t exp_lo, exp_hi; /* UNIFORM_EXP, CANCELLING */
    uint32_t exp_zero;       /* UNIFORM_EXP, CANCELLING */
    uint32_t scale_scope;    /* NORMAL, UNIFORM, NORMAL_OUTLIERS */
    double scale_target;     /* those three, with a scale scope */
} mmaemu_gen_params;

/* Writes n_tiles * elems_per_tile elements of type `dtype` to `out`.
 * `workspace`: device memory of at least 8 bytes, 8-byte aligned, needed (and
 * overwritten) only for the value families with MMAEMU_SCALE_TENSOR; may be NULL otherwise.
 * Errors: INVALID_ARG, UNSUPPORTED (exponent range outside the format), SHAPE
 * (elems_per_tile = 0 or total elements >= 2^62). */
mmaemu_status mmaemu_generate(const mmaemu_gen_params *gen, void *out, mmaemu_dtype dtype,
                              uint64_t elems_per_tile, uint64_t first_tile, uint64_t n_tiles,
                              void *workspace, void *hip_stream);

/*
 * mmaemu_generate for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without `workspace`, same output
 * bit for bit.  The eight bytes that per-tensor scaling needs come out of a 256-byte array that is part of the
 * library's image (one copy per GPU, held until the process ends); the call allocates and frees nothing.  At most
 * MMAEMU_GENERATE_NOALLOC_MAX_ELEMS (2^40) elements per call: more is MMAEMU_ERR_SHAPE.  Every call on a GPU uses
 * that GPU's one array, and the call clears what it needs first, so calls that may overlap on one GPU (different
 * streams, no ordering between them) race on it: order them, or use mmaemu_generate with a workspace of their own.
 */
#define MMAEMU_GENERATE_NOALLOC_MAX_ELEMS (1ull << 40)
mmaemu_status mmaemu_generate_noalloc(const mmaemu_gen_params *gen, void *out, mmaemu_dtype dtype,
                                      uint64_t elems_per_tile, uint64_t first_tile, uint64_t n_tiles,
                                      void *hip_stream);

/*
 * Native-instruction probe: the device under test of the closed loop (paper Sec. 3.3:
 * instruction-level MMA interfaces through intrinsics).  Runs one real v_mfma
 * instruction per tile on the same operand layout as mmaemu_emulate_mma:
 * A[batch][M][k], B[batch][N][k], C/D[batch][M][N] (FP32; FP64 for the two binary64 forms, whose pointers must
 * be 8-byte aligned) with M, N and K_native fixed by the instruction; k <= K_native, the missing k positions are
 * fed as zeros.
 */
typedef enum {
    MMAEMU_MFMA_F32_16X16X16_F16 = 0,
    MMAEMU_MFMA_F32_16X16X16_BF16 = 1,
    MMAEMU_MFMA_F32_32X32X8_F16 = 2,
    MMAEMU_MFMA_F32_32X32X8_BF16 = 3,
    MMAEMU_MFMA_F32_16X16X32_F16 = 4,
    MMAEMU_MFMA_F32_16X16X32_BF16 = 5,
    MMAEMU_MFMA_F32_16X16X32_FP8_FP8 = 6, /* A E4M3, B E4M3 */
    MMAEMU_MFMA_F32_16X16X32_FP8_BF8 = 7, /* A E4M3, B E5M2 */
    MMAEMU_MFMA_F32_16X16X32_BF8_FP8 = 8, /* A E5M2, B E4M3 */
    MMAEMU_MFMA_F32_16X16X32_BF8_BF8 = 9, /* A E5M2, B E5M2 */
    /* v_mfma_scale_f32_16x16x128_f8f6f4, only through mmaemu_mfma_probe_scaled: id = BASE + 5 fa + fb with the operand
     * formats fa (A) and fb (B) numbered as the instruction numbers them: 0 E4M3, 1 E5M2, 2 E2M3, 3 E3M2, 4 E2M1 */
    MMAEMU_MFMA_SCALE_F32_16X16X128_F8F6F4_BASE = 10,
    MMAEMU_MFMA_SCALE_F32_16X16X128_FP8_FP8 = 10,
    MMAEMU_MFMA_SCALE_F32_16X16X128_FP8_BF8 = 11,
    MMAEMU_MFMA_SCALE_F32_16X16X128_BF8_FP8 = 15,
    MMAEMU_MFMA_SCALE_F32_16X16X128_BF8_BF8 = 16,
    MMAEMU_MFMA_SCALE_F32_16X16X128_FP4_FP4 = 34,
    MMAEMU_MFMA_F32_32X32X16_F16 = 35,
    MMAEMU_MFMA_F32_32X32X16_BF16 = 36,
    MMAEMU_MFMA_F32_32X32X16_FP8_FP8 = 37,
    MMAEMU_MFMA_F32_32X32X16_FP8_BF8 = 38,
    MMAEMU_MFMA_F32_32X32X16_BF8_FP8 = 39,
    MMAEMU_MFMA_F32_32X32X16_BF8_BF8 = 40,
    /* FP32 operands (the paper's FP32 instructions are chains of FMAs, Sec. 4.1.2) */
    MMAEMU_MFMA_F32_16X16X4_F32 = 41,
    MMAEMU_MFMA_F32_32X32X2_F32 = 42,
    /* v_mfma_scale_f32_32x32x64_f8f6f4, numbered like the 16x16x128 form: id = BASE + 5 fa + fb (43 .. 67) */
    MMAEMU_MFMA_SCALE_F32_32X32X64_F8F6F4_BASE = 43,
    /* multi-block forms: one issue computes 64 / m independent m x m x k products (2, 4 or 16 "blocks").  Through
     * mmaemu_mfma_probe a block is a tile: tiles 0 .. 64/m - 1 go through the first issue, and so on; the blocks of a
     * last, partial issue beyond `batch` are fed zeros and not stored. */
    MMAEMU_MFMA_F32_32X32X4_2B_F16 = 68,
    MMAEMU_MFMA_F32_16X16X4_4B_F16 = 69,
    MMAEMU_MFMA_F32_4X4X4_16B_F16 = 70,
    MMAEMU_MFMA_F32_32X32X4_2B_BF16 = 71, /* the _1k forms (four BF16 values per lane) */
    MMAEMU_MFMA_F32_16X16X4_4B_BF16 = 72,
    MMAEMU_MFMA_F32_4X4X4_16B_BF16 = 73,
    MMAEMU_MFMA_F32_32X32X1_2B_F32 = 74,
    MMAEMU_MFMA_F32_16X16X1_4B_F32 = 75,
    MMAEMU_MFMA_F32_4X4X1_16B_F32 = 76,
    /* binary64 forms (the device under test for Algorithm "Phi_FMA" with F = FP64): A, B, C and D all MMAEMU_FP64 */
    MMAEMU_MFMA_F64_16X16X4_F64 = 77,
    MMAEMU_MFMA_F64_4X4X4_4B_F64 = 78, /* four blocks per issue, a block is a tile as above */
    MMAEMU_MFMA_COUNT = 79
} mmaemu_mfma_instr;

/* Shape and operand types of an instruction (host-side query). */
mmaemu_status mmaemu_mfma_info(mmaemu_mfma_instr instr, uint32_t *m, uint32_t *n, uint32_t *k_native,
                               mmaemu_dtype *a, mmaemu_dtype *b);
mmaemu_status mmaemu_mfma_probe(mmaemu_mfma_instr instr, const void *A, const void *B, const void *C,
                                void *D, uint32_t k, uint64_t batch, void *hip_stream);
/* The block-scaled instructions (device under test for Algorithm "ST-FDPA"): as above with E8M0 scales
 * SA[batch][16][k / 32], SB[batch][16][k / 32]; k a multiple of 32, at most 128. */
mmaemu_status mmaemu_mfma_probe_scaled(mmaemu_mfma_instr instr, const void *A, const void *B, const void *C,
                                       void *D, const void *SA, const void *SB, uint32_t k, uint64_t batch,
                                       void *hip_stream);

/*
 * Error of an emulated D against the exact dot product on a sample (methodology of the
 * paper's Sec. 6.2.4: deviation of a model's output from the real result; here the real
 * result is the exact integer dot product, C = 0).  One m x n output, A[m][k], B[n][k],
 * both FP8; flattened output index i*n + j is sampled when it is a multiple of `stride`.
 * With R = RNE-FP32(exact):
 *   n_equal_rne       D bits == R bits
 *   n_above / n_below ordered key of D greater / less than that of R
 *   ulp_hist          |key(D) - key(R)| bucketed as in mmaemu_stats
 *   sum/max_abs_err   |D - exact| (binary64, accumulation order unspecified)
 *   sum/max_rel_err   |D - exact| / |exact| over samples with exact != 0
 *   sum_signed_err    D - exact
 * Accumulates into *dev_err (device memory).  D must hold no NaN/Inf at sampled places
 * (such samples are skipped and counted in n_skipped).
 */
typedef struct {
    uint64_t n_samples, n_equal_rne, n_above, n_below, n_skipped;
    uint64_t ulp_hist[34];
    double sum_abs_err, max_abs_err, sum_rel_err, max_rel_err, sum_signed_err;
} mmaemu_err_stats;

mmaemu_status mmaemu_err_stats_reset(mmaemu_err_stats *dev_err, void *hip_stream);
mmaemu_status mmaemu_exact_dot_sample(const void *A, const void *B, const void *D, uint32_t m,
                                      uint32_t n, uint32_t k, mmaemu_dtypes dtypes, uint64_t stride,
                                      mmaemu_err_stats *dev_err, void *hip_stream);

/*
 * Distribution of the deviation of a model's (or an instruction's) outputs from the real result (Sec. 6.2.4: the
 * round-down modes of Algorithms "TR-FDPA" / "GTR-FDPA" shift it toward the negative side; with rd_toward_zero it is
 * symmetric).  For `batch` tiles A[batch][m][k], B[batch][n][k], C[batch][m][n] (FP32; NULL means zero) and
 * D[batch][m][n] (FP32), every output whose flattened index (over the whole batch) is a multiple of `stride` is
 * sampled: delta = D - (c + sum_k a_k b_k), the bracket taken exactly (a wide fixed-point sum: delta itself is exact).
 *   n_samples                      samples with finite operands, accumulator and output
 *   n_skipped                      the others (not counted anywhere else)
 *   n_negative / n_zero / n_positive   sign of delta
 *   bins[i]                        delta in [(i - 32) w, (i - 31) w) with w = 2^bin_exp; bins 0 and 63 also take
 *                                  everything below / above the range
 *   sum, sum_abs, sum_sq           of delta, |delta|, delta^2 in binary64 (each delta rounded once; accumulation order
 *                                  unspecified)
 * Accumulates into *dev_hist (device memory, 8-byte aligned; mmaemu_deviation_hist_reset clears it).  Operands of at
 * most 16 bits (FP8, FP6, FP4, FP16, BF16).
 * Errors: INVALID_ARG (NULL, alignment, bin_exp outside -280 .. 250), SHAPE (zero sizes, k > 2^20, stride 0, more than
 * 2^43 samples), UNSUPPORTED (types).
 */
#define MMAEMU_DEVIATION_BINS 64
typedef struct {
    uint64_t n_samples, n_skipped, n_negative, n_zero, n_positive;
    uint64_t bins[MMAEMU_DEVIATION_BINS];
    double sum, sum_abs, sum_sq;
} mmaemu_deviation_hist;

mmaemu_status mmaemu_deviation_hist_reset(mmaemu_deviation_hist *dev_hist, void *hip_stream);
mmaemu_status mmaemu_deviation_sample(const void *A, const void *B, const void *C, const void *D, uint32_t m, uint32_t n,
                                      uint32_t k, uint64_t batch, mmaemu_dtypes dtypes, uint64_t stride, int32_t bin_exp,
                                      mmaemu_deviation_hist *dev_hist, void *hip_stream);

/*
 * Issue-rate probes: the measured counterpart of the vector-ALU peak that the emulation kernels' roofline is quoted
 * against (the path is bound by integer / binary32 vector-ALU issue, not by the matrix cores or HBM).  Probe `op`
 * (0 .. mmaemu_issue_probe_count() - 1, one per instruction the hot loops are made of; mmaemu_issue_probe_name gives
 * its mnemonic, NULL beyond the last) enqueues `workgroups` workgroups of 256 threads that each issue
 * 8 * iterations instances of the instruction per lane in eight independent chains; the caller times the launch
 * (events on the stream) and divides workgroups * 256 * 8 * iterations by the duration.  `out`: 1 KiB of device
 * memory that the probe may write.  Errors: INVALID_ARG (op, out), SHAPE (zero counts).
 */
uint32_t mmaemu_issue_probe_count(void);
const char *mmaemu_issue_probe_name(uint32_t op);
mmaemu_status mmaemu_issue_probe(uint32_t op, uint32_t iterations, uint32_t workgroups, void *out, void *hip_stream);

const char *mmaemu_status_string(mmaemu_status s);
const char *mmaemu_last_error(void); /* thread-local, never NULL */
/* Name of the kernel family the calling thread's last successful mmaemu_emulate_mma
 * enqueued ("general", or "tiled TMxTN kc=.. L=.. c_mode=.."); for tests and reports. */
const char *mmaemu_last_kernel(void);
/* Library version as major*10000 + minor*100 + patch. */
uint32_t mmaemu_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MMAEMU_H */
