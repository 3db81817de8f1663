// Native-instruction probe for the block-scaled MFMAs of gfx950, v_mfma_scale_f32_16x16x128_f8f6f4 and
// v_mfma_scale_f32_32x32x64_f8f6f4, with every pairing of their operand formats (FP8 E4M3, BF8 E5M2, FP6 E2M3, BF6 E3M2,
// FP4 E2M1): the device under test for Algorithm "ST-FDPA" (paper Sec. 4.1.3).  One wavefront issues exactly one
// instruction per tile.
//
// Register layout (wave64), l = lane, M = 16 or 32, g = l / M; found with one-hot operands and distinct scales on raw
// registers, then fixed by exact small-integer tests.  Row (A) or column (B) l % M in every format.
//   8-bit formats: dwords 0..3 hold k = 16 g + 0..15 and dwords 4..7 hold k = K/2 + 16 g + 0..15, bytes in k order
//     (K = 128 for M = 16, 64 for M = 32);
//   6-bit and 4-bit formats: the lane holds k = 32 g + 0..31, codes packed back to back from bit 0 (six dwords for
//     FP6, four for FP4; the remaining dwords are ignored);
//   scales: the scale operand of lane l carries, in its byte 0, the E8M0 code of row l % M and block k = 32 g .. 32 g + 31;
//   C/D: as the unscaled instructions of the same shape (16x16: column l % 16, rows 4 g + r; 32x32: column l % 32,
//     rows 8 (r / 4) + 4 g + r % 4).
// In memory FP6 / FP4 codes sit one per byte.  k positions at or beyond the caller's k are fed as zeros with scale 2^0.
#include "common.hpp"

namespace mmaemu {

typedef int v8i32 __attribute__((ext_vector_type(8)));
typedef float v4f32s __attribute__((ext_vector_type(4)));
typedef float v16f32s __attribute__((ext_vector_type(16)));

// operand registers of one lane from a row of one-code-per-byte elements; FMT as the instruction numbers the formats
template <int FMT, int M>
__device__ __forceinline__ v8i32 load_operand(const uint8_t *row, uint32_t k, uint32_t g)
{
    v8i32 r;
#pragma unroll
    for (int q = 0; q < 8; ++q) r[q] = 0;
    if (FMT <= 1) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t k0 = (M == 16 ? 64 : 32) * h + 16 * g;
            if (k0 < k) {        // k is a multiple of 32, so the sixteen positions are inside together
                const uint32_t *p = reinterpret_cast<const uint32_t *>(row + k0);
#pragma unroll
                for (int q = 0; q < 4; ++q) r[4 * h + q] = (int)p[q];
            }
        }
    } else if (32 * g < k) {
        constexpr int BITS = FMT == 4 ? 4 : 6;
        constexpr uint32_t MASK = (1u << BITS) - 1u;
        const uint32_t *p = reinterpret_cast<const uint32_t *>(row + 32 * g);
        uint32_t regs[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 32; ++e) {
            const uint32_t code = (p[e / 4] >> (8 * (e % 4))) & MASK;
            const int bit = e * BITS, w = bit / 32, o = bit % 32;
            regs[w] |= code << o;
            if (o + BITS > 32) regs[w + 1] |= code >> (32 - o);
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) r[q] = (int)regs[q];
    }
    return r;
}

template <int FA, int FB, int M>
__global__ void __launch_bounds__(256)
mfma_scaled_probe_kernel(const uint8_t *__restrict__ A, const uint8_t *__restrict__ B, const float *C, float *D,
                         const uint8_t *__restrict__ SA, const uint8_t *__restrict__ SB, uint32_t k, uint64_t batch)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const uint64_t nwaves = ((uint64_t)gridDim.x * blockDim.x) >> 6;
    const uint32_t nblk = k / 32;
    for (uint64_t t = wave; t < batch; t += nwaves) {
        const uint32_t rc = lane % M, blk = lane / M;
        const v8i32 a = load_operand<FA, M>(A + (t * M + rc) * (uint64_t)k, k, blk);
        const v8i32 b = load_operand<FB, M>(B + (t * M + rc) * (uint64_t)k, k, blk);
        int sa = 127, sb = 127;
        if (blk < nblk) {
            sa = SA[(t * M + rc) * (uint64_t)nblk + blk];
            sb = SB[(t * M + rc) * (uint64_t)nblk + blk];
        }
        const float *c = C + t * (M * M);
        float *d = D + t * (M * M);
        if constexpr (M == 16) {
            const uint32_t j = lane % 16, i0 = 4 * (lane / 16);
            v4f32s acc;
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = c[(i0 + r) * 16 + j];
            acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc, FA, FB, 0, sa, 0, sb);
#pragma unroll
            for (int r = 0; r < 4; ++r) d[(i0 + r) * 16 + j] = acc[r];
        } else {
            const uint32_t j = lane % 32, ib = 4 * (lane / 32);
            v16f32s acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = c[(8 * (r / 4) + ib + r % 4) * 32 + j];
            acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc, FA, FB, 0, sa, 0, sb);
#pragma unroll
            for (int r = 0; r < 16; ++r) d[(8 * (r / 4) + ib + r % 4) * 32 + j] = acc[r];
        }
    }
}

template <int FA, int FB, int M>
static mmaemu_status launch_f(const void *A, const void *B, const void *C, void *D, const void *SA, const void *SB,
                              uint32_t k, uint64_t batch, hipStream_t s)
{
    uint64_t blocks = (batch + 3) / 4;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL((mfma_scaled_probe_kernel<FA, FB, M>), dim3((uint32_t)blocks), dim3(256), 0, s, (const uint8_t *)A,
                       (const uint8_t *)B, (const float *)C, (float *)D, (const uint8_t *)SA, (const uint8_t *)SB, k, batch);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

template <int M>
static mmaemu_status launch_m(uint32_t q, const void *A, const void *B, const void *C, void *D, const void *SA, const void *SB,
                              uint32_t k, uint64_t batch, hipStream_t s)
{
#define MMAEMU_ROW(X)                                                                                      \
    case 5 * X + 0: return launch_f<X, 0, M>(A, B, C, D, SA, SB, k, batch, s);                             \
    case 5 * X + 1: return launch_f<X, 1, M>(A, B, C, D, SA, SB, k, batch, s);                             \
    case 5 * X + 2: return launch_f<X, 2, M>(A, B, C, D, SA, SB, k, batch, s);                             \
    case 5 * X + 3: return launch_f<X, 3, M>(A, B, C, D, SA, SB, k, batch, s);                             \
    case 5 * X + 4: return launch_f<X, 4, M>(A, B, C, D, SA, SB, k, batch, s)
    switch (q) {
        MMAEMU_ROW(0); MMAEMU_ROW(1); MMAEMU_ROW(2); MMAEMU_ROW(3); MMAEMU_ROW(4);
    default:
        set_error("unknown scaled mfma instruction");
        return MMAEMU_ERR_INVALID_ARG;
    }
#undef MMAEMU_ROW
}

mmaemu_status launch_mfma_probe_scaled(uint32_t instr, const void *A, const void *B, const void *C, void *D,
                                       const void *SA, const void *SB, uint32_t k, uint64_t batch, hipStream_t s)
{
    if (instr >= MMAEMU_MFMA_SCALE_F32_32X32X64_F8F6F4_BASE)
        return launch_m<32>(instr - MMAEMU_MFMA_SCALE_F32_32X32X64_F8F6F4_BASE, A, B, C, D, SA, SB, k, batch, s);
    return launch_m<16>(instr - MMAEMU_MFMA_SCALE_F32_16X16X128_F8F6F4_BASE, A, B, C, D, SA, SB, k, batch, s);
}

} // namespace mmaemu
