// Native-instruction probe for the block-scaled MFMA of gfx950, v_mfma_scale_f32_16x16x128_f8f6f4 with FP8 (E4M3)
// or BF8 (E5M2) operands: the device under test for Algorithm "ST-FDPA" (paper Sec. 4.1.3).  One wavefront issues
// exactly one instruction per tile.
//
// Register layout (wave64), l = lane, g = l / 16, found with one-hot operands and distinct scales: A row i = l % 16;
// dwords 0..3 hold k = 16 g + 0..15 and dwords 4..7 hold k = 64 + 16 g + 0..15, bytes in k order (same for B with
// column j); the scale operand of lane l carries, in its byte 0, the E8M0 scale of row l % 16 and of the block
// k = 32 g .. 32 g + 31; C/D column j = l % 16, rows i = 4 g + r, r = 0..3.  k positions at or beyond the caller's k
// are fed as zeros with scale 2^0.
#include "common.hpp"

namespace mmaemu {

typedef int v8i32 __attribute__((ext_vector_type(8)));
typedef float v4f32s __attribute__((ext_vector_type(4)));

template <int FA, int FB>          // operand formats as the instruction encodes them: 0 = E4M3, 1 = E5M2
__global__ void __launch_bounds__(256)
mfma_scaled_probe_kernel(const uint8_t *__restrict__ A, const uint8_t *__restrict__ B, const float *C, float *D,
                         const uint8_t *__restrict__ SA, const uint8_t *__restrict__ SB, uint32_t k, uint64_t batch)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const uint64_t nwaves = ((uint64_t)gridDim.x * blockDim.x) >> 6;
    const uint32_t nblk = k / 32;
    for (uint64_t t = wave; t < batch; t += nwaves) {
        const uint32_t rc = lane % 16, blk = lane / 16;
        v8i32 a, b;
        int sa = 127, sb = 127;
#pragma unroll
        for (int q = 0; q < 8; ++q) { a[q] = 0; b[q] = 0; }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t k0 = 64 * h + 16 * blk;
            if (k0 < k) {        // k is a multiple of 32, so the sixteen positions are inside together
                const uint32_t *pa = reinterpret_cast<const uint32_t *>(A + (t * 16 + rc) * (uint64_t)k + k0);
                const uint32_t *pb = reinterpret_cast<const uint32_t *>(B + (t * 16 + rc) * (uint64_t)k + k0);
#pragma unroll
                for (int q = 0; q < 4; ++q) { a[4 * h + q] = (int)pa[q]; b[4 * h + q] = (int)pb[q]; }
            }
        }
        if (blk < nblk) {
            sa = SA[(t * 16 + rc) * (uint64_t)nblk + blk];
            sb = SB[(t * 16 + rc) * (uint64_t)nblk + blk];
        }
        const float *c = C + t * 256;
        float *d = D + t * 256;
        const uint32_t j = lane % 16, i0 = 4 * (lane / 16);
        v4f32s acc;
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[r] = c[(i0 + r) * 16 + j];
        acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc, FA, FB, 0, sa, 0, sb);
#pragma unroll
        for (int r = 0; r < 4; ++r) d[(i0 + r) * 16 + j] = acc[r];
    }
}

template <int FA, int FB>
static mmaemu_status launch_f(const void *A, const void *B, const void *C, void *D, const void *SA, const void *SB,
                              uint32_t k, uint64_t batch, hipStream_t s)
{
    uint64_t blocks = (batch + 3) / 4;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL((mfma_scaled_probe_kernel<FA, FB>), dim3((uint32_t)blocks), dim3(256), 0, s, (const uint8_t *)A,
                       (const uint8_t *)B, (const float *)C, (float *)D, (const uint8_t *)SA, (const uint8_t *)SB, k, batch);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

mmaemu_status launch_mfma_probe_scaled(uint32_t instr, const void *A, const void *B, const void *C, void *D,
                                       const void *SA, const void *SB, uint32_t k, uint64_t batch, hipStream_t s)
{
    switch (instr) {
    case MMAEMU_MFMA_SCALE_F32_16X16X128_FP8_FP8: return launch_f<0, 0>(A, B, C, D, SA, SB, k, batch, s);
    case MMAEMU_MFMA_SCALE_F32_16X16X128_FP8_BF8: return launch_f<0, 1>(A, B, C, D, SA, SB, k, batch, s);
    case MMAEMU_MFMA_SCALE_F32_16X16X128_BF8_FP8: return launch_f<1, 0>(A, B, C, D, SA, SB, k, batch, s);
    case MMAEMU_MFMA_SCALE_F32_16X16X128_BF8_BF8: return launch_f<1, 1>(A, B, C, D, SA, SB, k, batch, s);
    default:
        set_error("unknown scaled mfma instruction %u", instr);
        return MMAEMU_ERR_INVALID_ARG;
    }
}

} // namespace mmaemu
