// Native-instruction probe: the device under test of the closed loop (paper Sec. 3.3:
// instruction-level MMA interfaces through intrinsics).  One wavefront executes exactly
// one v_mfma instruction per tile; operands go from the tile-major, K-contiguous layout
// of the emulation entry point straight into the instruction's register layout.
//
// Register layouts (wave64), l = lane:
//   (the FP32 instructions 16x16x4 and 32x32x2 hold one element per lane: K/4 = 1, K/2 = 1)
//   16x16xK : A row  i = l % 16, k = (K/4) * (l / 16) + 0 .. K/4-1   (same for B with column j)
//             C/D column j = l % 16, rows i = 4 * (l / 16) + r, r = 0..3
//   32x32xK : A row  i = l % 32, k = (K/2) * (l / 32) + 0 .. K/2-1   (same for B with column j)
//             C/D column j = l % 32, rows i = 8 * (r / 4) + 4 * (l / 32) + r % 4, r = 0..15
// k positions at or beyond the caller's k are fed as zeros.
#include "common.hpp"

namespace mmaemu {

typedef _Float16 v4f16 __attribute__((ext_vector_type(4)));
typedef _Float16 v8f16 __attribute__((ext_vector_type(8)));
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf16 __attribute__((ext_vector_type(8)));
typedef float v4f32 __attribute__((ext_vector_type(4)));
typedef float v16f32 __attribute__((ext_vector_type(16)));

template <int INSTR> struct Instr;
#define DEF_INSTR(ID, M_, N_, K_, EB)                                 \
    template <> struct Instr<ID> {                                    \
        static constexpr int M = M_, N = N_, K = K_, ELEM_BYTES = EB; \
    }
DEF_INSTR(MMAEMU_MFMA_F32_16X16X16_F16, 16, 16, 16, 2);
DEF_INSTR(MMAEMU_MFMA_F32_16X16X16_BF16, 16, 16, 16, 2);
DEF_INSTR(MMAEMU_MFMA_F32_32X32X8_F16, 32, 32, 8, 2);
DEF_INSTR(MMAEMU_MFMA_F32_32X32X8_BF16, 32, 32, 8, 2);
DEF_INSTR(MMAEMU_MFMA_F32_16X16X32_F16, 16, 16, 32, 2);
DEF_INSTR(MMAEMU_MFMA_F32_16X16X32_BF16, 16, 16, 32, 2);
DEF_INSTR(MMAEMU_MFMA_F32_16X16X32_FP8_FP8, 16, 16, 32, 1);
DEF_INSTR(MMAEMU_MFMA_F32_16X16X32_FP8_BF8, 16, 16, 32, 1);
DEF_INSTR(MMAEMU_MFMA_F32_16X16X32_BF8_FP8, 16, 16, 32, 1);
DEF_INSTR(MMAEMU_MFMA_F32_16X16X32_BF8_BF8, 16, 16, 32, 1);
DEF_INSTR(MMAEMU_MFMA_F32_32X32X16_F16, 32, 32, 16, 2);
DEF_INSTR(MMAEMU_MFMA_F32_32X32X16_BF16, 32, 32, 16, 2);
DEF_INSTR(MMAEMU_MFMA_F32_32X32X16_FP8_FP8, 32, 32, 16, 1);
DEF_INSTR(MMAEMU_MFMA_F32_32X32X16_FP8_BF8, 32, 32, 16, 1);
DEF_INSTR(MMAEMU_MFMA_F32_32X32X16_BF8_FP8, 32, 32, 16, 1);
DEF_INSTR(MMAEMU_MFMA_F32_32X32X16_BF8_BF8, 32, 32, 16, 1);
DEF_INSTR(MMAEMU_MFMA_F32_16X16X4_F32, 16, 16, 4, 4);
DEF_INSTR(MMAEMU_MFMA_F32_32X32X2_F32, 32, 32, 2, 4);
#undef DEF_INSTR

// gather this lane's K/4 (16-wide) or 4 (32-wide) consecutive k elements of one row,
// zero beyond the caller's k; returns them packed little-endian in up to 128 bits
template <int NELEM, int EB>
__device__ __forceinline__ void load_row_slice(const uint8_t *row, uint32_t k0, uint32_t k, uint32_t out[4])
{
    out[0] = out[1] = out[2] = out[3] = 0u;
    // the whole slice inside the row and naturally aligned: one load (the bytes land as the loop below packs them)
    constexpr int SLICE = NELEM * EB;
    static_assert(SLICE == 4 || SLICE == 8 || SLICE == 16, "slice of 4, 8 or 16 bytes");
    const uint8_t *p = row + (size_t)k0 * EB;
    if (k0 + NELEM <= k && (reinterpret_cast<uintptr_t>(p) & (SLICE - 1)) == 0) {
        if (SLICE == 16) {
            const uint4 v = *reinterpret_cast<const uint4 *>(p);
            out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
        } else if (SLICE == 8) {
            const uint2 v = *reinterpret_cast<const uint2 *>(p);
            out[0] = v.x; out[1] = v.y;
        } else {
            out[0] = *reinterpret_cast<const uint32_t *>(p);
        }
        return;
    }
#pragma unroll
    for (int q = 0; q < NELEM; ++q) {
        const uint32_t kk = k0 + q;
        uint32_t v = 0;
        if (kk < k) v = (EB == 1) ? row[kk] : (EB == 2 ? reinterpret_cast<const uint16_t *>(row)[kk] : reinterpret_cast<const uint32_t *>(row)[kk]);
        const int bit = q * EB * 8;
        out[bit / 32] |= v << (bit % 32);
    }
}

template <int INSTR>
__global__ void __launch_bounds__(256)
mfma_probe_kernel(const uint8_t *__restrict__ A, const uint8_t *__restrict__ B, const float *C, float *D,
                  uint32_t k, uint64_t batch)
{
    using I = Instr<INSTR>;
    constexpr int KL = (I::M == 16) ? I::K / 4 : I::K / 2;  // k elements per lane
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const uint64_t nwaves = ((uint64_t)gridDim.x * blockDim.x) >> 6;
    for (uint64_t t = wave; t < batch; t += nwaves) {
        const uint32_t rc = lane % I::M;                  // row of A / column of B held by this lane
        const uint32_t k0 = KL * (lane / I::M);
        uint32_t ra[4], rb[4];
        load_row_slice<KL, I::ELEM_BYTES>(A + ((t * I::M + rc) * (uint64_t)k) * I::ELEM_BYTES, k0, k, ra);
        load_row_slice<KL, I::ELEM_BYTES>(B + ((t * I::N + rc) * (uint64_t)k) * I::ELEM_BYTES, k0, k, rb);
        const float *c = C + t * (uint64_t)(I::M * I::N);
        float *d = D + t * (uint64_t)(I::M * I::N);
        if constexpr (I::M == 16) {
            const uint32_t j = lane % 16, i0 = 4 * (lane / 16);
            v4f32 acc;
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = c[(i0 + r) * 16 + j];
            if constexpr (INSTR == MMAEMU_MFMA_F32_16X16X4_F32) {
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(ra[0]), __uint_as_float(rb[0]), acc, 0, 0, 0);
            } else if constexpr (INSTR == MMAEMU_MFMA_F32_16X16X16_F16) {
                v4f16 a, b;
                __builtin_memcpy(&a, ra, 8); __builtin_memcpy(&b, rb, 8);
                acc = __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, acc, 0, 0, 0);
            } else if constexpr (INSTR == MMAEMU_MFMA_F32_16X16X16_BF16) {
                v4i16 a, b;
                __builtin_memcpy(&a, ra, 8); __builtin_memcpy(&b, rb, 8);
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, acc, 0, 0, 0);
            } else if constexpr (INSTR == MMAEMU_MFMA_F32_16X16X32_F16) {
                v8f16 a, b;
                __builtin_memcpy(&a, ra, 16); __builtin_memcpy(&b, rb, 16);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc, 0, 0, 0);
            } else if constexpr (INSTR == MMAEMU_MFMA_F32_16X16X32_BF16) {
                v8bf16 a, b;
                __builtin_memcpy(&a, ra, 16); __builtin_memcpy(&b, rb, 16);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
            } else {
                long a, b;
                __builtin_memcpy(&a, ra, 8); __builtin_memcpy(&b, rb, 8);
                if constexpr (INSTR == MMAEMU_MFMA_F32_16X16X32_FP8_FP8)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a, b, acc, 0, 0, 0);
                else if constexpr (INSTR == MMAEMU_MFMA_F32_16X16X32_FP8_BF8)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_fp8_bf8(a, b, acc, 0, 0, 0);
                else if constexpr (INSTR == MMAEMU_MFMA_F32_16X16X32_BF8_FP8)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf8_fp8(a, b, acc, 0, 0, 0);
                else
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf8_bf8(a, b, acc, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) d[(i0 + r) * 16 + j] = acc[r];
        } else {
            const uint32_t j = lane % 32, ib = 4 * (lane / 32);
            v16f32 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = c[(8 * (r / 4) + ib + r % 4) * 32 + j];
            if constexpr (INSTR == MMAEMU_MFMA_F32_32X32X2_F32) {
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(ra[0]), __uint_as_float(rb[0]), acc, 0, 0, 0);
            } else if constexpr (INSTR == MMAEMU_MFMA_F32_32X32X8_F16) {
                v4f16 a, b;
                __builtin_memcpy(&a, ra, 8); __builtin_memcpy(&b, rb, 8);
                acc = __builtin_amdgcn_mfma_f32_32x32x8f16(a, b, acc, 0, 0, 0);
            } else if constexpr (INSTR == MMAEMU_MFMA_F32_32X32X16_F16) {
                v8f16 a, b;
                __builtin_memcpy(&a, ra, 16); __builtin_memcpy(&b, rb, 16);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
            } else if constexpr (INSTR == MMAEMU_MFMA_F32_32X32X16_BF16) {
                v8bf16 a, b;
                __builtin_memcpy(&a, ra, 16); __builtin_memcpy(&b, rb, 16);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
            } else if constexpr (I::ELEM_BYTES == 1) {
                long a, b;
                __builtin_memcpy(&a, ra, 8); __builtin_memcpy(&b, rb, 8);
                if constexpr (INSTR == MMAEMU_MFMA_F32_32X32X16_FP8_FP8)
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a, b, acc, 0, 0, 0);
                else if constexpr (INSTR == MMAEMU_MFMA_F32_32X32X16_FP8_BF8)
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_fp8_bf8(a, b, acc, 0, 0, 0);
                else if constexpr (INSTR == MMAEMU_MFMA_F32_32X32X16_BF8_FP8)
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf8_fp8(a, b, acc, 0, 0, 0);
                else
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf8_bf8(a, b, acc, 0, 0, 0);
            } else {
                v4i16 a, b;
                __builtin_memcpy(&a, ra, 8); __builtin_memcpy(&b, rb, 8);
                acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a, b, acc, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) d[(8 * (r / 4) + ib + r % 4) * 32 + j] = acc[r];
        }
    }
}

// ---- multi-block forms: one issue computes NB = 64 / M independent M x M x K products; a block is a tile ----------
// Register layout (found from the single-block forms by analogy, then fixed by exact small-integer tests), l = lane:
//   A: row i = l % M of block l / M, its K elements in k order (same for B with column j);
//   C/D register r:  M = 32: block r / 16, row 8 ((r % 16) / 4) + 4 (l / 32) + r % 4, column l % 32;
//                    M = 16: block r / 4,  row 4 (l / 16) + r % 4,                   column l % 16;
//                    M = 4:  block l / 4,  row r,                                     column l % 4.
typedef float v32f32 __attribute__((ext_vector_type(32)));

template <int M, int TYPE>      // TYPE 0: FP16, 1: BF16 (_1k), 2: FP32
__global__ void __launch_bounds__(256)
mfma_multiblock_kernel(const uint8_t *__restrict__ A, const uint8_t *__restrict__ B, const float *C, float *D, uint32_t k, uint64_t batch)
{
    constexpr int NB = 64 / M, KN = TYPE == 2 ? 1 : 4, EB = TYPE == 2 ? 4 : 2, NR = M * M * NB / 64;
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const uint64_t nwaves = ((uint64_t)gridDim.x * blockDim.x) >> 6;
    const uint64_t issues = (batch + NB - 1) / NB;
    for (uint64_t w = wave; w < issues; w += nwaves) {
        const uint64_t t0 = w * NB;
        const uint32_t rc = lane % M;
        const uint64_t ta = t0 + lane / M;                      // the tile whose row of A / column of B this lane holds
        uint32_t ra[4] = {0u, 0u, 0u, 0u}, rb[4] = {0u, 0u, 0u, 0u};
        if (ta < batch) {
            load_row_slice<KN, EB>(A + ((ta * M + rc) * (uint64_t)k) * EB, 0, k, ra);
            load_row_slice<KN, EB>(B + ((ta * M + rc) * (uint64_t)k) * EB, 0, k, rb);
        }
        typedef float vacc __attribute__((ext_vector_type(NR)));
        vacc acc;
        uint64_t tile[NR]; uint32_t off[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            uint32_t bb, ii, jj;
            if (M == 32) { bb = r / 16; ii = 8 * ((r % 16) / 4) + 4 * (lane / 32) + r % 4; jj = lane % 32; }
            else if (M == 16) { bb = r / 4; ii = 4 * (lane / 16) + r % 4; jj = lane % 16; }
            else { bb = lane / 4; ii = r; jj = lane % 4; }
            tile[r] = t0 + bb;
            off[r] = ii * M + jj;
            acc[r] = tile[r] < batch ? C[tile[r] * (uint64_t)(M * M) + off[r]] : 0.0f;
        }
        if constexpr (TYPE == 2) {
            const float a = __uint_as_float(ra[0]), b = __uint_as_float(rb[0]);
            if constexpr (M == 32) acc = __builtin_amdgcn_mfma_f32_32x32x1f32(a, b, acc, 0, 0, 0);
            else if constexpr (M == 16) acc = __builtin_amdgcn_mfma_f32_16x16x1f32(a, b, acc, 0, 0, 0);
            else acc = __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, acc, 0, 0, 0);
        } else if constexpr (TYPE == 0) {
            v4f16 a, b;
            __builtin_memcpy(&a, ra, 8); __builtin_memcpy(&b, rb, 8);
            if constexpr (M == 32) acc = __builtin_amdgcn_mfma_f32_32x32x4f16(a, b, acc, 0, 0, 0);
            else if constexpr (M == 16) acc = __builtin_amdgcn_mfma_f32_16x16x4f16(a, b, acc, 0, 0, 0);
            else acc = __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, acc, 0, 0, 0);
        } else {
            v4i16 a, b;
            __builtin_memcpy(&a, ra, 8); __builtin_memcpy(&b, rb, 8);
            if constexpr (M == 32) acc = __builtin_amdgcn_mfma_f32_32x32x4bf16_1k(a, b, acc, 0, 0, 0);
            else if constexpr (M == 16) acc = __builtin_amdgcn_mfma_f32_16x16x4bf16_1k(a, b, acc, 0, 0, 0);
            else acc = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, b, acc, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < NR; ++r)
            if (tile[r] < batch) D[tile[r] * (uint64_t)(M * M) + off[r]] = acc[r];
    }
}

// ---- binary64 forms ----------------------------------------------------------------------------------------------------
// Register layout (one-hot operands on raw registers, then fixed by exact small-integer tests), l = lane:
//   16x16x4:    A row i = l % 16, k = l / 16 (same for B with column j); C/D register r: row 4 r + l / 16, column l % 16
//               (the rows of a lane are 4 apart, where the binary32 forms hold 4 consecutive rows)
//   4x4x4_4b:   A row i = l % 4 of block (l / 4) % 4, k = l / 16 (same for B); C/D: block (l / 4) % 4, row l / 16, column l % 4
typedef double v4f64 __attribute__((ext_vector_type(4)));

template <int M>
__global__ void __launch_bounds__(256)
mfma_f64_kernel(const double *__restrict__ A, const double *__restrict__ B, const double *C, double *D, uint32_t k, uint64_t batch)
{
    constexpr int NB = M == 16 ? 1 : 4;
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const uint64_t nwaves = ((uint64_t)gridDim.x * blockDim.x) >> 6;
    const uint64_t issues = (batch + NB - 1) / NB;
    for (uint64_t w = wave; w < issues; w += nwaves) {
        const uint32_t kk = lane / 16u;
        if constexpr (M == 16) {
            const uint32_t rc = lane % 16u;
            const double a = kk < k ? A[(w * 16 + rc) * (uint64_t)k + kk] : 0.0;
            const double b = kk < k ? B[(w * 16 + rc) * (uint64_t)k + kk] : 0.0;
            const double *c = C + w * 256u;
            double *d = D + w * 256u;
            v4f64 acc;
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = c[(4 * r + kk) * 16 + rc];
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) d[(4 * r + kk) * 16 + rc] = acc[r];
        } else {
            const uint64_t t = w * 4 + (lane / 4u) % 4u;
            const uint32_t rc = lane % 4u;
            const bool live = t < batch;
            const double a = live && kk < k ? A[(t * 4 + rc) * (uint64_t)k + kk] : 0.0;
            const double b = live && kk < k ? B[(t * 4 + rc) * (uint64_t)k + kk] : 0.0;
            double acc = live ? C[t * 16u + kk * 4u + rc] : 0.0;
            acc = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc, 0, 0, 0);
            if (live) D[t * 16u + kk * 4u + rc] = acc;
        }
    }
}

template <int M>
static mmaemu_status launch_f64(const void *A, const void *B, const void *C, void *D, uint32_t k, uint64_t batch, hipStream_t s)
{
    const uint64_t issues = M == 16 ? batch : (batch + 3) / 4;
    uint64_t blocks = (issues + 3) / 4;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL((mfma_f64_kernel<M>), dim3((uint32_t)blocks), dim3(256), 0, s, (const double *)A, (const double *)B,
                       (const double *)C, (double *)D, k, batch);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

template <int M, int TYPE>
static mmaemu_status launch_mb(const void *A, const void *B, const void *C, void *D, uint32_t k, uint64_t batch, hipStream_t s)
{
    const uint64_t issues = (batch + 64 / M - 1) / (64 / M);
    uint64_t blocks = (issues + 3) / 4;                  // 4 wavefronts (issues) per workgroup
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL((mfma_multiblock_kernel<M, TYPE>), dim3((uint32_t)blocks), dim3(256), 0, s, (const uint8_t *)A,
                       (const uint8_t *)B, (const float *)C, (float *)D, k, batch);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

template <int INSTR>
static mmaemu_status launch_i(const void *A, const void *B, const void *C, void *D, uint32_t k, uint64_t batch,
                              hipStream_t s)
{
    uint64_t blocks = (batch + 3) / 4;                   // 4 wavefronts (tiles) per workgroup
    if (blocks > 256 * 64) blocks = 256 * 64;            // wave-stride beyond that
    hipLaunchKernelGGL((mfma_probe_kernel<INSTR>), dim3((uint32_t)blocks), dim3(256), 0, s, (const uint8_t *)A,
                       (const uint8_t *)B, (const float *)C, (float *)D, k, batch);
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

mmaemu_status launch_mfma_probe(uint32_t instr, const void *A, const void *B, const void *C, void *D,
                                uint32_t k, uint64_t batch, hipStream_t s)
{
    switch (instr) {
#define CASE(ID) case ID: return launch_i<ID>(A, B, C, D, k, batch, s)
        CASE(MMAEMU_MFMA_F32_16X16X16_F16);
        CASE(MMAEMU_MFMA_F32_16X16X16_BF16);
        CASE(MMAEMU_MFMA_F32_32X32X8_F16);
        CASE(MMAEMU_MFMA_F32_32X32X8_BF16);
        CASE(MMAEMU_MFMA_F32_16X16X32_F16);
        CASE(MMAEMU_MFMA_F32_16X16X32_BF16);
        CASE(MMAEMU_MFMA_F32_16X16X32_FP8_FP8);
        CASE(MMAEMU_MFMA_F32_16X16X32_FP8_BF8);
        CASE(MMAEMU_MFMA_F32_16X16X32_BF8_FP8);
        CASE(MMAEMU_MFMA_F32_16X16X32_BF8_BF8);
        CASE(MMAEMU_MFMA_F32_32X32X16_F16);
        CASE(MMAEMU_MFMA_F32_32X32X16_BF16);
        CASE(MMAEMU_MFMA_F32_32X32X16_FP8_FP8);
        CASE(MMAEMU_MFMA_F32_32X32X16_FP8_BF8);
        CASE(MMAEMU_MFMA_F32_32X32X16_BF8_FP8);
        CASE(MMAEMU_MFMA_F32_32X32X16_BF8_BF8);
        CASE(MMAEMU_MFMA_F32_16X16X4_F32);
        CASE(MMAEMU_MFMA_F32_32X32X2_F32);
#undef CASE
    case MMAEMU_MFMA_F32_32X32X4_2B_F16: return launch_mb<32, 0>(A, B, C, D, k, batch, s);
    case MMAEMU_MFMA_F32_16X16X4_4B_F16: return launch_mb<16, 0>(A, B, C, D, k, batch, s);
    case MMAEMU_MFMA_F32_4X4X4_16B_F16: return launch_mb<4, 0>(A, B, C, D, k, batch, s);
    case MMAEMU_MFMA_F32_32X32X4_2B_BF16: return launch_mb<32, 1>(A, B, C, D, k, batch, s);
    case MMAEMU_MFMA_F32_16X16X4_4B_BF16: return launch_mb<16, 1>(A, B, C, D, k, batch, s);
    case MMAEMU_MFMA_F32_4X4X4_16B_BF16: return launch_mb<4, 1>(A, B, C, D, k, batch, s);
    case MMAEMU_MFMA_F32_32X32X1_2B_F32: return launch_mb<32, 2>(A, B, C, D, k, batch, s);
    case MMAEMU_MFMA_F32_16X16X1_4B_F32: return launch_mb<16, 2>(A, B, C, D, k, batch, s);
    case MMAEMU_MFMA_F32_4X4X1_16B_F32: return launch_mb<4, 2>(A, B, C, D, k, batch, s);
    case MMAEMU_MFMA_F64_16X16X4_F64: return launch_f64<16>(A, B, C, D, k, batch, s);
    case MMAEMU_MFMA_F64_4X4X4_4B_F64: return launch_f64<4>(A, B, C, D, k, batch, s);
    default:
        set_error("unknown mfma instruction %u", instr);
        return MMAEMU_ERR_INVALID_ARG;
    }
}

} // namespace mmaemu
