// Algorithm "E-FDPA" (the exact sum of a group's products and the accumulator, converted once) with operand sharing: a
// workgroup owns a 16 x 16 block of D, one output per thread; the rows of A and B that the block needs are decoded once,
// into LDS, as binary64 values (32 values of k at a time).
//
// A thread keeps the exact sum as an unevaluated pair of binary64 numbers (efdpa_pair.hpp); a group whose sum does not stay
// exact there (BF16 or TF32 operands spread over hundreds of binary places) is run again by the integer routine with its
// 640-bit accumulator.  That routine costs the kernel which contains it 100 registers against 58, and with them half of
// its waves, so where D is not C it sits in a kernel of its own: the block kernel leaves a mark in D (a NaN pattern that
// no result has) at each output it could not finish, and a second launch runs those outputs' chains from C again.
// Shapes that are not whole blocks, and FP32 operands, take the same two launches with one thread per output and the
// operands read from memory.
#include "efdpa_pair.hpp"

namespace mmaemu {

constexpr int EKC = 32;                       // values of k staged at a time

// MARK: leave `mark` in D where a group's sum left the pair's reach, instead of running the integer routine here
template <bool MARK>
__global__ void __launch_bounds__(256)
emulate_efdpa_blocks_kernel(ModelArgs p, uint32_t ta, uint32_t tb, const void *__restrict__ A, const void *__restrict__ B, const uint32_t *C,
                            uint32_t *D, uint32_t m, uint32_t n, uint32_t k, uint64_t nblocks, uint32_t mark)
{
    constexpr int VS = EKC + 2;               // row stride in doubles: rows spread over the banks, pairs stay 16-byte aligned
    __shared__ __attribute__((aligned(16))) double As[16][VS];
    __shared__ __attribute__((aligned(16))) double Bs[16][VS];
    const uint32_t tid = threadIdx.x, i = tid / 16u, j = tid % 16u;
    const uint32_t bpr = n / 16u, bpt = (m / 16u) * bpr;
    const uint32_t esa = elem_bytes(ta), esb = elem_bytes(tb);
    const uint32_t L = p.L;
    for (uint64_t w = blockIdx.x; w < nblocks; w += gridDim.x) {
        const uint64_t t = w / bpt;
        const uint32_t r = (uint32_t)(w - t * bpt), bi = r / bpr, bj = r - bi * bpr;
        const uint64_t arow0 = t * m + 16u * bi, brow0 = t * n + 16u * bj;          // first row of the block in A and in B
        const uint64_t o = (arow0 + i) * (uint64_t)n + 16u * bj + j;
        uint32_t d = C[o];
        bool marked = false;
        uint32_t into = 0;                                 // terms of the current group already added
        ExactPair sum;
        sum.start(0u);
        for (uint32_t k0 = 0; k0 < k; k0 += EKC) {
            const uint32_t kc = k - k0 < (uint32_t)EKC ? k - k0 : (uint32_t)EKC;
            __syncthreads();                               // (the previous chunk's readers)
            // (thread (i, j) stages columns j and j + 16 of row i of both operands)
            for (uint32_t kk = j; kk < kc; kk += 16u) {
                As[i][kk] = elem_value(ta, elem_bits(ta, esa, A, (arow0 + i) * (uint64_t)k + k0 + kk), p.ftz_in);
                Bs[i][kk] = elem_value(tb, elem_bits(tb, esb, B, (brow0 + i) * (uint64_t)k + k0 + kk), p.ftz_in);
            }
            __syncthreads();
            // the groups (or the part of a longer group) inside this chunk: a group of at most 32 terms starts and ends
            // here (L divides 32, k0 and k, so it divides kc), a longer one is made of whole chunks
            const uint32_t glen = L < kc ? L : kc;
            for (uint32_t g0 = 0; g0 < kc; g0 += glen) {
                if (into == 0) {
                    // a group starts: the accumulator (flushed if the model flushes inputs) is its first term
                    sum.start((p.ftz_in && (d & 0x7F800000u) == 0) ? 0u : d);
                }
                into += glen;
                if (glen % 2 == 0) {
                    // (g0 is even then: pairs of k come with one 128-bit LDS read per row)
#pragma unroll 2
                    for (uint32_t kk = g0; kk < g0 + glen; kk += 2) {
                        const double2 x = *reinterpret_cast<const double2 *>(&As[i][kk]), y = *reinterpret_cast<const double2 *>(&Bs[j][kk]);
                        sum.add(x.x, y.x);
                        sum.add(x.y, y.y);
                    }
                } else {
                    for (uint32_t kk = g0; kk < g0 + glen; ++kk) sum.add(As[i][kk], Bs[j][kk]);
                }
                if (into == L) {
                    // the group ends
                    into = 0;
                    uint32_t out;
                    if (!sum.finish(p, out)) {
                        // the sum left the pair's reach: the integer routine, from the operands in memory
                        if constexpr (MARK) {
                            marked = true;                 // (in the second launch; what this chain gives from here on is not used)
                            out = 0u;
                        } else {
                            const uint32_t gk = k0 + g0 + glen - L;
                            const uint8_t *ap = static_cast<const uint8_t *>(A) + ((arow0 + i) * (uint64_t)k + gk) * esa;
                            const uint8_t *bp = static_cast<const uint8_t *>(B) + ((brow0 + j) * (uint64_t)k + gk) * esb;
                            out = fdpa_group<true>(p, dyn_fmt(ta), dyn_fmt(tb), ap, bp, L, d, no_scales());
                        }
                    }
                    d = out;
                }
            }
        }
        D[o] = marked ? mark : d;
    }
}

// Any shape, one thread per output: the pair alone, a mark where it does not hold a group's sum.
__global__ void __launch_bounds__(256)
emulate_efdpa_pairs_kernel(ModelArgs p, uint32_t ta, uint32_t tb, const void *__restrict__ A, const void *__restrict__ B,
                           const uint32_t *__restrict__ C, uint32_t *__restrict__ D, uint32_t m, uint32_t n, uint32_t k, uint64_t total,
                           uint32_t mark)
{
    const uint64_t mn = (uint64_t)m * n;
    const uint32_t esa = elem_bytes(ta), esb = elem_bytes(tb);
    for (uint64_t o = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total; o += (uint64_t)gridDim.x * blockDim.x) {
        // (a 64-bit division costs about as much as four terms: 32-bit arithmetic where the output index allows it)
        const uint64_t t = (total >> 32) == 0 ? (uint64_t)((uint32_t)o / (uint32_t)mn) : o / mn;
        const uint32_t r = (uint32_t)(o - t * mn), i = r / n, j = r - i * n;
        const uint64_t a0 = (t * m + i) * (uint64_t)k, b0 = (t * n + j) * (uint64_t)k;
        uint32_t d = C[o];
        bool marked = false;
        for (uint32_t k0 = 0; k0 < k && !marked; k0 += p.L) {
            ExactPair sum;
            sum.start((p.ftz_in && (d & 0x7F800000u) == 0) ? 0u : d);
            uint32_t kk = k0;
            for (; kk + 4 <= k0 + p.L; kk += 4) {
                // (four elements of each row fetched, then decoded behind one branch on the type)
                uint32_t ra[4], rb[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) { ra[q] = elem_bits(ta, esa, A, a0 + kk + q); rb[q] = elem_bits(tb, esb, B, b0 + kk + q); }
                double xa[4], xb[4];
                elem_values(ta, ra, p.ftz_in, xa);
                elem_values(tb, rb, p.ftz_in, xb);
#pragma unroll
                for (int q = 0; q < 4; ++q) sum.add(xa[q], xb[q]);
            }
            for (; kk < k0 + p.L; ++kk) sum.add(elem_value(ta, elem_bits(ta, esa, A, a0 + kk), p.ftz_in), elem_value(tb, elem_bits(tb, esb, B, b0 + kk), p.ftz_in));
            marked = !sum.finish(p, d);
        }
        D[o] = marked ? mark : d;
    }
}

// The second launch: every output that carries the mark, from its accumulator in C, through the integer routine.
__global__ void __launch_bounds__(256)
emulate_efdpa_marked_kernel(ModelArgs p, uint32_t ta, uint32_t tb, const void *__restrict__ A, const void *__restrict__ B,
                            const uint32_t *__restrict__ C, uint32_t *D, uint32_t m, uint32_t n, uint32_t k, uint64_t total, uint32_t mark)
{
    const uint32_t esa = elem_bytes(ta), esb = elem_bytes(tb);
    const uint64_t mn = (uint64_t)m * n;
    for (uint64_t o = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total; o += (uint64_t)gridDim.x * blockDim.x) {
        if (D[o] != mark) continue;
        const uint64_t t = o / mn;
        const uint32_t r = (uint32_t)(o - t * mn), i = r / n, j = r - i * n;
        const uint8_t *ap = static_cast<const uint8_t *>(A) + (t * m + i) * (uint64_t)k * esa;
        const uint8_t *bp = static_cast<const uint8_t *>(B) + (t * n + j) * (uint64_t)k * esb;
        uint32_t d = C[o];
        if (ta == MMAEMU_FP32) {           // (pairs with itself; the run-time format table has no 32-bit significands)
            for (uint32_t k0 = 0; k0 < k; k0 += p.L)
                d = fdpa_group<true>(p, StaticFmt<MMAEMU_FP32>{}, StaticFmt<MMAEMU_FP32>{}, ap + (uint64_t)k0 * 4u, bp + (uint64_t)k0 * 4u, p.L, d, no_scales());
        } else {
            for (uint32_t k0 = 0; k0 < k; k0 += p.L)
                d = fdpa_group<true>(p, dyn_fmt(ta), dyn_fmt(tb), ap + (uint64_t)k0 * esa, bp + (uint64_t)k0 * esb, p.L, d, no_scales());
        }
        D[o] = d;
    }
}

// Whether the kernel takes the problem: whole 16 x 16 blocks, operands of at most 24 significant bits other than FP32
// words, and groups that either lie inside a staged chunk of 32 (L = 1, 2, 4, 8, 16, 32) or are made of whole chunks.
bool efdpa_blocks_take(const ModelArgs &p, uint32_t ta, uint32_t tb, uint32_t m, uint32_t n, uint32_t k)
{
    if (p.c_mode != MMAEMU_C_EXACT || (p.flags & (FL_ACC16 | FL_NAN_PROPAGATE))) return false;
    if (ta == MMAEMU_FP32 || tb == MMAEMU_FP32) return false;
    if (m % 16 != 0 || n % 16 != 0 || p.L == 0 || k == 0 || k % p.L != 0) return false;    // (k > 0: every output is a group's result, so none is the mark)
    return (p.L <= (uint32_t)EKC && EKC % p.L == 0) || p.L % EKC == 0;
}

// Whether the pair of launches for any shape takes the problem: D apart from C (the second launch reads C), k > 0 (every
// output is then a group's result, so none is the mark).
bool efdpa_pairs_take(const ModelArgs &p, const void *C, const void *D, uint32_t k)
{
    return p.c_mode == MMAEMU_C_EXACT && !(p.flags & (FL_ACC16 | FL_NAN_PROPAGATE)) && C != D && p.L != 0 && k != 0 && k % p.L == 0;
}

static uint32_t efdpa_mark(const ModelArgs &p)
{
    // a NaN pattern other than the model's: results are never NaN except as that one
    return p.nan_bits == 0x7FEDCBA9u ? 0x7FEDCBA8u : 0x7FEDCBA9u;
}

static mmaemu_status launch_marked(const ModelArgs &p, const void *A, const void *B, const void *C, void *D, uint32_t m, uint32_t n, uint32_t k,
                                   uint64_t batch, uint32_t ta, uint32_t tb, hipStream_t s)
{
    const uint64_t total = batch * m * n;
    uint64_t blocks = (total + 255) / 256;
    if (blocks > (1ull << 20)) blocks = 1ull << 20;
    hipLaunchKernelGGL(emulate_efdpa_marked_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, p, ta, tb, A, B, (const uint32_t *)C, (uint32_t *)D,
                       m, n, k, total, efdpa_mark(p));
    MMAEMU_HIP(hipGetLastError());
    return MMAEMU_OK;
}

mmaemu_status launch_emulate_efdpa_pairs(const ModelArgs &p, const void *A, const void *B, const void *C, void *D, uint32_t m, uint32_t n,
                                         uint32_t k, uint64_t batch, uint32_t ta, uint32_t tb, hipStream_t s)
{
    const uint64_t total = batch * m * n;
    uint64_t blocks = (total + 255) / 256;
    if (blocks > (1ull << 20)) blocks = 1ull << 20;
    hipLaunchKernelGGL(emulate_efdpa_pairs_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, p, ta, tb, A, B, (const uint32_t *)C, (uint32_t *)D,
                       m, n, k, total, efdpa_mark(p));
    MMAEMU_HIP(hipGetLastError());
    const mmaemu_status st = launch_marked(p, A, B, C, D, m, n, k, batch, ta, tb, s);
    if (st != MMAEMU_OK) return st;
    set_last_kernel("e-fdpa, one thread per output");
    return MMAEMU_OK;
}

mmaemu_status launch_emulate_efdpa(const ModelArgs &p, const void *A, const void *B, const void *C, void *D, uint32_t m, uint32_t n,
                                   uint32_t k, uint64_t batch, uint32_t ta, uint32_t tb, hipStream_t s)
{
    const uint64_t nblocks = batch * (m / 16) * (n / 16);
    const uint64_t grid = nblocks < (1ull << 16) ? nblocks : (1ull << 16);
    if (C == D) {
        // in place: the accumulators are gone once the block kernel has run, so it finishes every output itself
        hipLaunchKernelGGL(emulate_efdpa_blocks_kernel<false>, dim3((uint32_t)grid), dim3(256), 0, s, p, ta, tb, A, B, (const uint32_t *)C,
                           (uint32_t *)D, m, n, k, nblocks, 0u);
        MMAEMU_HIP(hipGetLastError());
        set_last_kernel("e-fdpa, 16x16 blocks through LDS, in place");
        return MMAEMU_OK;
    }
    hipLaunchKernelGGL(emulate_efdpa_blocks_kernel<true>, dim3((uint32_t)grid), dim3(256), 0, s, p, ta, tb, A, B, (const uint32_t *)C,
                       (uint32_t *)D, m, n, k, nblocks, efdpa_mark(p));
    MMAEMU_HIP(hipGetLastError());
    const mmaemu_status st = launch_marked(p, A, B, C, D, m, n, k, batch, ta, tb, s);
    if (st != MMAEMU_OK) return st;
    set_last_kernel("e-fdpa, 16x16 blocks through LDS");
    return MMAEMU_OK;
}

} // namespace mmaemu
