// Map builder for double-precision inputs (the paper reports float and double runs: section 4,
// table of the server machines).  Same maps as mmm_build.hip, from 8-byte elements:
//   a_bits[i,k]  = pred(X[i,k]) & keep_bits[i,k] & (X[i,k] != 0)          (section 3 "Optimizations",
//                                                                           Fig. "Blocked sparse row preprocessing")
//   b_bits[k,jb] = keep_rows[k] & keep_blocks[k,jb] & (some Y[k, jb*bw ..) != 0)
//                                                                          (section 3 "Block-Random Sparsity in B")
// plus the column-any words of A and the transposed B map.  Double-precision inputs are multiplied by
// the pair kernel only, which needs the bitmaps and nothing else: no blocked lists are written.
// Predicates are decided on the 64-bit pattern with integer compares, like the 32-bit ones.
#include "mmm_internal.h"

namespace {

__device__ __forceinline__ uint64_t order_key64(uint64_t u)
{
    if ((u & 0x7fffffffffffffffull) == 0) u = 0;
    return (u & 0x8000000000000000ull) ? ~u : (u | 0x8000000000000000ull);
}

__device__ __forceinline__ bool keep_element64(int32_t pred, uint64_t u, uint64_t thr)
{
    const uint64_t a = u & 0x7fffffffffffffffull;
    if (pred == MMM_PRED_NONZERO) return a != 0;
    const bool ok = a != 0 && a <= 0x7ff0000000000000ull;   // not zero, not NaN
    if (pred == MMM_PRED_GT) return ok && order_key64(u) > thr;
    return ok && a > thr;
}

// One workgroup = one 32-row tile x one 64-column word; wave v scans rows 8v .. 8v+7.
__global__ __launch_bounds__(256) void mmm_build64_a_kernel(const double *X, int64_t ldx, const uint64_t *keep_a,
                                                            uint64_t *a_bits, uint64_t *a_colany, int64_t M, int64_t K,
                                                            int64_t WA, int32_t pred, uint64_t thr)
{
    __shared__ uint64_t any[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t t = blockIdx.x / WA, w = blockIdx.x % WA;
    const int64_t k = w * 64 + lane;
    uint64_t u[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        // loaded unconditionally at a clamped position and masked afterwards: a load inside a branch is
        // waited for before the next one is issued
        const int64_t r = t * 32 + wave * 8 + j;
        u[j] = (uint64_t)__double_as_longlong(X[min(r, M - 1) * ldx + min(k, K - 1)]);
        if (r >= M || k >= K) u[j] = 0;
    }
    uint64_t colany = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int64_t r = t * 32 + wave * 8 + j;
        uint64_t m = __ballot(keep_element64(pred, u[j], thr));   // lanes past K or M hold +0
        if (r < M) {
            if (keep_a != nullptr) m &= keep_a[r * WA + w];
            if (lane == 0) a_bits[r * WA + w] = m;
            colany |= m;
        }
    }
    if (lane == 0) any[wave] = colany;
    __syncthreads();
    if (threadIdx.x == 0) a_colany[t * WA + w] = any[0] | any[1] | any[2] | any[3];
}

// One wave = one row k x one word of 64 blocks.  Blocks the keep bitmaps switch off are not read.
template <int BW>
__global__ __launch_bounds__(256) void mmm_build64_b_kernel(const double *Y, int64_t ldy, const uint64_t *keep_rows,
                                                            const uint64_t *keep_blocks, uint64_t *b_bits, int64_t K,
                                                            int64_t NB, int64_t WB)
{
    constexpr int BPL = 64 / BW;   // blocks covered by one 64-lane load
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t idx = (int64_t)blockIdx.x * 4 + wave;
    const int64_t k = idx / WB, w = idx % WB;
    if (k >= K) return;
    const int64_t nb_left = NB - w * 64;
    uint64_t kept = nb_left >= 64 ? ~0ull : ((1ull << nb_left) - 1ull);
    if (keep_rows != nullptr && !((keep_rows[k >> 6] >> (k & 63)) & 1ull)) kept = 0;
    if (keep_blocks != nullptr) kept &= keep_blocks[k * WB + w];
    uint64_t word = 0;
    if (kept != 0) {
        const double *row = Y + k * ldy + w * 64 * BW;
        const uint64_t bwmask = BW == 32 ? 0xffffffffull : ((1ull << BW) - 1ull);
        uint64_t mine = 0;
        // unconditional loads, eight in flight: lanes whose block is switched off read the first switched-on
        // block of the word instead (a block that may be read) and are masked afterwards
        const int first_on = __builtin_ctzll(kept) * BW + lane % BW;
#pragma unroll
        for (int j0 = 0; j0 < BW; j0 += 8) {
            uint64_t u[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {   // load j0 + j holds the blocks (j0 + j) * BPL .. of the word
                const int blk = (j0 + j) * BPL + lane / BW;
                u[j] = (uint64_t)__double_as_longlong(row[(kept >> blk) & 1ull ? (j0 + j) * 64 + lane : first_on]);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int blk = (j0 + j) * BPL + lane / BW;
                const uint64_t m = __ballot(((kept >> blk) & 1ull) && (u[j] & 0x7fffffffffffffffull) != 0);
                if (lane / BPL == j0 + j) mine = m;   // lane L collects the load that holds block L
            }
        }
        word = __ballot(((mine >> ((lane % BPL) * BW)) & bwmask) != 0);
    }
    if (lane == 0) b_bits[k * WB + w] = word;
}

// bt_bits[jb][kw] bit b = b_bits[kw * 64 + b][jb]: one thread per word of the transposed map.
__global__ __launch_bounds__(256) void mmm_transpose_bits_kernel(const uint64_t *b_bits, uint64_t *bt_bits, int64_t K,
                                                                 int64_t NB, int64_t WA, int64_t WB)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= NB * WA) return;
    const int64_t kw = idx / NB, jb = idx % NB;   // consecutive threads: consecutive blocks, the same rows of b_bits
    uint64_t out = 0;
    for (int b = 0; b < 64; ++b) {
        const int64_t k = kw * 64 + b;
        if (k < K) out |= ((b_bits[k * WB + (jb >> 6)] >> (jb & 63)) & 1ull) << b;
    }
    bt_bits[jb * WA + kw] = out;
}

uint64_t threshold_key64(int32_t pred, float threshold)
{
    union { double f; uint64_t u; } cv;
    cv.f = (double)threshold;
    uint64_t t = cv.u;
    const uint64_t at = t & 0x7fffffffffffffffull;
    if (at > 0x7ff0000000000000ull) return ~0ull;   // NaN threshold: nothing passes
    if (pred == MMM_PRED_GT) {
        if (at == 0) t = 0;
        return (t & 0x8000000000000000ull) ? ~t : (t | 0x8000000000000000ull);
    }
    if (pred == MMM_PRED_ABS_GT) return (t & 0x8000000000000000ull) ? 0ull : at;
    return 0;
}

}   // namespace

uint64_t mmm_threshold_key64(int32_t pred, float threshold) { return threshold_key64(pred, threshold); }

hipError_t mmm_launch_build64(const mmm_maps *m, const mmm_build_args &a, hipStream_t s)
{
    (void)hipGetLastError();
    if (a.X != nullptr) {
        const int64_t wgs = m->MT * m->WA;
        if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
        hipLaunchKernelGGL(mmm_build64_a_kernel, dim3((uint32_t)wgs), dim3(256), 0, s, static_cast<const double *>(a.X), a.ldx,
                           a.keep_a, m->a_bits, m->a_colany, m->M, m->K, m->WA, a.pred, threshold_key64(a.pred, a.threshold));
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    if (a.Y != nullptr) {
        const int64_t waves = m->K * m->WB, wgs = (waves + 3) / 4;
        const int64_t tw = (m->NB * m->WA + 255) / 256;
        if (wgs > 0x7fffffffLL || tw > 0x7fffffffLL) return hipErrorInvalidValue;
        const double *Y = static_cast<const double *>(a.Y);
        if (m->bw == 8)
            hipLaunchKernelGGL(mmm_build64_b_kernel<8>, dim3((uint32_t)wgs), dim3(256), 0, s, Y, a.ldy, a.keep_rows,
                               a.keep_blocks, m->b_bits, m->K, m->NB, m->WB);
        else if (m->bw == 16)
            hipLaunchKernelGGL(mmm_build64_b_kernel<16>, dim3((uint32_t)wgs), dim3(256), 0, s, Y, a.ldy, a.keep_rows,
                               a.keep_blocks, m->b_bits, m->K, m->NB, m->WB);
        else
            hipLaunchKernelGGL(mmm_build64_b_kernel<32>, dim3((uint32_t)wgs), dim3(256), 0, s, Y, a.ldy, a.keep_rows,
                               a.keep_blocks, m->b_bits, m->K, m->NB, m->WB);
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
        hipLaunchKernelGGL(mmm_transpose_bits_kernel, dim3((uint32_t)tw), dim3(256), 0, s, m->b_bits, m->bt_bits, m->K, m->NB,
                           m->WA, m->WB);
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    return hipSuccess;
}
