// Masked GEMM on the vector ALUs, over exactly the surviving products:
//   C[i,j] = sum over k with a_bits[i,k] & b_bits[k, j div bw] of X[i,k] * Y[k,j]
// (paper, section 3 "Random sparsity in A": a zero element of A skips a whole row of B;
// section 3 "Block-Random Sparsity in B": an empty block of B is skipped; Fig. "MMM
// Pseudocode" does both).  No product with a zero element of A or an empty block of B is
// ever formed here, so the work is p_A * p_B of the dense work, and skipped operands cannot
// reach the arithmetic at all.
//
// Mapping onto a 64-lane wavefront.  A wave owns one row i of C and 64 consecutive columns
// = G = 64 / bw blocks of B, lane group g <-> block jb0 + g.  For a range of k the wave
// intersects the bitmap row of A with the transposed B map of each of its blocks (one 64-bit
// AND per 64 values of k, the words spread over the lanes of a group), ranks the survivors with
// a prefix sum inside the group, writes the surviving k of every block into a short list in
// LDS, and then walks the G lists side by side: in round t lane group g multiplies X[i, k_t(g)]
// with its 1 x bw block of row k_t(g) of Y and adds it to its accumulator.  Lists are padded
// with copies of their first entry (multiplied by 0) so that a batch of 8 rounds needs no
// per-entry branch; only a lane group whose list is empty is switched off.  The bitmap
// intersection plays the role of the paper's pattern lookup: the branch per element is taken
// once, on 64 elements at a time.
//
// There is no staging and no workgroup barrier on this path (two dependent memory round trips:
// map words, then operands), which is what makes it fast for matrices of few rows, where the
// multiplication is latency-bound.  Waves of a workgroup that share a column span split K
// between them and add their partial sums in a fixed order at the end.
//
// The matrix-instruction kernel multiplies every listed row of B with all 64 rows of a tile of
// A, zeros included; this kernel pays two gathers per product instead.  It needs only the two
// bitmaps, not the blocked lists of A.  With FUSED the mask M is evaluated right here (the
// waves of a workgroup ballot the predicate over the row of X into LDS first), so no A-side map
// pass is needed.
#include <type_traits>

#include "mmm_internal.h"

namespace {

constexpr int MAX_WAVE_WORDS = 64;  // map words (64 k each) one wave intersects at a time, at most: 4096 values of k
constexpr int LIST_SLOTS = 1024;    // list entries per wave, shared by its G lists
constexpr int U = 8;                // list entries per batch (one 16-byte LDS read); 16 was measured slower
constexpr int SUPER_WORDS = 1024;   // FUSED: bitmap words of the row kept in LDS at a time (65536 values of k)

struct PairsParams {
    const void *X;
    int64_t ldx;
    const void *Y;
    int64_t ldy;
    void *C;                  // float, or double for double inputs
    int64_t ldc;
    const uint64_t *a_bits;   // M x WA words (not FUSED)
    const uint64_t *keep_a;   // FUSED: optional keep bitmap of M, M x WA words
    const uint64_t *bt_bits;  // NB x WA words
    int64_t M, K, N, NB, WA;
    uint64_t thr_bits;        // FUSED: threshold key of the predicate
    int32_t pred;
    int32_t accumulate;
};

template <typename T> __device__ __forceinline__ uint32_t bits_of(T v);
template <> __device__ __forceinline__ uint32_t bits_of<float>(float v) { return __float_as_uint(v); }
template <> __device__ __forceinline__ uint32_t bits_of<uint16_t>(uint16_t v) { return (uint32_t)v << 16; }   // bf16
template <> __device__ __forceinline__ uint32_t bits_of<_Float16>(_Float16 v) { return __float_as_uint((float)v); }

__device__ __forceinline__ uint32_t pairs_order_key(uint32_t u)
{
    if ((u & 0x7fffffffu) == 0) u = 0;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint64_t pairs_order_key64(uint64_t u)
{
    if ((u & 0x7fffffffffffffffull) == 0) u = 0;
    return (u & 0x8000000000000000ull) ? ~u : (u | 0x8000000000000000ull);
}

// Per element type: the type products are accumulated in (float; double for double inputs), the exact
// widening of an element to it, and the element predicate of M on the bit pattern, non-zero test
// included (same decisions as the map builder: integer compares, NaN fails > and |.| >, denormals
// are non-zero).  thr: the threshold key the host prepares (32-bit key in the low half for the float types).
__device__ __forceinline__ float fma_acc(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double fma_acc(double a, double b, double c) { return __builtin_fma(a, b, c); }

template <typename T> struct Elem {
    typedef float acc;
    static __device__ __forceinline__ acc value(T v) { return __uint_as_float(bits_of<T>(v)); }
    static __device__ __forceinline__ bool keep(int32_t pred, T v, uint64_t thr64)
    {
        const uint32_t u = bits_of<T>(v), thr = (uint32_t)thr64;
        const uint32_t a = u & 0x7fffffffu;
        if (pred == MMM_PRED_NONZERO) return a != 0;
        const bool ok = a != 0 && a <= 0x7f800000u;
        if (pred == MMM_PRED_GT) return ok && pairs_order_key(u) > thr;
        return ok && a > thr;
    }
    static __device__ __forceinline__ T zero() { return T(0); }
};
template <> struct Elem<double> {
    typedef double acc;
    static __device__ __forceinline__ acc value(double v) { return v; }
    static __device__ __forceinline__ bool keep(int32_t pred, double v, uint64_t thr)
    {
        const uint64_t u = (uint64_t)__double_as_longlong(v);
        const uint64_t a = u & 0x7fffffffffffffffull;
        if (pred == MMM_PRED_NONZERO) return a != 0;
        const bool ok = a != 0 && a <= 0x7ff0000000000000ull;
        if (pred == MMM_PRED_GT) return ok && pairs_order_key64(u) > thr;
        return ok && a > thr;
    }
    static __device__ __forceinline__ double zero() { return 0.0; }
};

__device__ __forceinline__ uint32_t pairs_xcd_id(uint32_t b, uint32_t n)
{
    const uint32_t x = b & 7u, i = b >> 3, q = n >> 3, rem = n & 7u;
    return x * q + (x < rem ? x : rem) + i;
}

// CW: waves side by side (64 columns each); KS: waves that share a column span and take the
// 4096-wide ranges of k in turn (their partial sums are added in a fixed order at the end).
// WAVE_WORDS: map words one wave intersects at a time (a range of 64 * WAVE_WORDS values of k).
template <typename T, int BW, int CW, int KS, int WAVE_WORDS, bool FUSED>
__global__ __launch_bounds__(CW *KS * 64) void mmm_pairs_kernel(const PairsParams p)
{
    static_assert(WAVE_WORDS <= MAX_WAVE_WORDS && WAVE_WORDS % BW == 0, "whole words per lane, offsets fit the lists");
    constexpr int NW = CW * KS;
    constexpr int G = 64 / BW;                 // blocks (lists) per wave
    constexpr int CAP = LIST_SLOTS / G;        // entries per list and pass
    constexpr int WPL = WAVE_WORDS / BW;       // words per lane and range
    constexpr uint32_t ESZ = (uint32_t)sizeof(T);
    typedef typename Elem<T>::acc acc_t;
    static_assert(CAP % U == 0, "a batch never leaves its list");

    __shared__ uint64_t aw[FUSED ? SUPER_WORDS : 1];   // FUSED: bitmap words of the row
    __shared__ __align__(16) uint16_t lists[NW][LIST_SLOTS];
    __shared__ acc_t red[KS > 1 ? (KS - 1) * CW * 64 : 1];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cw = wave % CW, ks = wave / CW;
    const int g = lane / BW, c = lane % BW;

    // Consecutive workgroups of one XCD work on consecutive rows of the same column span, so the
    // blocks of Y and the map words of that span stay in that XCD's L2.
    const uint32_t L = pairs_xcd_id(blockIdx.x, gridDim.x);
    const uint32_t ct = L / (uint32_t)p.M;
    const int64_t i = L % (uint32_t)p.M;
    const int64_t col0 = ((int64_t)ct * CW + cw) * 64;
    const int64_t col = col0 + lane;
    const int64_t jb = col0 / BW + g;          // this lane group's block column
    const bool blk_ok = jb < p.NB;

    const T *Xrow = static_cast<const T *>(p.X) + i * p.ldx;
    const uint64_t *arow = p.a_bits + i * p.WA;
    const uint64_t *btrow = p.bt_bits + (blk_ok ? jb : 0) * p.WA;
    const uint32_t ldyb = (uint32_t)p.ldy * ESZ;
    const uint32_t ldy = (uint32_t)p.ldy;   // below 2^22: a 24-bit multiplier
    // first column of the wave (wave-uniform); a lane adds a 32-bit offset to it
    const char *Ycol = static_cast<const char *>(p.Y) + min(col0, p.N - 1) * ESZ;
    const uint32_t lane_off = blk_ok ? (uint32_t)lane * ESZ : 0u;
    uint16_t *lst = &lists[wave][g * CAP];
    acc_t acc = 0;

    for (int64_t sw0 = 0; sw0 < p.WA; sw0 += SUPER_WORDS) {   // one trip unless FUSED and K > 65536
        const int sw = (int)min((int64_t)SUPER_WORDS, p.WA - sw0);
        if (FUSED) {
            __syncthreads();   // the words of the previous trip are no longer needed
            // Every load below is unconditional (indices are clamped, results masked afterwards): a load
            // inside a branch is waited for before the next one is issued.
            constexpr int PU = 8;   // words per trip: their loads are in flight together
            auto ballots = [&](auto with_keep) __attribute__((always_inline)) {
                for (int w = wave; w < sw; w += PU * NW) {
                    T u[PU];
                    uint64_t kp[PU];
#pragma unroll
                    for (int q = 0; q < PU; ++q) {
                        const int wq = min(w + q * NW, sw - 1);
                        const int64_t k = min((sw0 + wq) * 64 + lane, p.K - 1);
                        u[q] = Xrow[k];
                        kp[q] = ~0ull;
                        if constexpr (decltype(with_keep)::value) kp[q] = p.keep_a[i * p.WA + sw0 + wq];
                    }
#pragma unroll
                    for (int q = 0; q < PU; ++q) {
                        const int wq = w + q * NW;
                        const bool inside = wq < sw && (sw0 + wq) * 64 + lane < p.K;   // lanes past K are never kept
                        const uint64_t m = __ballot(inside && Elem<T>::keep(p.pred, u[q], p.thr_bits)) & kp[q];
                        if (lane == 0 && wq < sw) aw[wq] = m;
                    }
                }
            };
            if (p.keep_a != nullptr)
                ballots(std::true_type{});
            else
                ballots(std::false_type{});
            __syncthreads();
        }
        // this wave's ranges of the trip: ranges ks, ks + KS, ... of WAVE_WORDS words each
        for (int rw0 = ks * WAVE_WORDS; rw0 < sw; rw0 += KS * WAVE_WORDS) {
            const int rw1 = min(sw, rw0 + WAVE_WORDS);
            const int64_t word0 = sw0 + rw0;               // first word of the range
            // this lane's words of the range: rw0 + c, rw0 + c + BW, ...
            uint64_t m[WPL];
            uint32_t cnt = 0;
#pragma unroll
            for (int j = 0; j < WPL; ++j) {
                const int wi = rw0 + c + j * BW;
                const int wic = min(wi, rw1 - 1);   // loaded unconditionally (a load inside a branch is waited for at once), masked below
                const uint64_t wa = FUSED ? aw[wic] : arow[sw0 + wic], wb = btrow[sw0 + wic];
                m[j] = wi < rw1 && blk_ok ? wa & wb : 0ull;
                cnt += (uint32_t)__popcll(m[j]);
            }
            // ranks: exclusive prefix of the counts inside the lane group, and the group's total
            uint32_t incl = cnt;
#pragma unroll
            for (int d = 1; d < BW; d <<= 1) {
                const uint32_t o = (uint32_t)__shfl_up((int)incl, d, BW);
                if (c >= d) incl += o;
            }
            const uint32_t first = incl - cnt;
            const uint32_t n_g = (uint32_t)__shfl((int)incl, BW - 1, BW);
            uint32_t nmax = 0;
#pragma unroll
            for (int q = 0; q < G; ++q) nmax = max(nmax, (uint32_t)__builtin_amdgcn_readlane((int)n_g, q * BW));
            if (nmax == 0) continue;

            const int64_t k0 = word0 * 64;                       // first k of the range
            const char *Yr = Ycol + k0 * (int64_t)ldyb;          // row k0 of Y at the wave's first column
            const char *Xr = reinterpret_cast<const char *>(Xrow + k0);

            // Lists longer than CAP are walked in several passes of CAP entries.
            for (uint32_t base = 0; base < nmax; base += CAP) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();   // the previous pass has read its entries
                uint32_t pos = first - base;       // rank of this lane's next survivor within the pass (wraps below 0)
#pragma unroll
                for (int j = 0; j < WPL; ++j) {
                    uint64_t mm = m[j];
                    const uint32_t kw = (uint32_t)(c + j * BW) * 64u;   // entries are byte offsets into the row of X
                    while (mm != 0) {
                        const uint32_t bit = (uint32_t)__builtin_ctzll(mm);
                        mm &= mm - 1;
                        if (pos < (uint32_t)CAP) lst[pos] = (uint16_t)((kw + bit) * ESZ);
                        ++pos;
                    }
                }
                const uint32_t n_here = n_g > base ? min(n_g - base, (uint32_t)CAP) : 0u;   // entries of this lane group
                uint32_t rmax = 0, rmin = CAP;
#pragma unroll
                for (int q = 0; q < G; ++q) {
                    const uint32_t v = (uint32_t)__builtin_amdgcn_readlane((int)n_here, q * BW);
                    rmax = max(rmax, v);
                    rmin = min(rmin, v);
                }
                const uint32_t rend = (rmax + U - 1) / U * U;   // at most CAP
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                // pad the list up to the last batch the wave runs with copies of its first entry: a valid
                // row of Y for this block, multiplied by 0 below
                if (n_here != 0 && n_here < rend) {
                    const uint16_t e0 = lst[0];
                    for (uint32_t q = n_here + c; q < rend; q += BW) lst[q] = e0;
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                }
                __builtin_amdgcn_wave_barrier();
                const bool alive = n_here != 0;
                uint32_t t = 0;
                // rounds in which every lane group has an entry
                for (; t + U <= rmin; t += U) {
                    const uint4 e4 = *reinterpret_cast<const uint4 *>(lst + t);
                    const uint32_t e[4] = {e4.x, e4.y, e4.z, e4.w};
                    acc_t a[U], b[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const uint32_t kb = (u & 1) ? (e[u >> 1] >> 16) : (e[u >> 1] & 0xffffu);   // k * ESZ
                        a[u] = Elem<T>::value(*reinterpret_cast<const T *>(Xr + kb));
                        b[u] = Elem<T>::value(*reinterpret_cast<const T *>(Yr + (__umul24(kb, ldy) + lane_off)));
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) acc = fma_acc(a[u], b[u], acc);
                }
                // ragged ends: padded entries count for nothing, empty lists are switched off
                for (; t < rend; t += U) {
                    acc_t a[U], b[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) a[u] = b[u] = 0;
                    if (alive) {
                        const uint4 e4 = *reinterpret_cast<const uint4 *>(lst + t);
                        const uint32_t e[4] = {e4.x, e4.y, e4.z, e4.w};
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const uint32_t kb = (u & 1) ? (e[u >> 1] >> 16) : (e[u >> 1] & 0xffffu);
                            a[u] = Elem<T>::value(*reinterpret_cast<const T *>(Xr + kb));
                            b[u] = Elem<T>::value(*reinterpret_cast<const T *>(Yr + (__umul24(kb, ldy) + lane_off)));
                        }
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) acc = fma_acc(t + u < n_here ? a[u] : acc_t(0), b[u], acc);
                }
            }
        }
    }

    if (KS > 1) {   // add the partial sums of the waves that shared this column span, in wave order
        if (ks > 0) red[((ks - 1) * CW + cw) * 64 + lane] = acc;
        __syncthreads();
        if (ks == 0)
#pragma unroll
            for (int q = 1; q < KS; ++q) acc += red[((q - 1) * CW + cw) * 64 + lane];
    }
    if (ks == 0 && col < p.N) {
        acc_t *dst = static_cast<acc_t *>(p.C) + i * p.ldc + col;
        *dst = p.accumulate ? *dst + acc : acc;
    }
}

typedef void (*pairs_kernel_fn)(const PairsParams);

struct PairsShape { int cw, ks; };

template <typename T, int BW, bool FUSED> pairs_kernel_fn pick_shape(int shape)
{
    switch (shape) {
    case 1: return mmm_pairs_kernel<T, BW, 2, 4, 64, FUSED>;    // few rows: 128 columns, K in four shares
    case 2: return mmm_pairs_kernel<T, BW, 8, 2, 64, FUSED>;    // few rows, mask evaluated here: the predicate work is shared by 512 columns
    case 3: return mmm_pairs_kernel<T, BW, 4, 4, 64, FUSED>;    // very few rows, mask evaluated here: one range of k per wave
    default: return mmm_pairs_kernel<T, BW, 8, 1, 64, FUSED>;   // 512 columns side by side
    }
}
constexpr PairsShape kShapes[] = {{8, 1}, {2, 4}, {8, 2}, {4, 4}};

template <typename T, bool FUSED> pairs_kernel_fn pick(int32_t bw, int shape)
{
    if (bw == 8) return pick_shape<T, 8, FUSED>(shape);
    if (bw == 16) return pick_shape<T, 16, FUSED>(shape);
    return pick_shape<T, 32, FUSED>(shape);
}

uint32_t pairs_threshold_key(int32_t pred, float threshold)
{
    union { float f; uint32_t u; } cv;
    cv.f = threshold;
    uint32_t t = cv.u;
    const uint32_t at = t & 0x7fffffffu;
    if (at > 0x7f800000u) return 0xffffffffu;   // NaN threshold: nothing passes
    if (pred == MMM_PRED_GT) {
        if (at == 0) t = 0;
        return (t & 0x80000000u) ? ~t : (t | 0x80000000u);
    }
    if (pred == MMM_PRED_ABS_GT) return (t & 0x80000000u) ? 0u : at;
    return 0;
}

}   // namespace

bool mmm_pairs_supports(int32_t dtype, int64_t ldy)
{
    const int64_t esz = dtype == MMM_F64 ? 8 : dtype == MMM_F32 ? 4 : 2;
    return ldy * esz * (MAX_WAVE_WORDS * 64) + 256 <= 0xffffffffLL;
}

// fused: evaluate M (pred, threshold, keep_a) on X in the kernel; otherwise take a_bits from the maps.
hipError_t mmm_launch_pairs(const mmm_maps *m, int32_t dtype, const void *X, int64_t ldx, const void *Y, int64_t ldy,
                            void *C, int64_t ldc, int32_t accumulate, bool fused, int32_t pred, float threshold,
                            const uint64_t *keep_a, hipStream_t s)
{
    PairsParams p{};
    p.X = X;
    p.ldx = ldx;
    p.Y = Y;
    p.ldy = ldy;
    p.C = C;
    p.ldc = ldc;
    p.a_bits = m->a_bits;
    p.keep_a = keep_a;
    p.bt_bits = m->bt_bits;
    p.M = m->M;
    p.K = m->K;
    p.N = m->N;
    p.NB = m->NB;
    p.WA = m->WA;
    p.pred = pred;
    p.thr_bits = dtype == MMM_F64 ? mmm_threshold_key64(pred, threshold) : (uint64_t)pairs_threshold_key(pred, threshold);
    p.accumulate = accumulate;
    // Workgroups of 8 waves x 64 columns; when that gives the machine too little to do (few rows:
    // the decode shape), fewer columns per workgroup and K shared out over several waves.
    const int64_t wide = (m->N + 511) / 512 * m->M;
    const int shape = wide >= 1024 ? 0 : !fused ? 1 : m->M <= 16 ? 3 : 2;
    const PairsShape sh = kShapes[shape];
    const int64_t span = sh.cw * 64;
    const int64_t ctiles = (m->N + span - 1) / span;
    const int64_t wgs = ctiles * m->M;
    if (wgs <= 0 || wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    pairs_kernel_fn fn;
    if (fused)
        fn = dtype == MMM_F64 ? pick<double, true>(m->bw, shape) : dtype == MMM_BF16 ? pick<uint16_t, true>(m->bw, shape) : dtype == MMM_F16 ? pick<_Float16, true>(m->bw, shape)
                                                                                         : pick<float, true>(m->bw, shape);
    else
        fn = dtype == MMM_F64 ? pick<double, false>(m->bw, shape) : dtype == MMM_BF16 ? pick<uint16_t, false>(m->bw, shape) : dtype == MMM_F16 ? pick<_Float16, false>(m->bw, shape)
                                                                                          : pick<float, false>(m->bw, shape);
    (void)hipGetLastError();
    hipLaunchKernelGGL(fn, dim3((uint32_t)wgs), dim3((uint32_t)(sh.cw * sh.ks * 64)), 0, s, p);
    return hipGetLastError();
}
