// Map builder: evaluates the masks M and N on the device and writes the
// sparsity maps (paper, section 3 "Preprocessing": a single sequential, aligned
// pass per matrix).  Everything here is integer work on float bit patterns,
// bound by HBM bandwidth.
//
// A side (section 3 "Optimizations", Fig. "Blocked sparse row preprocessing"):
// per block of 64 rows x 128 columns the count of non-zero elements and their
// positions inside the block, here together with the values, in row-major order;
// plus the plain non-zero bitmap and its column-any summary.
// B side (section 3 "Block-Random Sparsity in B", Fig. "Preprocessing
// patterns"): one bit per block, 1 = some non-zero value; plus the same map
// transposed to one bit-row per block column.
//
// One launch covers both matrices: the first n_a workgroups scan X, the rest
// scan Y.  Every output word in device memory has exactly one producer, so no
// global atomics are used and nothing needs clearing beforehand.
#include "mmm_internal.h"

namespace {

constexpr int BUILD_WAVES = 8;
constexpr int BUILD_THREADS = BUILD_WAVES * 64;
constexpr int A_ROWS_PER_WAVE = MMM_AB_ROWS / BUILD_WAVES;   // 8
constexpr int A_WORDS = MMM_AB_COLS / 64;                    // 2
constexpr int B_ROWS_PER_WAVE = MMM_BT_PIECE / BUILD_WAVES;  // 2

struct BuildParams {
    const void *X;
    int64_t ldx;
    const uint64_t *keep_a;
    uint64_t *a_bits;
    uint64_t *a_colany;
    uint32_t *a_cnt;
    uint2 *a_ent;
    const void *Y;
    int64_t ldy;
    const uint64_t *keep_rows;
    const uint64_t *keep_blocks;
    uint64_t *b_bits;
    uint16_t *bt_pieces;   // the transposed B map seen as pieces of MMM_BT_PIECE bits
    int64_t M, K, N, NB, WA, WB, MT, KBA;
    uint32_t thr_bits;
    int32_t pred;
    uint32_t n_a;   // workgroups that scan X
};

template <typename T> __device__ __forceinline__ uint32_t f32_bits(T v);
template <> __device__ __forceinline__ uint32_t f32_bits<float>(float v) { return __float_as_uint(v); }
template <> __device__ __forceinline__ uint32_t f32_bits<uint16_t>(uint16_t v) { return (uint32_t)v << 16; }   // bf16
template <> __device__ __forceinline__ uint32_t f32_bits<_Float16>(_Float16 v) { return __float_as_uint((float)v); }

// Order-preserving key of a non-NaN float with both zeros mapped to +0.
__device__ __forceinline__ uint32_t order_key(uint32_t u)
{
    if ((u & 0x7fffffffu) == 0) u = 0;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Element predicate of M, decided on the bit pattern so that no denormal mode
// of the float pipeline can change a map bit.  Includes the non-zero test.
// `thr` is prepared by the host (see threshold_key): for GT the order key of the
// threshold, for ABS_GT its magnitude bits; NaN never passes GT / ABS_GT.
template <int PRED> __device__ __forceinline__ bool keep_element(uint32_t u, uint32_t thr)
{
    const uint32_t a = u & 0x7fffffffu;
    if (PRED == MMM_PRED_NONZERO) return a != 0;
    const bool ok = a != 0 && a <= 0x7f800000u;
    if (PRED == MMM_PRED_GT) return ok && order_key(u) > thr;
    return ok && a > thr;
}

__device__ __forceinline__ uint64_t ballot64(bool p) { return __ballot(p); }

__device__ __forceinline__ uint32_t mbcnt64(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// ---- A side: one workgroup = one block of 64 rows x 128 columns ------------------------------
// Wave w scans rows 8w..8w+7, one 64-column word per load.  Lane 2j+h of the wave ends up
// holding the bitmap word (row j, half h); entries are appended in (row, column) order.
template <typename T, int PRED>
__device__ __forceinline__ void scan_a(const BuildParams &p, uint32_t b, int lane, int wave, uint64_t *red,
                                       uint32_t *tot)
{
    const int64_t bi = b / p.KBA, bj = b % p.KBA;
    const int64_t k_lo = bj * MMM_AB_COLS;
    const int64_t rbase = bi * MMM_AB_ROWS + wave * A_ROWS_PER_WAVE;
    const int64_t w_lo = k_lo / 64;
    const T *X = static_cast<const T *>(p.X);
    // keep words of the wave's 16 (row, half) pairs, one per lane 2j+h, requested together with X
    uint64_t kw = ~0ull;
    if (p.keep_a != nullptr && lane < 2 * A_ROWS_PER_WAVE && rbase + (lane >> 1) < p.M && w_lo + (lane & 1) < p.WA)
        kw = p.keep_a[(rbase + (lane >> 1)) * p.WA + w_lo + (lane & 1)];
    uint32_t u[A_ROWS_PER_WAVE][A_WORDS];
#pragma unroll
    for (int j = 0; j < A_ROWS_PER_WAVE; ++j) {
#pragma unroll
        for (int h = 0; h < A_WORDS; ++h) {
            const int64_t r = rbase + j, k = k_lo + 64 * h + lane;
            u[j][h] = 0;
            if (r < p.M && k < p.K) u[j][h] = f32_bits<T>(X[r * p.ldx + k]);
        }
    }
    uint64_t colany[A_WORDS] = {0, 0};
    uint32_t mine_lo = 0, mine_hi = 0;   // lane 2j+h: the bitmap word of (row j, half h)
#pragma unroll
    for (int j = 0; j < A_ROWS_PER_WAVE; ++j) {
#pragma unroll
        for (int h = 0; h < A_WORDS; ++h) {
            uint64_t m = ballot64(keep_element<PRED>(u[j][h], p.thr_bits));   // lanes past K or M hold +0
            m &= ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)(kw >> 32), 2 * j + h) << 32) |
                 (uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)kw, 2 * j + h);
            colany[h] |= m;
            const bool owner = __builtin_amdgcn_inverse_ballot_w64(1ull << (2 * j + h));   // lane 2j+h, as a constant mask
            mine_lo = owner ? (uint32_t)m : mine_lo;
            mine_hi = owner ? (uint32_t)(m >> 32) : mine_hi;
        }
    }
    const uint64_t mine = ((uint64_t)mine_hi << 32) | mine_lo;
    // bitmap words and per-wave entry offsets
    const bool have_word = lane < 2 * A_ROWS_PER_WAVE && rbase + (lane >> 1) < p.M && w_lo + (lane & 1) < p.WA;
    if (have_word) p.a_bits[(rbase + (lane >> 1)) * p.WA + w_lo + (lane & 1)] = mine;
    const uint32_t my_cnt = (uint32_t)__popcll(mine);   // lanes past the wave's words hold 0
    uint32_t incl = my_cnt;
#pragma unroll
    for (int d = 1; d < 2 * A_ROWS_PER_WAVE; d <<= 1) {
        const uint32_t o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
    }
    const uint32_t excl = incl - my_cnt;
    if (lane == 2 * A_ROWS_PER_WAVE - 1) tot[wave] = incl;
    if (lane == 0) {
        red[wave * A_WORDS + 0] = colany[0];
        red[wave * A_WORDS + 1] = colany[1];
    }
    __syncthreads();
    uint32_t base = 0;
    for (int w = 0; w < wave; ++w) base += tot[w];
    uint32_t total = 0;
    for (int w = 0; w < BUILD_WAVES; ++w) total += tot[w];
    if (threadIdx.x == 0) p.a_cnt[b] = total;
    if (threadIdx.x < 2 * A_WORDS) {   // column-any words of the two 32-row tiles of this block
        const int t = threadIdx.x >> 1, h = threadIdx.x & 1;
        const int64_t tile = bi * (MMM_AB_ROWS / MMM_COLANY_ROWS) + t;
        if (tile < p.MT && w_lo + h < p.WA)
        {
            uint64_t any = 0;   // waves t*W/2 .. (t+1)*W/2-1 cover the 32 rows of tile t
            for (int w = t * (BUILD_WAVES / 2); w < (t + 1) * (BUILD_WAVES / 2); ++w) any |= red[w * A_WORDS + h];
            p.a_colany[tile * p.WA + w_lo + h] = any;
        }
    }
    // compacted entries {byte offset inside the multiplier's LDS slab, value}, in (row, column) order
    uint2 *ent = p.a_ent + (size_t)b * MMM_AB_CAP;
#pragma unroll
    for (int j = 0; j < A_ROWS_PER_WAVE; ++j) {
#pragma unroll
        for (int h = 0; h < A_WORDS; ++h) {
            const uint32_t lo = __builtin_amdgcn_readlane(mine_lo, 2 * j + h);
            const uint32_t hi = __builtin_amdgcn_readlane(mine_hi, 2 * j + h);
            const uint64_t m = ((uint64_t)hi << 32) | lo;
            if (m == 0) continue;
            const uint32_t off = base + __builtin_amdgcn_readlane(excl, 2 * j + h);
            if (__builtin_amdgcn_inverse_ballot_w64(m)) {   // the word is the lane mask of its own non-zero elements
                const uint32_t slab = mmm_slab_pos((uint32_t)(wave * A_ROWS_PER_WAVE + j), (uint32_t)(64 * h + lane));
                ent[off + mbcnt64(m)] = make_uint2(slab, u[j][h]);
            }
        }
    }
    // pad the list to a whole number of wavefronts with entries that write 0 to a spare slab cell
    if (wave == BUILD_WAVES - 1) {
        const uint32_t e = total + lane;
        if (e < ((total + 63u) & ~63u)) ent[e] = make_uint2(MMM_SLAB_SPARE, 0u);
    }
}

// ---- B side: one workgroup = 16 rows (values of k) x 64 blocks -------------------------------
template <typename T, int BW>
__device__ __forceinline__ void scan_b(const BuildParams &p, uint32_t bb, int lane, int wave, uint32_t *pieces,
                                       uint8_t (*gpos)[B_ROWS_PER_WAVE][64], uint64_t (*gword)[B_ROWS_PER_WAVE])
{
    constexpr int BPL = 64 / BW;   // blocks covered by one 64-lane load
    const int64_t piece = bb / p.WB, w = bb % p.WB;
    const int64_t kbase = piece * MMM_BT_PIECE + wave * B_ROWS_PER_WAVE;
    const T *Y = static_cast<const T *>(p.Y);
    const int64_t nb_left = p.NB - w * 64;
    const uint64_t valid = nb_left >= 64 ? ~0ull : ((1ull << nb_left) - 1ull);
    uint32_t piece_bits = 0;
    // which blocks of the wave's rows the keep bitmaps leave switched on: lane r fetches the two
    // keep words of row r, so that all of them are in flight together
    uint64_t krw = ~0ull, kbw = ~0ull;
    {
        const int64_t kl = kbase + lane;
        const bool mine = lane < B_ROWS_PER_WAVE && kl < p.K;
        if (p.keep_rows != nullptr && mine) krw = p.keep_rows[kl >> 6];
        if (p.keep_blocks != nullptr && mine) kbw = p.keep_blocks[kl * p.WB + w];
    }
    uint64_t kept[B_ROWS_PER_WAVE];
#pragma unroll
    for (int r = 0; r < B_ROWS_PER_WAVE; ++r) {
        const int64_t k = kbase + r;
        const uint64_t kr = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)(krw >> 32), r) << 32) |
                            (uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)krw, r);
        const uint64_t kb = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)(kbw >> 32), r) << 32) |
                            (uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)kbw, r);
        kept[r] = k < p.K ? valid & kb & (0ull - ((kr >> (k & 63)) & 1ull)) : 0ull;
    }
    constexpr int PER = BW <= 16 ? BW : 16;   // loads in flight per lane and row
#pragma unroll
    for (int r = 0; r < B_ROWS_PER_WAVE; ++r) {
        const int64_t k = kbase + r;
        uint64_t word = 0;
        if (kept[r] != 0) {
            const T *row = Y + k * p.ldy + w * 64 * BW;
            const uint64_t bwmask = BW == 32 ? 0xffffffffull : ((1ull << BW) - 1ull);
            constexpr int ROUNDS = 4;   // gather path: at most ROUNDS loads of BPL kept blocks each
            const int nkept = __popcll(kept[r]);
            if (nkept <= ROUNDS * BPL) {
                // Few blocks are switched on: their positions are compacted into a short list (lane b
                // writes b at the rank of bit b), and one load fetches BPL listed blocks, wherever
                // they are.  The list and the result word are private to the wave and the row; LDS
                // executes the wave's accesses in order.
                uint8_t *plist = gpos[wave][r];
                uint64_t *res = &gword[wave][r];
                if ((kept[r] >> lane) & 1ull) plist[mbcnt64(kept[r])] = (uint8_t)lane;
                if (lane == 0) *res = 0;
                const int slot = lane / BW;   // which of the load's blocks this lane reads
                uint32_t u[ROUNDS];
                int pos[ROUNDS];
#pragma unroll
                for (int t = 0; t < ROUNDS; ++t) {
                    const int j = t * BPL + slot;
                    pos[t] = j < nkept ? (int)plist[j] : -1;
                    u[t] = 0;
                    if (pos[t] >= 0) u[t] = f32_bits<T>(row[pos[t] * BW + lane % BW]);
                }
#pragma unroll
                for (int t = 0; t < ROUNDS; ++t) {
                    if (t * BPL >= nkept) break;   // wave-uniform
                    const uint64_t m = ballot64((u[t] & 0x7fffffffu) != 0);
                    if (lane % BW == 0 && pos[t] >= 0 && ((m >> (slot * BW)) & bwmask) != 0)
                        __hip_atomic_fetch_or(res, 1ull << pos[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
                word = *res;
            } else {
                uint64_t mine = 0;
#pragma unroll
                for (int j0 = 0; j0 < BW; j0 += PER) {
                    uint32_t u[PER];
#pragma unroll
                    for (int j = 0; j < PER; ++j) {
                        const int blk = (j0 + j) * BPL + lane / BW;   // block (inside this word) of this lane's element
                        u[j] = 0;
                        if ((kept[r] >> blk) & 1ull) u[j] = f32_bits<T>(row[(j0 + j) * 64 + lane]);
                    }
#pragma unroll
                    for (int j = 0; j < PER; ++j) {
                        const uint64_t m = ballot64((u[j] & 0x7fffffffu) != 0);
                        if (lane / BPL == j0 + j) mine = m;   // lane L collects the load that holds block L
                    }
                }
                word = ballot64(((mine >> ((lane % BPL) * BW)) & bwmask) != 0);
            }
        }
        if (k < p.K && lane == 0) p.b_bits[k * p.WB + w] = word;
        piece_bits |= (uint32_t)((word >> lane) & 1ull) << (wave * B_ROWS_PER_WAVE + r);
    }
    pieces[wave * 64 + lane] = piece_bits;
    __syncthreads();
    if (wave == 0) {
        uint32_t v = 0;
        for (int w = 0; w < BUILD_WAVES; ++w) v |= pieces[w * 64 + lane];
        const int64_t blk = w * 64 + lane;
        if (blk < p.NB) p.bt_pieces[blk * (p.WA * (64 / MMM_BT_PIECE)) + piece] = (uint16_t)v;
    }
}

template <typename T>
__global__ __launch_bounds__(BUILD_THREADS) void mmm_build_kernel(const BuildParams p)
{
    __shared__ uint64_t red[BUILD_WAVES * A_WORDS];
    __shared__ uint32_t tot[BUILD_WAVES];
    __shared__ uint32_t pieces[BUILD_WAVES * 64];
    __shared__ uint8_t gpos[BUILD_WAVES][B_ROWS_PER_WAVE][64];   // B side: positions of the kept blocks of a row word
    __shared__ uint64_t gword[BUILD_WAVES][B_ROWS_PER_WAVE];     // B side: occupancy word gathered from them
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t b = blockIdx.x;
    if (b < p.n_a) {
        if (p.pred == MMM_PRED_NONZERO)
            scan_a<T, MMM_PRED_NONZERO>(p, b, lane, wave, red, tot);
        else if (p.pred == MMM_PRED_GT)
            scan_a<T, MMM_PRED_GT>(p, b, lane, wave, red, tot);
        else
            scan_a<T, MMM_PRED_ABS_GT>(p, b, lane, wave, red, tot);
    } else {
        const int64_t bw = p.N / p.NB;
        if (bw == 8)
            scan_b<T, 8>(p, b - p.n_a, lane, wave, pieces, gpos, gword);
        else if (bw == 16)
            scan_b<T, 16>(p, b - p.n_a, lane, wave, pieces, gpos, gword);
        else
            scan_b<T, 32>(p, b - p.n_a, lane, wave, pieces, gpos, gword);
    }
}

// ---- statistics (off the hot path) -----------------------------------------------------------
__global__ void mmm_stats_clear_kernel(uint64_t *stats)
{
    if (threadIdx.x < 4) stats[threadIdx.x] = 0;
}

// One workgroup per 64 values of k: lane kb of every wave counts column k of A
// over a slice of rows and row k of B over its words.
__global__ __launch_bounds__(256) void mmm_stats_kernel(const uint64_t *a_bits, const uint64_t *b_bits,
                                                        int64_t M, int64_t K, int64_t WA, int64_t WB,
                                                        int64_t bw, uint64_t *stats)
{
    __shared__ uint32_t col[4 * 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t w = blockIdx.x;
    uint32_t cnt = 0;
    for (int64_t r = wave; r < M; r += 4) cnt += (uint32_t)((a_bits[r * WA + w] >> lane) & 1ull);
    col[wave * 64 + lane] = cnt;
    __syncthreads();
    if (wave == 0) {
        const uint64_t colcount = (uint64_t)col[lane] + col[64 + lane] + col[128 + lane] + col[192 + lane];
        const int64_t k = w * 64 + lane;
        uint64_t rowcount = 0;
        if (k < K)
            for (int64_t j = 0; j < WB; ++j) rowcount += (uint64_t)__popcll(b_bits[k * WB + j]);
        uint64_t v[3] = {colcount, rowcount, colcount * rowcount * (uint64_t)bw};
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            uint64_t x = v[q];
            for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
            if (lane == 0 && x != 0) atomicAdd((unsigned long long *)&stats[q], (unsigned long long)x);
        }
    }
}

}   // namespace

// What keep_element compares against.  GT: x > t  <=>  key(x) > key(t) on the order-preserving key
// (both zeros map to the same key).  ABS_GT: |x| > t; a negative t passes every non-zero x (magnitude
// bits of x > 0), t = -0 is t = 0.  A NaN threshold passes nothing (nothing exceeds 0xffffffff).
static_assert(MMM_BT_PIECE == 16, "pieces of the transposed map are stored as 16-bit words");

static uint32_t threshold_key(int32_t pred, float threshold)
{
    union { float f; uint32_t u; } cv;
    cv.f = threshold;
    uint32_t t = cv.u;
    const uint32_t at = t & 0x7fffffffu;
    if (at > 0x7f800000u) return 0xffffffffu;
    if (pred == MMM_PRED_GT) {
        if (at == 0) t = 0;
        return (t & 0x80000000u) ? ~t : (t | 0x80000000u);
    }
    if (pred == MMM_PRED_ABS_GT) return (t & 0x80000000u) ? 0u : at;
    return 0;
}

hipError_t mmm_launch_build(const mmm_maps *m, const mmm_build_args &a, hipStream_t s)
{
    BuildParams p{};
    p.X = a.X;
    p.ldx = a.ldx;
    p.keep_a = a.keep_a;
    p.a_bits = m->a_bits;
    p.a_colany = m->a_colany;
    p.a_cnt = m->a_cnt;
    p.a_ent = reinterpret_cast<uint2 *>(m->a_ent);
    p.Y = a.Y;
    p.ldy = a.ldy;
    p.keep_rows = a.keep_rows;
    p.keep_blocks = a.keep_blocks;
    p.b_bits = m->b_bits;
    p.bt_pieces = reinterpret_cast<uint16_t *>(m->bt_bits);
    p.M = m->M;
    p.K = m->K;
    p.N = m->N;
    p.NB = m->NB;
    p.WA = m->WA;
    p.WB = m->WB;
    p.MT = m->MT;
    p.KBA = m->KBA;
    p.pred = a.pred;
    p.thr_bits = threshold_key(a.pred, a.threshold);
    const int64_t n_a = a.X ? m->MBA * m->KBA : 0;
    const int64_t n_b = a.Y ? (m->WA * (64 / MMM_BT_PIECE)) * m->WB : 0;
    if (n_a + n_b <= 0 || n_a + n_b > 0x7fffffffLL) return hipErrorInvalidValue;
    p.n_a = (uint32_t)n_a;
    const dim3 grid((uint32_t)(n_a + n_b)), block(BUILD_THREADS);
    (void)hipGetLastError();   // drop any stale error another library left on this thread
    if (a.dtype == MMM_BF16)
        hipLaunchKernelGGL(mmm_build_kernel<uint16_t>, grid, block, 0, s, p);
    else if (a.dtype == MMM_F16)
        hipLaunchKernelGGL(mmm_build_kernel<_Float16>, grid, block, 0, s, p);
    else
        hipLaunchKernelGGL(mmm_build_kernel<float>, grid, block, 0, s, p);
    return hipGetLastError();
}

hipError_t mmm_launch_stats(const mmm_maps *m, hipStream_t s)
{
    (void)hipGetLastError();
    hipLaunchKernelGGL(mmm_stats_clear_kernel, dim3(1), dim3(64), 0, s, m->stats);
    hipLaunchKernelGGL(mmm_stats_kernel, dim3((uint32_t)m->WA), dim3(256), 0, s, m->a_bits, m->b_bits, m->M,
                       m->K, m->WA, m->WB, (int64_t)m->bw, m->stats);
    return hipGetLastError();
}
