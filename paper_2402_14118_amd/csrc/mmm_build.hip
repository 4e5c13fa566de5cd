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
    uint32_t n_a;    // workgroups that scan X block by block (bitmaps and, unless row-compacted, lists)
    uint32_t n_ac;   // row-compacted mode: workgroups that list the blocks of A over the live k only
    uint32_t n_b;    // workgroups that scan Y
    // row-compacted mode (whole rows of B switched off by keep_rows): k' = 0 .. *kinfo - 1 numbers the live rows
    const uint32_t *kinfo;   // [0] = number of live k
    const uint32_t *kmap;    // k' -> k
    uint64_t *a_colany_c;    // column-any words of A over k'
    uint16_t *btc_pieces;    // transposed B map over k'
    void *Bc;                // the live rows of Y, row k' at Bc + k' * N elements (kept blocks only)
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
// MODE A_FULL: bitmap words, column-any words and the block's list, all over the original k.
// MODE A_MAPS: bitmap and column-any words only (row-compacted mode: the lists are made by A_LISTS).
// MODE A_LISTS: the block is 64 rows x 128 *live* k (k' = 128 bj ..): its elements are gathered through
//   kmap; it writes the list and the column-any words over k'.
enum { A_FULL = 0, A_MAPS = 1, A_LISTS = 2 };

template <typename T, int PRED, int MODE>
__device__ __forceinline__ void scan_a(const BuildParams &p, uint32_t b, int lane, int wave, uint64_t *red,
                                       uint32_t *tot)
{
    const int64_t bi = b / p.KBA, bj = b % p.KBA;
    const int64_t k_lo = bj * MMM_AB_COLS;
    const int64_t rbase = bi * MMM_AB_ROWS + wave * A_ROWS_PER_WAVE;
    const int64_t w_lo = k_lo / 64;
    const T *X = static_cast<const T *>(p.X);
    const int64_t klim = MODE == A_LISTS ? (int64_t)*p.kinfo : p.K;   // number of (live) k
    if (MODE == A_LISTS && k_lo >= klim) return;                      // no live k left for this block (whole workgroup)
    // Every load below is unconditional: indices are clamped into the matrix and the results masked
    // afterwards.  A load inside a branch is waited for before the next one is issued; written this way
    // the wave's 16 row pieces and its keep words are all in flight together.
    const bool has_keep = p.keep_a != nullptr;
    // keep words of the wave's 16 (row, half) pairs, one per lane 2j+h (lanes 16.. repeat them; unused)
    uint64_t kw = ~0ull;
    if (MODE != A_LISTS && has_keep) {   // wave-uniform
        const int64_t kr = min(rbase + ((lane & 15) >> 1), p.M - 1), kwd = min(w_lo + (lane & 1), p.WA - 1);
        kw = p.keep_a[kr * p.WA + kwd];
    }
    int64_t korig[A_WORDS];   // A_LISTS: the original k of this lane's two columns (-1: none)
#pragma unroll
    for (int h = 0; h < A_WORDS; ++h) {
        const int64_t k = k_lo + 64 * h + lane;
        korig[h] = k < p.K ? k : -1;
        if (MODE == A_LISTS) {
            const uint32_t km = p.kmap[min(k, p.K - 1)];
            korig[h] = k < klim ? (int64_t)km : -1;
        }
    }
    uint32_t u[A_ROWS_PER_WAVE][A_WORDS];
    uint32_t kbyte[A_ROWS_PER_WAVE][A_WORDS];   // A_LISTS with a keep bitmap: the byte that holds the element's keep bit
#pragma unroll
    for (int j = 0; j < A_ROWS_PER_WAVE; ++j) {
#pragma unroll
        for (int h = 0; h < A_WORDS; ++h) {
            const int64_t rc = min(rbase + j, p.M - 1), kc = max(korig[h], (int64_t)0);
            u[j][h] = f32_bits<T>(X[rc * p.ldx + kc]);
            kbyte[j][h] = 0xffu;
            if (MODE == A_LISTS && has_keep)   // wave-uniform
                kbyte[j][h] = reinterpret_cast<const uint8_t *>(p.keep_a)[(rc * p.WA) * 8 + (kc >> 3)];
        }
    }
    uint32_t kbit[A_ROWS_PER_WAVE] = {};   // A_LISTS: keep bits of this lane's elements, bit h of entry j
#pragma unroll
    for (int j = 0; j < A_ROWS_PER_WAVE; ++j) {
#pragma unroll
        for (int h = 0; h < A_WORDS; ++h) {
            const bool inside = rbase + j < p.M && korig[h] >= 0;
            if (!inside) u[j][h] = 0;   // +0: never kept
            if (MODE == A_LISTS) kbit[j] |= (inside ? (kbyte[j][h] >> (korig[h] & 7)) & 1u : 0u) << h;
        }
    }
    uint64_t colany[A_WORDS] = {0, 0};
    uint32_t mine_lo = 0, mine_hi = 0;   // lane 2j+h: the bitmap word of (row j, half h)
#pragma unroll
    for (int j = 0; j < A_ROWS_PER_WAVE; ++j) {
#pragma unroll
        for (int h = 0; h < A_WORDS; ++h) {
            uint64_t m;
            if (MODE == A_LISTS) {
                m = ballot64(keep_element<PRED>(u[j][h], p.thr_bits) && ((kbit[j] >> h) & 1u));
            } else {
                m = ballot64(keep_element<PRED>(u[j][h], p.thr_bits));   // lanes past K or M hold +0
                m &= ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)(kw >> 32), 2 * j + h) << 32) |
                     (uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)kw, 2 * j + h);
            }
            colany[h] |= m;
            const bool owner = __builtin_amdgcn_inverse_ballot_w64(1ull << (2 * j + h));   // lane 2j+h, as a constant mask
            mine_lo = owner ? (uint32_t)m : mine_lo;
            mine_hi = owner ? (uint32_t)(m >> 32) : mine_hi;
        }
    }
    const uint64_t mine = ((uint64_t)mine_hi << 32) | mine_lo;
    // bitmap words and per-wave entry offsets
    const bool have_word = lane < 2 * A_ROWS_PER_WAVE && rbase + (lane >> 1) < p.M && w_lo + (lane & 1) < p.WA;
    if (MODE != A_LISTS && have_word) p.a_bits[(rbase + (lane >> 1)) * p.WA + w_lo + (lane & 1)] = mine;
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
    if (MODE != A_MAPS && threadIdx.x == 0) p.a_cnt[b] = total;
    if (threadIdx.x < 2 * A_WORDS) {   // column-any words of the two 32-row tiles of this block
        const int t = threadIdx.x >> 1, h = threadIdx.x & 1;
        const int64_t tile = bi * (MMM_AB_ROWS / MMM_COLANY_ROWS) + t;
        if (tile < p.MT && w_lo + h < p.WA)
        {
            uint64_t any = 0;   // waves t*W/2 .. (t+1)*W/2-1 cover the 32 rows of tile t
            for (int w = t * (BUILD_WAVES / 2); w < (t + 1) * (BUILD_WAVES / 2); ++w) any |= red[w * A_WORDS + h];
            (MODE == A_LISTS ? p.a_colany_c : p.a_colany)[tile * p.WA + w_lo + h] = any;
        }
    }
    if (MODE == A_MAPS) return;
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
template <typename T> __device__ __forceinline__ T raw_zero();
template <> __device__ __forceinline__ float raw_zero<float>() { return 0.f; }
template <> __device__ __forceinline__ uint16_t raw_zero<uint16_t>() { return 0; }
template <> __device__ __forceinline__ _Float16 raw_zero<_Float16>() { return (_Float16)0; }

// COMPACT (row-compacted mode): the workgroup's 16 rows are the live rows k' = 16 piece ..; they are read
// through kmap, their kept blocks are copied to row k' of Bc, and the transposed map over k' is written
// instead of b_bits and the transposed map over k (which the plain workgroups write).
template <typename T, int BW, bool COMPACT>
__device__ __forceinline__ void scan_b(const BuildParams &p, uint32_t bb, int lane, int wave, uint32_t *pieces,
                                       uint8_t (*gpos)[B_ROWS_PER_WAVE][64], uint64_t (*gword)[B_ROWS_PER_WAVE])
{
    constexpr int BPL = 64 / BW;   // blocks covered by one 64-lane load
    const int64_t piece = bb / p.WB, w = bb % p.WB;
    const int64_t kbase = piece * MMM_BT_PIECE + wave * B_ROWS_PER_WAVE;
    const T *Y = static_cast<const T *>(p.Y);
    const int64_t klive = COMPACT ? (int64_t)*p.kinfo : 0;
    // pieces past the last 128-step that holds a live k are never looked at (whole workgroup leaves)
    if (COMPACT && piece * MMM_BT_PIECE >= (klive + MMM_AB_COLS - 1) / MMM_AB_COLS * MMM_AB_COLS) return;
    const int64_t nb_left = p.NB - w * 64;
    const uint64_t valid = nb_left >= 64 ? ~0ull : ((1ull << nb_left) - 1ull);
    uint32_t piece_bits = 0;
    // which blocks of the wave's rows the keep bitmaps leave switched on: lane r fetches the two
    // keep words of row r, so that all of them are in flight together
    uint64_t krw = ~0ull, kbw = ~0ull;
    int64_t krow = -1;   // lane r: the row of Y behind the wave's row r (-1: none)
    {
        const int64_t kl = kbase + lane;
        const int64_t kmapped = COMPACT ? (int64_t)p.kmap[min(kl, p.K - 1)] : kl;   // loaded unconditionally
        if (lane < B_ROWS_PER_WAVE && kl < (COMPACT ? klive : p.K)) krow = kmapped;
        const bool mine = krow >= 0;
        const int64_t kc = max(krow, (int64_t)0);   // unconditional loads at clamped rows, masked below
        if (p.keep_rows != nullptr) krw = p.keep_rows[kc >> 6];        // wave-uniform branches
        if (p.keep_blocks != nullptr) kbw = p.keep_blocks[kc * p.WB + w];
        if (!mine) krw = kbw = ~0ull;
    }
    uint64_t kept[B_ROWS_PER_WAVE];
    int64_t korig[B_ROWS_PER_WAVE];
#pragma unroll
    for (int r = 0; r < B_ROWS_PER_WAVE; ++r) {
        korig[r] = ((int64_t)__builtin_amdgcn_readlane((int32_t)(krow >> 32), r) << 32) |
                   (int64_t)(uint32_t)__builtin_amdgcn_readlane((int32_t)krow, r);
    }
#pragma unroll
    for (int r = 0; r < B_ROWS_PER_WAVE; ++r) {
        const int64_t k = korig[r];
        const uint64_t kr = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)(krw >> 32), r) << 32) |
                            (uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)krw, r);
        const uint64_t kb = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)(kbw >> 32), r) << 32) |
                            (uint64_t)(uint32_t)__builtin_amdgcn_readlane((uint32_t)kbw, r);
        kept[r] = k >= 0 ? valid & kb & (0ull - ((kr >> (k & 63)) & 1ull)) : 0ull;
    }
    constexpr int PER = BW <= 8 ? BW : 8;     // loads in flight per lane and row
#pragma unroll
    for (int r = 0; r < B_ROWS_PER_WAVE; ++r) {
        const int64_t k = korig[r];
        uint64_t word = 0;
        if (kept[r] != 0) {
            const T *row = Y + k * p.ldy + w * 64 * BW;
            T *crow = COMPACT ? static_cast<T *>(p.Bc) + (kbase + r) * p.N + w * 64 * BW : nullptr;
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
                // Loads are unconditional, so that all of them are in flight together (a load inside a
                // branch is waited for at once): slots past the end of the list read the first listed
                // block again, which is a block that may be read, and are masked afterwards.
                uint32_t u[ROUNDS];
                int pos[ROUNDS];
                T raw[ROUNDS];
#pragma unroll
                for (int t = 0; t < ROUNDS; ++t) {
                    const int j = t * BPL + slot;
                    const int pj = (int)plist[j < nkept ? j : 0];
                    pos[t] = j < nkept ? pj : -1;
                    raw[t] = row[pj * BW + lane % BW];
                }
#pragma unroll
                for (int t = 0; t < ROUNDS; ++t) {
                    u[t] = pos[t] >= 0 ? f32_bits<T>(raw[t]) : 0u;
                    if (COMPACT && pos[t] >= 0) crow[pos[t] * BW + lane % BW] = raw[t];
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
                    // unconditional loads (see above): lanes whose block is switched off read the first
                    // switched-on block of the word instead, and are masked afterwards
                    uint32_t u[PER];
                    T raw[PER];
                    const int first_on = __builtin_ctzll(kept[r]) * BW + lane % BW;
#pragma unroll
                    for (int j = 0; j < PER; ++j) {
                        const int blk = (j0 + j) * BPL + lane / BW;   // block (inside this word) of this lane's element
                        raw[j] = row[(kept[r] >> blk) & 1ull ? (j0 + j) * 64 + lane : first_on];
                    }
#pragma unroll
                    for (int j = 0; j < PER; ++j) {
                        const int blk = (j0 + j) * BPL + lane / BW;
                        const bool on = (kept[r] >> blk) & 1ull;
                        u[j] = on ? f32_bits<T>(raw[j]) : 0u;
                        if (COMPACT && on) crow[(j0 + j) * 64 + lane] = raw[j];
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
        if (!COMPACT && k >= 0 && lane == 0) p.b_bits[k * p.WB + w] = word;
        piece_bits |= (uint32_t)((word >> lane) & 1ull) << (wave * B_ROWS_PER_WAVE + r);
    }
    pieces[wave * 64 + lane] = piece_bits;
    __syncthreads();
    if (wave == 0) {
        uint32_t v = 0;
        for (int w = 0; w < BUILD_WAVES; ++w) v |= pieces[w * 64 + lane];
        const int64_t blk = w * 64 + lane;
        if (blk < p.NB) (COMPACT ? p.btc_pieces : p.bt_pieces)[blk * (p.WA * (64 / MMM_BT_PIECE)) + piece] = (uint16_t)v;
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
    // workgroup ranges: [blocks of A over k | blocks of A over the live k | rows of Y | live rows of Y]
    if (b < p.n_a + p.n_ac) {
        const bool lists = b >= p.n_a;   // row-compacted mode: the second range makes the lists
        const uint32_t ba = lists ? b - p.n_a : b;
        if (p.n_ac == 0) {
            if (p.pred == MMM_PRED_NONZERO)
                scan_a<T, MMM_PRED_NONZERO, A_FULL>(p, ba, lane, wave, red, tot);
            else if (p.pred == MMM_PRED_GT)
                scan_a<T, MMM_PRED_GT, A_FULL>(p, ba, lane, wave, red, tot);
            else
                scan_a<T, MMM_PRED_ABS_GT, A_FULL>(p, ba, lane, wave, red, tot);
        } else if (!lists) {
            if (p.pred == MMM_PRED_NONZERO)
                scan_a<T, MMM_PRED_NONZERO, A_MAPS>(p, ba, lane, wave, red, tot);
            else if (p.pred == MMM_PRED_GT)
                scan_a<T, MMM_PRED_GT, A_MAPS>(p, ba, lane, wave, red, tot);
            else
                scan_a<T, MMM_PRED_ABS_GT, A_MAPS>(p, ba, lane, wave, red, tot);
        } else {
            if (p.pred == MMM_PRED_NONZERO)
                scan_a<T, MMM_PRED_NONZERO, A_LISTS>(p, ba, lane, wave, red, tot);
            else if (p.pred == MMM_PRED_GT)
                scan_a<T, MMM_PRED_GT, A_LISTS>(p, ba, lane, wave, red, tot);
            else
                scan_a<T, MMM_PRED_ABS_GT, A_LISTS>(p, ba, lane, wave, red, tot);
        }
    } else {
        const uint32_t bb = b - p.n_a - p.n_ac;
        const int64_t bw = p.N / p.NB;
        if (bb < p.n_b) {
            if (bw == 8)
                scan_b<T, 8, false>(p, bb, lane, wave, pieces, gpos, gword);
            else if (bw == 16)
                scan_b<T, 16, false>(p, bb, lane, wave, pieces, gpos, gword);
            else
                scan_b<T, 32, false>(p, bb, lane, wave, pieces, gpos, gword);
        } else {
            if (bw == 8)
                scan_b<T, 8, true>(p, bb - p.n_b, lane, wave, pieces, gpos, gword);
            else if (bw == 16)
                scan_b<T, 16, true>(p, bb - p.n_b, lane, wave, pieces, gpos, gword);
            else
                scan_b<T, 32, true>(p, bb - p.n_b, lane, wave, pieces, gpos, gword);
        }
    }
}

// Row-compacted mode: number the rows of B that keep_rows leaves on.  One workgroup: every thread
// counts a contiguous run of map words, a prefix sum over the threads places the runs, and every
// thread then writes out the positions of its own bits:  kmap[k'] = k.  kinfo[0] = number of live k.
__global__ __launch_bounds__(1024) void mmm_kmap_kernel(const uint64_t *keep_rows, int64_t K, int64_t WA, uint32_t *kinfo,
                                                        uint32_t *kmap)
{
    __shared__ uint32_t sums[1024];
    const int t = threadIdx.x;
    const int64_t per = (WA + 1023) / 1024;
    const int64_t w0 = (int64_t)t * per, w1 = min(WA, w0 + per);
    auto word = [&](int64_t w) -> uint64_t {
        uint64_t m = keep_rows[w];
        const int64_t left = K - w * 64;   // bits past K do not count
        if (left < 64) m &= (1ull << left) - 1ull;
        return m;
    };
    uint32_t cnt = 0;
    for (int64_t w = w0; w < w1; ++w) cnt += (uint32_t)__popcll(word(w));
    sums[t] = cnt;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {   // inclusive prefix sum in LDS
        const uint32_t o = t >= d ? sums[t - d] : 0u;
        __syncthreads();
        sums[t] += o;
        __syncthreads();
    }
    uint32_t pos = sums[t] - cnt;
    for (int64_t w = w0; w < w1; ++w) {
        uint64_t m = word(w);
        while (m != 0) {
            kmap[pos++] = (uint32_t)(w * 64 + __builtin_ctzll(m));
            m &= m - 1;
        }
    }
    if (t == 1023) kinfo[0] = sums[1023];
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
    p.kinfo = m->kinfo;
    p.kmap = m->kmap;
    p.a_colany_c = m->a_colany_c;
    p.btc_pieces = reinterpret_cast<uint16_t *>(m->btc_bits);
    p.Bc = m->Bc;
    const int64_t n_a = a.X ? m->MBA * m->KBA : 0;
    const int64_t n_ac = a.X && a.a_compact ? n_a : 0;
    const int64_t n_b = a.Y ? (m->WA * (64 / MMM_BT_PIECE)) * m->WB : 0;
    const int64_t n_bc = a.Y && a.b_compact ? n_b : 0;
    const int64_t n_all = n_a + n_ac + n_b + n_bc;
    if (n_all <= 0 || n_all > 0x7fffffffLL) return hipErrorInvalidValue;
    p.n_a = (uint32_t)n_a;
    p.n_ac = (uint32_t)n_ac;
    p.n_b = (uint32_t)n_b;
    const dim3 grid((uint32_t)n_all), block(BUILD_THREADS);
    (void)hipGetLastError();   // drop any stale error another library left on this thread
    if (a.Y && a.b_compact) {   // number the live rows first: the scans below read the numbering
        hipLaunchKernelGGL(mmm_kmap_kernel, dim3(1), dim3(1024), 0, s, a.keep_rows, m->K, m->WA, m->kinfo, m->kmap);
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
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
