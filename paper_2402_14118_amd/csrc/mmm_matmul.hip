// Masked GEMM:  C[i,j] = sum over k with a_bits[i,k] & b_bits[k, j div bw] of X[i,k] * Y[k,j]
// (paper, section 3 "Matrix Multiplication", Fig. "MMM Pseudocode").
//
// How the skipping is mapped onto a 64-lane wavefront.  The paper's conclusion
// notes that on a GPU all lanes of a wave must work on the same pattern of B
// rows and A elements.  Here the unit a wave owns is a 16-column group of C
// (one B block for bw = 16).  For that group the occupied rows k of B are known
// from the transposed B map, so the wave walks a *compacted* list of k: every
// step takes four listed k, gathers the 4 x 16 slab of occupied B blocks and the
// matching 16 x 4 slab of A, and issues one 16x16x4 fp32 MFMA per 16 rows.  B's
// block sparsity is skipped exactly: no unoccupied block is ever loaded or
// multiplied.  The iteration over the list is uniform across the wave: no
// lane-divergent branch exists in the inner loop.
//
// A's element sparsity is used where it pays on this machine, in data movement:
// only the non-zero elements of A travel.  The map builder lists, per block of
// 64 rows x 128 columns, the count of non-zeros with their offsets and values
// (the blocked sparse row structure of section 3, "Optimizations").  A
// workgroup owns 64 rows of C; per 128-wide step of k it scatters that block's
// list into a zeroed LDS slab, which all of its waves then read as the dense
// 16 x 4 MFMA operand; afterwards it zeroes the same positions again.  Columns
// of the slab that are zero for all 64 rows are dropped from the k lists
// (column-any words).
//
// Pipeline: while step c is multiplied, the list entries of step c+1 are in
// flight into registers, the k lists of step c+1 are built, and its first B
// operands are in flight too; inside a k list the B operands of the next batch
// are requested before the current batch is multiplied.  The map words and
// block counts a workgroup needs are copied to LDS in windows of many steps.
#include "mmm_internal.h"

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int TM = MMM_AB_ROWS;   // rows of C per workgroup = rows of a block of A
constexpr int KC = MMM_AB_COLS;   // k per step = columns of a block of A
constexpr int KCP = MMM_SLAB_LD;  // LDS row pitch; column KC stays zero (the A operand of a k-list slot past the end)
constexpr int WPC = KC / 64;      // map words per step
constexpr int QB = 4;             // k-list quads per batch
constexpr int LPAD = 4 * QB;


struct MatmulParams {
    const void *Y;
    int64_t ldy;
    float *C;
    int64_t ldc;
    float *P;   // split-K partial sums, [split][M][N]
    const uint32_t *a_cnt;
    const uint2 *a_ent;
    const uint64_t *a_colany;
    const uint64_t *b_bits;
    const uint64_t *bt_bits;
    int64_t M, K, N, NB, WA, WB, MT, KBA;
    int32_t bw;
    int32_t tiles_m, tiles_n, split_k, chunks_total, chunks_per_split;
    int32_t window_chunks;   // steps whose map words and counts are held in LDS at a time
    int32_t accumulate;
};

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<uint16_t>(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// Workgroups are dealt round-robin to the 8 XCDs.  Re-number them so that each
// XCD works on a contiguous range of logical tiles: neighbours in that range
// share the same block row of A and neighbouring column tiles of B, which then
// stay in that XCD's L2.
__device__ __forceinline__ uint32_t xcd_contiguous_id(uint32_t b, uint32_t n)
{
    const uint32_t x = b & 7u, i = b >> 3, q = n >> 3, rem = n & 7u;
    return x * q + (x < rem ? x : rem) + i;
}

// [NG][nwords] 64-bit words (per group: transposed-B word AND column-any word of A),
// followed by window_chunks 32-bit block counts
extern __shared__ uint64_t mmm_dyn_words[];

// RT  16-row MFMA sub-tiles computed (4: all 64 rows of the block; 2: matrices of at most 32 rows)
// GW  16-column groups per wave, NW waves per workgroup: TN = 16*GW*NW columns
template <int RT, int GW, int NW, typename T, bool BW8>
__global__ __launch_bounds__(NW * 64) void mmm_matmul_kernel(const MatmulParams p)
{
    constexpr int NG = NW * GW;
    constexpr int NT = NW * 64;
    constexpr int EPT = 1024 / NT;    // list entries of A per thread and round
    constexpr int ROUND = NT * EPT;   // list entries one round of the workgroup moves

    __shared__ __align__(16) float As[TM * KCP];
    __shared__ uint8_t lists[NW][64 * 64 + 4];   // per wave: k lists of its groups for one window

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, s = lane >> 4;

    const uint32_t L = xcd_contiguous_id(blockIdx.x, gridDim.x);
    const int tile_n = (int)(L % (uint32_t)p.tiles_n);
    const int split = (int)((L / (uint32_t)p.tiles_n) % (uint32_t)p.split_k);
    const int tile_m = (int)(L / ((uint32_t)p.tiles_n * (uint32_t)p.split_k));
    const int64_t row0 = (int64_t)tile_m * TM;
    const int chunk_begin = split * p.chunks_per_split;
    const int chunk_end = min(chunk_begin + p.chunks_per_split, p.chunks_total);
    const int nwords = p.window_chunks * WPC;
    uint32_t *cnt_lds = reinterpret_cast<uint32_t *>(mmm_dyn_words + NG * nwords);

    const T *Y = static_cast<const T *>(p.Y);
    const uint32_t ldy32 = (uint32_t)p.ldy;

    floatx4 acc[GW][RT];
#pragma unroll
    for (int g = 0; g < GW; ++g)
#pragma unroll
        for (int r = 0; r < RT; ++r) acc[g][r] = floatx4{0.f, 0.f, 0.f, 0.f};

    // the slab starts out all zero and every step leaves it all zero again
    for (int i = tid; i < TM * KCP / 4; i += NT) reinterpret_cast<floatx4 *>(As)[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    int wbegin = chunk_begin;   // first step of the current window

    // map words and block counts of the steps [wb, wb + window_chunks) -> LDS
    auto load_words = [&](int wb) {
        for (int idx = tid; idx < NG * nwords; idx += NT) {
            const int gi = idx / nwords, wi = idx % nwords;
            const int64_t widx = (int64_t)wb * WPC + wi;
            const int64_t G = (int64_t)tile_n * NG + gi;   // global 16-column group
            uint64_t m = 0;
            if (widx < p.WA && G * 16 < p.N) {
                if (p.bw == 16) {
                    m = p.bt_bits[G * p.WA + widx];
                } else if (p.bw == 32) {
                    m = p.bt_bits[(G >> 1) * p.WA + widx];
                } else {
                    m = p.bt_bits[(2 * G) * p.WA + widx];
                    if (2 * G + 1 < p.NB) m |= p.bt_bits[(2 * G + 1) * p.WA + widx];
                }
                uint64_t any = 0;   // k whose column of A is zero in all rows of this tile are dropped
#pragma unroll
                for (int t = 0; t < RT * 16 / MMM_COLANY_ROWS; ++t) {
                    const int64_t tt = row0 / MMM_COLANY_ROWS + t;
                    if (tt < p.MT) any |= p.a_colany[tt * p.WA + widx];
                }
                m &= any;
            }
            mmm_dyn_words[idx] = m;
        }
        for (int i = tid; i < p.window_chunks; i += NT)
            cnt_lds[i] = wb + i < p.chunks_total ? p.a_cnt[(int64_t)tile_m * p.KBA + wb + i] : 0u;
    };

    // One round of a block's non-zero list, in registers: entry tid + j * NT is entry j of this
    // thread.  The builder pads every list to a multiple of 64, so whether a wave has an entry j
    // is a wave-uniform question.
    struct Entries {
        uint32_t pos[EPT];   // byte offset inside the slab
        uint32_t val[EPT];   // float bit pattern
        int cnt;             // entries of the block, rounded up to whole wavefronts
    };
    // First batch of B operands of one step, per group of this wave.
    struct BFirst {
        float b[GW][QB];
        int kk[GW][QB];      // the listed k they belong to
        int cnt[GW], start[GW];
    };
    Entries ecur, eP, eQ;
    BFirst bP, bQ;
    ecur.cnt = 0;

    const int wave_e0 = wave * 64;
    char *slab = reinterpret_cast<char *>(As);
    // request the first round of list entries of step ci (relative to the window)
    auto issue_entries = [&](int ci, Entries &e) {
        e.cnt = ((int)cnt_lds[ci] + 63) & ~63;
        const uint2 *ent = p.a_ent + ((size_t)tile_m * p.KBA + wbegin + ci) * MMM_AB_CAP + tid;
        // Loaded unconditionally (a round always lies inside the block's list area); what lies
        // past the padded count is never used.  No branch, so nothing here waits for the data.
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const uint2 v = ent[j * NT];
            e.pos[j] = v.x;
            e.val[j] = v.y;
        }
    };
    // The slab is filled and emptied with integer adds on the float bit patterns: a cell goes
    // 0 -> bits -> 0 exactly, whatever the order in which the adds of different threads land, so
    // emptying step c and filling step c+1 need no barrier between them.
    auto slab_add = [&](uint32_t pos, uint32_t v) {
        __hip_atomic_fetch_add(reinterpret_cast<uint32_t *>(slab + pos), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    // blocks with more entries than one round: the rest is fetched and applied on the spot
    auto apply_rest = [&](int ci, int cnt, bool fill) {
        const uint2 *ent = p.a_ent + ((size_t)tile_m * p.KBA + wbegin + ci) * MMM_AB_CAP;
        for (int e = ROUND + tid; e < cnt; e += NT) {
            const uint2 v = ent[e];
            slab_add(v.x, fill ? v.y : 0u - v.y);
        }
    };
    auto fill_slab = [&](int ci, const Entries &e) {
#pragma unroll
        for (int j = 0; j < EPT; ++j)
            if (wave_e0 + j * NT < e.cnt) slab_add(e.pos[j], e.val[j]);
        if (e.cnt > ROUND) apply_rest(ci, e.cnt, true);
    };
    auto empty_slab = [&](int ci, const Entries &e) {
#pragma unroll
        for (int j = 0; j < EPT; ++j)
            if (wave_e0 + j * NT < e.cnt) slab_add(e.pos[j], 0u - e.val[j]);
        if (e.cnt > ROUND) apply_rest(ci, e.cnt, false);
    };

    // ---- k lists.  Once per window every wave turns the map words of its groups into compacted
    // lists of live k: lane (g, w) owns word w of group g, a segmented prefix sum of the popcounts
    // gives every word its place in the list of its group, and each lane then writes out the bit
    // positions of its own word.  Entries are step-relative k (0..127); the entries of one step
    // are contiguous, and `pref` (read with readlane) tells where each step starts.
    constexpr int SEG = 64 / GW;          // lanes (= map words) per group: SEG / WPC steps per window
    constexpr int REGION = SEG * 64;      // list bytes per group: the worst case
    uint32_t pref = 0, incl = 0;          // exclusive / inclusive popcount prefix of this lane's word inside its group
    auto build_lists = [&](int nchunks) {
        const int g = lane / SEG, wi = lane % SEG;
        uint64_t m = wi < nchunks * WPC ? mmm_dyn_words[(wave * GW + g) * nwords + wi] : 0ull;
        const uint32_t cnt = (uint32_t)__popcll(m);
        incl = cnt;
#pragma unroll
        for (int d = 1; d < SEG; d <<= 1) {
            const uint32_t o = __shfl_up(incl, d, 64);
            if (wi >= d) incl += o;
        }
        pref = incl - cnt;
        uint8_t *dst = &lists[wave][g * REGION + pref];
        const uint32_t half = (uint32_t)(wi % WPC) * 64u;
        while (m != 0) {   // as many rounds as the fullest word of the wave has bits
            *dst++ = (uint8_t)(half + (uint32_t)__ffsll((unsigned long long)m) - 1u);
            m &= m - 1;
        }
    };
    // first list slot and number of live k of step ci for group g
    auto step_range = [&](int ci, int g, int &start, int &n) {
        start = (int)__builtin_amdgcn_readlane(pref, g * SEG + ci * WPC);
        n = (int)__builtin_amdgcn_readlane(incl, g * SEG + ci * WPC + WPC - 1) - start;
    };

    // B operands.  Every load is unconditional and in bounds: a slot past the end of the list
    // re-reads the last listed row (its A operand is the zero column of the slab, so the product
    // vanishes), and lanes past column N re-read column N-1 (their results are never written).
    const int64_t col_base = ((int64_t)tile_n * NG + wave * GW) * 16 + c;   // column of this lane in its first group
    int coff[GW];
#pragma unroll
    for (int g = 0; g < GW; ++g) coff[g] = (int)(min(col_base + g * 16, p.N - 1) - col_base);
    auto load_b = [&](const T *Yc, int64_t k0, int kb, int g) -> float {
        float v = to_f32<T>(Yc[(int)__umul24((uint32_t)kb, ldy32) + coff[g]]);
        if (BW8) {   // a group spans two blocks: take only this lane's own block
            const int64_t blk = (col_base + coff[g]) >> 3;
            if (!((p.b_bits[(k0 + kb) * p.WB + (blk >> 6)] >> (blk & 63)) & 1ull)) v = 0.f;
        }
        return v;
    };
    // list slot t of a step with n live k: the listed k, clamped to the last one
    auto list_k = [&](const uint8_t *lst, int t, int n) -> int { return lst[min(t, n - 1)]; };
    auto issue_b_first = [&](int ci, BFirst &f) {
        const int64_t k0 = (int64_t)(wbegin + ci) * KC;
        const T *Yc = Y + k0 * p.ldy + col_base;
#pragma unroll
        for (int g = 0; g < GW; ++g) {
            step_range(ci, g, f.start[g], f.cnt[g]);
            if (f.cnt[g] > 0) {
                const uint8_t *lst = &lists[wave][g * REGION + f.start[g]];
#pragma unroll
                for (int u = 0; u < QB; ++u) {
                    f.kk[g][u] = list_k(lst, 4 * u + s, f.cnt[g]);
                    f.b[g][u] = load_b(Yc, k0, f.kk[g][u], g);
                }
            }
        }
    };

    // ---- multiply step ci: 4 listed k per MFMA
    auto multiply = [&](int ci, const BFirst &f) {
        const int64_t k0 = (int64_t)(wbegin + ci) * KC;
        const T *Yc = Y + k0 * p.ldy + col_base;
        // First batch of every group: the listed k are already in registers, so all A operands
        // are requested at once, then multiplied.
        {
            float a[GW][QB][RT];
#pragma unroll
            for (int g = 0; g < GW; ++g) {
#pragma unroll
                for (int u = 0; u < QB; ++u) {
                    if (4 * u < f.cnt[g]) {
                        const int kk = 4 * u + s < f.cnt[g] ? f.kk[g][u] : KC;   // KC: the zero column
#pragma unroll
                        for (int r = 0; r < RT; ++r) a[g][u][r] = As[c * KCP + kk + r * 16 * KCP];
                    }
                }
            }
#pragma unroll
            for (int g = 0; g < GW; ++g) {
#pragma unroll
                for (int u = 0; u < QB; ++u) {
                    if (4 * u < f.cnt[g]) {
#pragma unroll
                        for (int r = 0; r < RT; ++r)
                            acc[g][r] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[g][u][r], f.b[g][u], acc[g][r], 0, 0, 0);
                    }
                }
            }
        }
        // further batches of long lists: B operands one batch ahead
#pragma unroll
        for (int g = 0; g < GW; ++g) {
            const int n = f.cnt[g];
            if (n <= LPAD) continue;
            const uint8_t *lst = &lists[wave][g * REGION + f.start[g]];
            float b[QB];
#pragma unroll
            for (int u = 0; u < QB; ++u) b[u] = load_b(Yc, k0, list_k(lst, LPAD + 4 * u + s, n), g);
            for (int q = LPAD; q < n; q += LPAD) {
                float bn[QB];
                if (q + LPAD < n) {
#pragma unroll
                    for (int u = 0; u < QB; ++u) bn[u] = load_b(Yc, k0, list_k(lst, q + LPAD + 4 * u + s, n), g);
                } else {
#pragma unroll
                    for (int u = 0; u < QB; ++u) bn[u] = 0.f;
                }
                float a[QB][RT];
#pragma unroll
                for (int u = 0; u < QB; ++u) {
                    const int t = q + 4 * u + s;
                    const int kk = t < n ? (int)lst[min(t, n - 1)] : KC;
#pragma unroll
                    for (int r = 0; r < RT; ++r) a[u][r] = As[c * KCP + kk + r * 16 * KCP];
                }
#pragma unroll
                for (int u = 0; u < QB; ++u) {
                    if (q + 4 * u < n) {
#pragma unroll
                        for (int r = 0; r < RT; ++r)
                            acc[g][r] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u][r], b[u], acc[g][r], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int u = 0; u < QB; ++u) b[u] = bn[u];
            }
        }
    };

    // One step.  On entry the slab holds block ci; `have` holds the list of block ci+1 (requested
    // a step ago), `load` is free and receives the request for block ci+2; likewise the B
    // operands of step ci are in `use` and those of step ci+1 are requested into `next`.
    auto do_step = [&](int ci, int nchunks, Entries &have, Entries &load, const BFirst &use, BFirst &next) {
        if (ci + 2 < nchunks) issue_entries(ci + 2, load);
        if (ci + 1 < nchunks) issue_b_first(ci + 1, next);
        multiply(ci, use);
        __syncthreads();   // every wave is done reading the slab of step ci
        empty_slab(ci, ecur);
        if (ci + 1 < nchunks) {
            fill_slab(ci + 1, have);
            ecur = have;
        }
        __syncthreads();   // the slab holds block ci+1 (or is all zero after the last step)
    };

    // K range of this workgroup, in windows of SEG / WPC steps
    for (wbegin = chunk_begin; wbegin < chunk_end; wbegin += p.window_chunks) {
        const int nchunks = min(p.window_chunks, chunk_end - wbegin);
        __syncthreads();   // previous window fully consumed; the slab is all zero
        load_words(wbegin);
        __syncthreads();
        build_lists(nchunks);
        issue_entries(0, ecur);
        if (nchunks > 1) issue_entries(1, eP);
        issue_b_first(0, bP);
        fill_slab(0, ecur);
        __syncthreads();
        for (int ci = 0; ci < nchunks; ci += 2) {
            do_step(ci, nchunks, eP, eQ, bP, bQ);
            if (ci + 1 < nchunks) do_step(ci + 1, nchunks, eQ, eP, bQ, bP);
        }
    }

    // ---- write C (or this split's partial sums): every element exactly once.
    // Accumulator layout of the 16x16x4 MFMA: lane holds rows 4*s + v (v = 0..3) of column c.
    // Each wave first lays its 16*RT x 16*GW tile out row-major in its own piece of the (now
    // free) slab, then stores whole rows with 16-byte lanes, so full cache lines leave the CU.
    float *out = p.split_k > 1 ? p.P + (int64_t)split * p.M * p.N : p.C;
    const int64_t ldo = p.split_k > 1 ? p.N : p.ldc;
    const bool add = p.split_k == 1 && p.accumulate;
    const int64_t wcol0 = ((int64_t)tile_n * NG + wave * GW) * 16;   // first column of this wave
    constexpr int WCOLS = 16 * GW;
    constexpr bool FITS = NW * RT * 16 * WCOLS <= TM * KCP;
    const bool vec_ok = FITS && (reinterpret_cast<uintptr_t>(out) % 16 == 0) && (ldo % 4 == 0) && wcol0 + WCOLS <= p.N;
    if (vec_ok) {
        float *mine = As + wave * (RT * 16 * WCOLS);
#pragma unroll
        for (int g = 0; g < GW; ++g)
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int v = 0; v < 4; ++v) mine[(r * 16 + s * 4 + v) * WCOLS + g * 16 + c] = acc[g][r][v];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        constexpr int V4 = WCOLS / 4;                  // 16-byte pieces per row
        constexpr int ROWS_PER_PASS = 64 / V4;
#pragma unroll
        for (int pass = 0; pass < RT * 16 / ROWS_PER_PASS; ++pass) {
            const int rr = pass * ROWS_PER_PASS + lane / V4, c4 = lane % V4;
            const int64_t row = row0 + rr;
            if (row < p.M) {
                floatx4 val = *reinterpret_cast<const floatx4 *>(&mine[rr * WCOLS + 4 * c4]);
                floatx4 *dst = reinterpret_cast<floatx4 *>(out + row * ldo + wcol0 + 4 * c4);
                if (add) val += *dst;
                *dst = val;
            }
        }
    } else {
#pragma unroll
        for (int g = 0; g < GW; ++g) {
            const int64_t col = wcol0 + g * 16 + c;
            if (col >= p.N) continue;
#pragma unroll
            for (int r = 0; r < RT; ++r) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int64_t row = row0 + r * 16 + s * 4 + v;
                    if (row >= p.M) continue;
                    float *dst = out + row * ldo + col;
                    *dst = add ? *dst + acc[g][r][v] : acc[g][r][v];
                }
            }
        }
    }
}

// Sum of the split-K partials in a fixed order (split 0, 1, ...), so the result
// does not depend on the order in which workgroups finish.
__global__ __launch_bounds__(256) void mmm_splitk_reduce_kernel(const float *P, float *C, int64_t ldc, int64_t M,
                                                                int64_t N, int32_t splits, int32_t accumulate)
{
    const int64_t total = M * N;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = e / N, col = e % N;
        float sum = P[e];
        for (int sp = 1; sp < splits; ++sp) sum += P[(int64_t)sp * total + e];
        float *dst = C + row * ldc + col;
        *dst = accumulate ? *dst + sum : sum;
    }
}

typedef void (*matmul_kernel_fn)(const MatmulParams);

struct VariantEntry {
    mmm_variant_info info;
    matmul_kernel_fn f32, bf16, f32_bw8, bf16_bw8;
};

#define MMM_VARIANT(RT, GW, NW)                                                                             \
    {                                                                                                       \
        {"R" #RT "x16_TN" #GW "x" #NW "x16", TM, 16 * GW * NW, KC, NW * 64, NW * GW, 16 * RT},                 \
            mmm_matmul_kernel<RT, GW, NW, float, false>, mmm_matmul_kernel<RT, GW, NW, uint16_t, false>,     \
            mmm_matmul_kernel<RT, GW, NW, float, true>, mmm_matmul_kernel<RT, GW, NW, uint16_t, true>        \
    }

const VariantEntry g_variants[] = {
    MMM_VARIANT(4, 2, 4),   // 0: 64 x 128
    MMM_VARIANT(4, 4, 4),   // 1: 64 x 256
    MMM_VARIANT(4, 1, 4),   // 2: 64 x 64
    MMM_VARIANT(4, 1, 8),   // 3: 64 x 128, eight waves
    MMM_VARIANT(4, 2, 8),   // 4: 64 x 256, eight waves
    MMM_VARIANT(2, 2, 4),   // 5: 32 x 128   (matrices of at most 32 rows)
    MMM_VARIANT(2, 4, 4),   // 6: 32 x 256
    MMM_VARIANT(2, 1, 4),   // 7: 32 x 64
};
constexpr int32_t kVariants = (int32_t)(sizeof(g_variants) / sizeof(g_variants[0]));

}   // namespace

int32_t mmm_variant_count() { return kVariants; }
const mmm_variant_info &mmm_variant(int32_t i) { return g_variants[i].info; }

hipError_t mmm_launch_matmul(const mmm_maps *m, const mmm_plan &pl, int32_t dtype, const void *X, int64_t ldx,
                             const void *Y, int64_t ldy, float *C, int64_t ldc, int32_t accumulate, hipStream_t s)
{
    (void)X;   // the non-zero values of A travel inside the map (they were copied from X when it was built)
    (void)ldx;
    if (pl.variant < 0 || pl.variant >= kVariants) return hipErrorInvalidValue;
    const VariantEntry &v = g_variants[pl.variant];
    if (m->M > v.info.rows && v.info.rows < TM) return hipErrorInvalidValue;
    MatmulParams p{};
    p.Y = Y;
    p.ldy = ldy;
    p.C = C;
    p.ldc = ldc;
    p.P = m->partials;
    p.a_cnt = m->a_cnt;
    p.a_ent = reinterpret_cast<const uint2 *>(m->a_ent);
    p.a_colany = m->a_colany;
    p.b_bits = m->b_bits;
    p.bt_bits = m->bt_bits;
    p.M = m->M;
    p.K = m->K;
    p.N = m->N;
    p.NB = m->NB;
    p.WA = m->WA;
    p.WB = m->WB;
    p.MT = m->MT;
    p.KBA = m->KBA;
    p.bw = m->bw;
    p.tiles_m = pl.tiles_m;
    p.tiles_n = pl.tiles_n;
    p.split_k = pl.split_k;
    p.chunks_total = pl.chunks_total;
    p.chunks_per_split = pl.chunks_per_split;
    p.accumulate = accumulate;
    if (pl.workgroups <= 0 || pl.workgroups > 0x7fffffffLL) return hipErrorInvalidValue;
    if (pl.split_k > 1 && (size_t)pl.split_k * (size_t)m->M * (size_t)m->N * sizeof(float) > m->partial_bytes)
        return hipErrorInvalidValue;
    const int64_t per_chunk = (int64_t)v.info.groups * WPC * sizeof(uint64_t) + sizeof(uint32_t);
    const int64_t gw = v.info.groups / (v.info.threads / 64);
    int64_t window = 64 / (gw * WPC);   // one map word per lane: 64 words per wave and window
    if (window > pl.chunks_per_split) window = pl.chunks_per_split;
    if (window < 1) return hipErrorInvalidValue;
    p.window_chunks = (int32_t)window;
    const size_t dyn = (size_t)(window * per_chunk + 7) / 8 * 8;
    matmul_kernel_fn fn = m->bw == 8 ? (dtype == MMM_BF16 ? v.bf16_bw8 : v.f32_bw8) : (dtype == MMM_BF16 ? v.bf16 : v.f32);
    (void)hipGetLastError();   // drop any stale error another library left on this thread
    hipLaunchKernelGGL(fn, dim3((uint32_t)pl.workgroups), dim3((uint32_t)v.info.threads), dyn, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (pl.split_k > 1) {
        const int64_t total = m->M * m->N;
        int64_t blocks = (total + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(mmm_splitk_reduce_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, m->partials, C, ldc,
                           m->M, m->N, pl.split_k, accumulate);
        e = hipGetLastError();
    }
    return e;
}
