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
// workgroup owns 64 rows of C and keeps two LDS slabs.  While the waves multiply
// step c out of one slab (reading it as the dense 16 x 4 MFMA operand), they
// take the list of block c-1 out of the other slab and put the list of block
// c+1 into it, both with integer adds on the float bit patterns, which commute:
// one barrier per step.  Columns of a block that are zero in all its rows are
// dropped from the k lists (column-any words).
//
// Pipeline: list entries travel into registers two steps before they are
// added, the first B operands of a step are requested one step ahead, and inside
// a long k list the B operands of the next batch are requested before the
// current batch is multiplied.  The map words a workgroup needs are copied to
// LDS, and expanded to k lists, in windows of several steps.  The kernel is
// bound by instruction issue and latency rather than by any pipe, so the
// workgroup shapes that do best are those that put sixteen waves on a compute
// unit (eight or sixteen waves per workgroup, one 16-column group per wave).
#include "mmm_internal.h"

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int TM = MMM_AB_ROWS;   // rows of C per workgroup = rows of a block of A
constexpr int KC = MMM_AB_COLS;   // k per step = columns of a block of A
constexpr int WPC = KC / 64;      // map words per step
constexpr int QB = 6;             // k-list quads per batch
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
    int32_t window_chunks;   // steps whose map words are held in LDS (and whose k lists exist) at a time
    int32_t zero;            // always 0
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

// [NG][nwords] 64-bit words (per group: transposed-B word AND column-any word of A)
extern __shared__ uint64_t mmm_dyn_words[];

// map words one wave expands into k lists per window (fewer for the eight-wave workgroups, whose
// lists would otherwise keep a second workgroup off the compute unit)
constexpr int list_words(int nw) { return nw >= 8 ? 16 : 32; }

// RT  16-row MFMA sub-tiles computed (4: all 64 rows of the block; 2: matrices of at most 32 rows)
// GW  16-column groups per wave, NW waves per workgroup: TN = 16*GW*NW columns
template <int RT, int GW, int NW, typename T, bool BW8>
__global__ __launch_bounds__(NW * 64) void mmm_matmul_kernel(const MatmulParams p)
{
    constexpr int NG = NW * GW;
    constexpr int NT = NW * 64;
    constexpr int EPT = 1024 / NT;    // list entries of A per thread and round
    constexpr int ROUND = NT * EPT;   // list entries one round of the workgroup moves
    constexpr int SLAB = MMM_SLAB_FLOATS;   // floats per slab; column KC stays zero (the A operand of a k-list slot past the end)
    constexpr int LW = list_words(NW);
    constexpr int SEG = LW / GW;      // lanes (= map words) per group: SEG / WPC steps per window
    constexpr int REGION = SEG * 64;  // list bytes per group: the worst case

    __shared__ __align__(16) float As[2 * SLAB];       // two slabs: one is multiplied from while the other changes
    __shared__ uint8_t lists[NW][GW * REGION + 4];     // per wave: k lists of its groups for one window

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

    const T *Y = static_cast<const T *>(p.Y);
    const uint32_t ldy32 = (uint32_t)p.ldy;

    floatx4 acc[GW][RT];
#pragma unroll
    for (int g = 0; g < GW; ++g)
#pragma unroll
        for (int r = 0; r < RT; ++r) acc[g][r] = floatx4{0.f, 0.f, 0.f, 0.f};

    // both slabs start out all zero; whatever is added to a slab is subtracted again later
    for (int i = tid; i < 2 * SLAB / 4; i += NT) reinterpret_cast<floatx4 *>(As)[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    int wbegin = chunk_begin;   // first step of the current window
    int wchunks = 0;            // steps in the current window

    // map words of the steps [wb, wb + window_chunks) -> LDS
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
    };

    // One round of a block's non-zero list, in registers: entry tid + j * NT is entry j of this
    // thread.  The builder pads every list to a multiple of 64, so whether a wave has an entry j
    // is a wave-uniform question.
    struct Entries {
        uint32_t pos[EPT];   // byte offset inside a slab
        uint32_t val[EPT];   // float bit pattern
        uint32_t cntv;       // entries of the block (the same value in every lane); 0: no block
    };
    // First batch of B operands of one step, per group of this wave.
    struct BFirst {
        float b[GW][QB];
        int kk[GW][QB];      // the listed k they belong to
        int cnt[GW], start[GW];
    };
    Entries eprev, ecur, enext, eload;
    BFirst buse, bnext;
    eprev.cntv = ecur.cntv = enext.cntv = eload.cntv = 0;

    const int wave_e0 = wave * 64;
    // request the first round of the list of block ch (and its count) into registers
    auto issue_entries = [&](int ch, Entries &e) {
        const size_t blk = (size_t)tile_m * p.KBA + ch;
        // the count comes through the vector memory path like the entries, so that it arrives in
        // order with them (the lane term is always 0)
        e.cntv = p.a_cnt[blk + (size_t)(lane & p.zero)];
        const uint2 *ent = p.a_ent + blk * MMM_AB_CAP + tid;
        // Loaded unconditionally (a round always lies inside the block's list area); what lies
        // past the padded count is never used.  No branch, so nothing here waits for the data.
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const uint2 v = ent[j * NT];
            e.pos[j] = v.x;
            e.val[j] = v.y;
        }
    };
    auto padded_count = [&](const Entries &e) -> int {
        return ((int)__builtin_amdgcn_readfirstlane(e.cntv) + 63) & ~63;
    };
    // A slab is filled and emptied with integer adds on the float bit patterns: a cell goes
    // 0 -> bits -> 0 exactly, whatever the order in which the adds of different threads land, so
    // removing block c-1 from a slab and putting block c+1 into it need no barrier between them.
    auto slab_add = [&](char *slab, uint32_t pos, uint32_t v) {
        __hip_atomic_fetch_add(reinterpret_cast<uint32_t *>(slab + pos), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    // the first round of a list, from registers
    auto apply_round = [&](char *slab, const Entries &e, int cnt, bool fill) {
#pragma unroll
        for (int j = 0; j < EPT; ++j)
            if (wave_e0 + j * NT < cnt) slab_add(slab, e.pos[j], fill ? e.val[j] : 0u - e.val[j]);
    };
    // blocks with more entries than one round: the rest is fetched and applied on the spot
    auto apply_rest = [&](char *slab, int ch, int cnt, bool fill) {
        const uint2 *ent = p.a_ent + ((size_t)tile_m * p.KBA + ch) * MMM_AB_CAP;
        for (int e = ROUND + tid; e < cnt; e += NT) {
            const uint2 v = ent[e];
            slab_add(slab, v.x, fill ? v.y : 0u - v.y);
        }
    };

    // ---- k lists.  Once per window every wave turns the map words of its groups into compacted
    // lists of live k: lane (g, w) owns word w of group g, a segmented prefix sum of the popcounts
    // gives every word its place in the list of its group, and each lane then writes out the bit
    // positions of its own word.  Entries are step-relative k (0..127); the entries of one step
    // are contiguous, and `pref` (read with readlane) tells where each step starts.
    uint32_t pref = 0, incl = 0;          // exclusive / inclusive popcount prefix of this lane's word inside its group
    auto build_lists = [&](int nchunks) {
        const int g = (lane / SEG) % GW, wi = lane % SEG;
        uint64_t m = (lane < LW && wi < nchunks * WPC) ? mmm_dyn_words[(wave * GW + g) * nwords + wi] : 0ull;
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

    // ---- multiply step ci from slab S: 4 listed k per MFMA.  `between` runs after the first A
    // operands have been requested and before the first MFMA.
    auto multiply = [&](int ci, const BFirst &f, const float *S, auto &&between) {
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
                        for (int r = 0; r < RT; ++r) a[g][u][r] = S[kk * 64 + ((c + kk) & 15) * 4 + r];
                    }
                }
            }
            between();
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
                    for (int r = 0; r < RT; ++r) a[u][r] = S[kk * 64 + ((c + kk) & 15) * 4 + r];
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

    // start of a window: map words -> LDS -> k lists, and the first B operands of its first step
    auto open_window = [&](int wb) {
        wbegin = wb;
        wchunks = min(p.window_chunks, chunk_end - wb);
        load_words(wb);
        __syncthreads();
        build_lists(wchunks);
        issue_b_first(0, buse);
    };

    if (chunk_begin < chunk_end) {
        issue_entries(chunk_begin, ecur);
        if (chunk_begin + 1 < chunk_end) issue_entries(chunk_begin + 1, enext);
        open_window(chunk_begin);   // its barrier also makes the zeroed slabs visible
        {
            const int cnt = padded_count(ecur);
            apply_round(reinterpret_cast<char *>(As), ecur, cnt, true);
            if (cnt > ROUND) apply_rest(reinterpret_cast<char *>(As), chunk_begin, cnt, true);
        }
    }
    // Step ch multiplies from slab (ch - chunk_begin) & 1, which holds block ch.  Meanwhile the other
    // slab, which held block ch-1, loses that block and receives block ch+1: one barrier per step.
    // In registers: eprev / ecur / enext = lists of blocks ch-1 / ch / ch+1, eload receives ch+2.
    for (int ch = chunk_begin; ch < chunk_end; ++ch) {
        if (ch == wbegin + wchunks) open_window(ch);
        const int ci = ch - wbegin;
        __syncthreads();   // block ch is complete in its slab; nobody reads the other slab any more
        if (ch + 2 < chunk_end)
            issue_entries(ch + 2, eload);
        else
            eload.cntv = 0;
        if (ci + 1 < wchunks) issue_b_first(ci + 1, bnext);
        const int par = (ch - chunk_begin) & 1;
        const float *S = As + par * SLAB;
        char *other = reinterpret_cast<char *>(As + (par ^ 1) * SLAB);
        const int cprev = padded_count(eprev), cnext = padded_count(enext);
        multiply(ci, buse, S, [&]() {
            apply_round(other, eprev, cprev, false);
            apply_round(other, enext, cnext, true);
        });
        if (cprev > ROUND) apply_rest(other, ch - 1, cprev, false);
        if (cnext > ROUND) apply_rest(other, ch + 1, cnext, true);
        eprev = ecur;
        ecur = enext;
        enext = eload;
        buse = bnext;
    }
    __syncthreads();   // the slabs are free: the epilogue reuses them

    // ---- write C (or this split's partial sums): every element exactly once.
    // Accumulator layout of the 16x16x4 MFMA: lane holds rows 4*s + v (v = 0..3) of column c.
    // Each wave first lays its 16*RT x 16*GW tile out row-major in its own piece of the (now
    // free) slab, then stores whole rows with 16-byte lanes, so full cache lines leave the CU.
    float *out = p.split_k > 1 ? p.P + (int64_t)split * p.M * p.N : p.C;
    const int64_t ldo = p.split_k > 1 ? p.N : p.ldc;
    const bool add = p.split_k == 1 && p.accumulate;
    const int64_t wcol0 = ((int64_t)tile_n * NG + wave * GW) * 16;   // first column of this wave
    constexpr int WCOLS = 16 * GW;
    constexpr bool FITS = NW * RT * 16 * WCOLS <= 2 * SLAB;
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
    MMM_VARIANT(4, 1, 16),  // 8: 64 x 256, sixteen waves
    MMM_VARIANT(2, 1, 8),   // 9: 32 x 128, eight waves
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
    const int64_t per_chunk = (int64_t)v.info.groups * WPC * sizeof(uint64_t);
    const int64_t gw = v.info.groups / (v.info.threads / 64);
    int64_t window = list_words(v.info.threads / 64) / (gw * WPC);   // one map word per lane
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
