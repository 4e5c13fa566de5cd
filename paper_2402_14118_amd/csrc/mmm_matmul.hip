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
// current batch is multiplied.  Every lane fetches half a map word of its
// wave's column group and expands it into the k lists, in windows of several
// steps.  The kernel is bound by instruction issue on the SIMDs (an fp32 MFMA
// and a vector instruction do not run side by side there), so it is written to
// need few instructions per MFMA, and the workgroup shapes that do best are
// those that put sixteen waves on a compute unit (eight or sixteen waves per
// workgroup, one 16-column group per wave).
#include <mutex>

#include "mmm_internal.h"

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int TM = MMM_AB_ROWS;   // rows of C per workgroup = rows of a block of A
constexpr int KC = MMM_AB_COLS;   // k per step = columns of a block of A
constexpr int WPC = KC / 64;      // map words per step
constexpr int QB = 4;             // k-list quads per batch
constexpr int BATCH = 4 * QB;     // list slots per batch (a power of two that divides KC)
constexpr int SLAB = MMM_SLAB_FLOATS;                 // floats per slab
constexpr uint32_t SLAB_BYTES = (uint32_t)SLAB * 4u;
constexpr uint32_t COLB = MMM_SLAB_COL_BYTES;         // bytes per slab column; column KC stays zero
static_assert(WPC == 2, "a step is one pair of map words");

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
    uint8_t *dump;           // DUMP instantiation only: where the k lists are written out (see mmm_debug_k_lists)
    const uint32_t *kinfo;   // row-compacted mode: [0] = number of live k (the maps, lists and Y above are then over k'); else null
    int64_t M, K, N, NB, WA, WB, MT, KBA;
    int32_t bw;
    int32_t tiles_m, tiles_n, split_k, chunks_total, chunks_per_split;
    int32_t window_chunks;   // steps whose k lists are built in one go
    int32_t zero;            // always 0
    int32_t accumulate;
};

typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));

// 16-bit inputs are contracted by the matrix instructions of their own type, 16 values of k per
// instruction (fp32 accumulate).  Operands reach the multiply step widened to float (the slab and
// the lists of A hold float bit patterns); two of them are narrowed back into one register here,
// which is exact because they were widened from that type.
template <typename T> struct Narrow;
template <> struct Narrow<uint16_t> {   // bf16: the upper halves of the two float patterns
    static __device__ __forceinline__ uint32_t pack(float lo, float hi)
    {
        return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
    }
    static __device__ __forceinline__ floatx4 mfma(uint2 a, uint2 b, floatx4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, a), __builtin_bit_cast(shortx4, b), c, 0, 0, 0);
    }
};
template <> struct Narrow<_Float16> {
    static __device__ __forceinline__ uint32_t pack(float lo, float hi)
    {
        return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
    }
    static __device__ __forceinline__ floatx4 mfma(uint2 a, uint2 b, floatx4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(halfx4, a), __builtin_bit_cast(halfx4, b), c, 0, 0, 0);
    }
};

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<uint16_t>(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }   // bf16
template <> __device__ __forceinline__ float to_f32<_Float16>(_Float16 v) { return (float)v; }

// Workgroups are dealt round-robin to the 8 XCDs.  Re-number them so that each
// XCD works on a contiguous range of logical tiles: neighbours in that range
// share the same block row of A and neighbouring column tiles of B, which then
// stay in that XCD's L2.
__device__ __forceinline__ uint32_t xcd_contiguous_id(uint32_t b, uint32_t n)
{
    const uint32_t x = b & 7u, i = b >> 3, q = n >> 3, rem = n & 7u;
    return x * q + (x < rem ? x : rem) + i;
}

// map words one wave expands into k lists per window (fewer for the eight-wave workgroups, whose
// lists would otherwise keep a second workgroup off the compute unit)
constexpr int list_words(int nw) { return nw == 8 ? 16 : 32; }

// On this machine the fp32 MFMA and the vector ALU do not run side by side on a SIMD: every
// vector instruction of the inner loop costs matrix time.  The loop is therefore written to
// need few of them: addresses are a wave-uniform base plus one multiply-add per operand, the
// k lists are padded so that no index needs clamping, LDS offsets are immediates, and the
// registers that carry operands from step to step rotate by unrolling, not by moves.
//
// RT  16-row MFMA sub-tiles computed (4: all 64 rows of the block; 2: matrices of at most 32 rows)
// GW  16-column groups per wave, NW waves per workgroup: TN = 16*GW*NW columns
template <int RT, int GW, int NW, typename T, bool BW8, bool DUMP = false>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(NW >= 8 && GW == 1 ? 4 : 2))) void mmm_matmul_kernel(const MatmulParams p)
{
    constexpr int NG = NW * GW;
    constexpr int NT = NW * 64;
    constexpr int EPT = 1024 / NT;    // list entries of A per thread and round
    constexpr int ROUND = NT * EPT;   // list entries one round of the workgroup moves
    constexpr int LW = list_words(NW);
    constexpr int SEG = LW / GW;      // map words per group and window: SEG / WPC steps
    constexpr int REGION = SEG * 64;  // list bytes per group: the worst case
    constexpr uint32_t ESZ = (uint32_t)sizeof(T);
    typedef float avec __attribute__((ext_vector_type(RT)));   // A operands of the RT row tiles for one k

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
    // steps of this workgroup; in row-compacted mode only the steps that hold a live k exist, shared out anew
    int chunks_live = p.chunks_total, per_split = p.chunks_per_split;
    if (p.kinfo != nullptr) {
        chunks_live = (int)(((int64_t)*p.kinfo + KC - 1) / KC);
        per_split = (chunks_live + p.split_k - 1) / p.split_k;
    }
    const int chunk_begin = min(split * per_split, chunks_live);
    const int chunk_end = min(chunk_begin + per_split, chunks_live);
    const uint32_t ldyb = (uint32_t)p.ldy * ESZ;   // bytes per row of Y (below 2^24: the host checks)

    floatx4 acc[GW][RT];
#pragma unroll
    for (int g = 0; g < GW; ++g)
#pragma unroll
        for (int r = 0; r < RT; ++r) acc[g][r] = floatx4{0.f, 0.f, 0.f, 0.f};

    // both slabs start out all zero; whatever is added to a slab is subtracted again later
    for (int i = tid; i < 2 * SLAB / 4; i += NT) reinterpret_cast<floatx4 *>(As)[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    int wbegin = chunk_begin;   // first step of the current window
    int wchunks = 0;            // steps in the current window

    // Half a map word (32 values of k) of one 16-column group: the transposed B map of the group's
    // block(s), without the k whose column of A is zero in all rows of this tile.  h: which half of
    // 64-bit word widx (the maps are little-endian, so half h is 32-bit word 2 * widx + h).
    auto map_half = [&](int64_t G, int64_t widx, int h) __attribute__((always_inline)) -> uint32_t {
        const uint32_t *bt = reinterpret_cast<const uint32_t *>(p.bt_bits);
        const uint32_t *ca = reinterpret_cast<const uint32_t *>(p.a_colany);
        uint32_t m = 0;
        if (widx < p.WA && G * 16 < p.N) {
            if (p.bw == 16) {
                m = bt[(G * p.WA + widx) * 2 + h];
            } else if (p.bw == 32) {
                m = bt[((G >> 1) * p.WA + widx) * 2 + h];
            } else {
                m = bt[((2 * G) * p.WA + widx) * 2 + h];
                if (2 * G + 1 < p.NB) m |= bt[((2 * G + 1) * p.WA + widx) * 2 + h];
            }
            uint32_t any = 0;
#pragma unroll
            for (int t = 0; t < RT * 16 / MMM_COLANY_ROWS; ++t) {
                const int64_t tt = row0 / MMM_COLANY_ROWS + t;
                if (tt < p.MT) any |= ca[(tt * p.WA + widx) * 2 + h];
            }
            m &= any;
        }
        return m;
    };

    // One round of a block's non-zero list, in registers: entry tid + j * NT is entry j of this
    // thread.  The builder pads every list to a multiple of 64, so whether a wave has an entry j
    // is a wave-uniform question.
    struct Entries {
        uint32_t pos[EPT];   // byte offset inside a slab
        uint32_t val[EPT];   // float bit pattern
        uint32_t cntv;       // entries of the block (the same value in every lane)
    };
    Entries E0, E1, E2, E3;
    E0.cntv = E1.cntv = E2.cntv = E3.cntv = 0;

    const int wave_e0 = wave * 64;
    const char *ent_tile = reinterpret_cast<const char *>(p.a_ent) + (size_t)tile_m * p.KBA * (MMM_AB_CAP * 8);
    const char *cnt_tile = reinterpret_cast<const char *>(p.a_cnt) + (size_t)tile_m * p.KBA * 4;
    const uint32_t tid8 = (uint32_t)tid * 8u;
    // the count comes through the vector memory path like the entries, so that it arrives in
    // order with them (this lane offset is always 0)
    const uint32_t zoff = (uint32_t)(lane & p.zero) * 4u;
    // request the first round of the list of block ch (and its count) into registers
    auto issue_entries = [&](int ch, Entries &e) __attribute__((always_inline)) {
        // Everything is loaded unconditionally, so that nothing here waits for data: past the end
        // of the K range the last block is read again (and not used); a round always lies
        // inside the block's list area, and what lies past the padded count is never used.
        ch = min(ch, p.chunks_total - 1);
        const char *eb = ent_tile + (size_t)ch * (MMM_AB_CAP * 8);   // wave-uniform
        e.cntv = *reinterpret_cast<const uint32_t *>(cnt_tile + (size_t)ch * 4 + zoff);
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const uint2 v = *reinterpret_cast<const uint2 *>(eb + tid8 + (uint32_t)(j * NT * 8));
            e.pos[j] = v.x;
            e.val[j] = v.y;
        }
    };
    // entries of block ch, rounded up to whole wavefronts; 0 if the block lies outside this workgroup's K range
    auto padded_count = [&](const Entries &e, int ch) __attribute__((always_inline)) -> int {
        return ch >= chunk_begin && ch < chunk_end ? ((int)__builtin_amdgcn_readfirstlane(e.cntv) + 63) & ~63 : 0;
    };
    // A slab is filled and emptied with integer adds on the float bit patterns: a cell goes
    // 0 -> bits -> 0 exactly, whatever the order in which the adds of different threads land, so
    // removing block c-1 from a slab and putting block c+1 into it need no barrier between them.
    auto slab_add = [&](char *slab, uint32_t pos, uint32_t v, bool fill) __attribute__((always_inline)) {
        uint32_t *cell = reinterpret_cast<uint32_t *>(slab + pos);
        if (fill)
            __hip_atomic_fetch_add(cell, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        else
            __hip_atomic_fetch_sub(cell, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    // the first round of a list, from registers
    auto apply_round = [&](char *slab, const Entries &e, int cnt, bool fill) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < EPT; ++j)
            if (wave_e0 + j * NT < cnt) slab_add(slab, e.pos[j], e.val[j], fill);
    };
    // blocks with more entries than one round: the rest is fetched and applied on the spot
    auto apply_rest = [&](char *slab, int ch, int cnt, bool fill) __attribute__((always_inline)) {
        const uint2 *ent = reinterpret_cast<const uint2 *>(ent_tile + (size_t)ch * (MMM_AB_CAP * 8));
        for (int e = ROUND + tid; e < cnt; e += NT) {
            const uint2 v = ent[e];
            slab_add(slab, v.x, v.y, fill);
        }
    };

    // ---- k lists.  Once per window every wave turns the map words of its groups into compacted
    // lists of live k.  A lane owns 32 values of k of one group (half a map word), so the four lanes
    // 4j .. 4j+3 of a group's segment own step j.  A prefix sum over the steps' list lengths, each
    // rounded up to whole batches of 4 * QB slots, gives every step its place in the list of its
    // group, and each lane then writes out the bit positions of its own half word.  Entries are
    // step-relative k (0..127).  The slots that round a step's list up repeat its last k, so that
    // a batch can always be read without clamping and always names rows of B that may be read.
    constexpr int HSEG = 2 * SEG;   // lanes per group
    uint32_t lpos = 0, ltot = 0;    // list position of this lane's half word; live k of this lane's step
    auto build_lists = [&](int wb, int nchunks) __attribute__((always_inline)) {
        const int g = (lane / HSEG) % GW, hi = lane % HSEG;   // hi: half word inside the group's window
        const int q = hi & 3;                                  // place inside the step
        uint32_t m = 0;   // every lane fetches its own half word: no staging, nothing to wait for but the load
        if (lane < 2 * LW && hi < nchunks * 4)
            m = map_half((int64_t)tile_n * NG + wave * GW + g, (int64_t)wb * WPC + (hi >> 1), hi & 1);
        const uint32_t cnt = (uint32_t)__popc(m);
        const int top = cnt ? q * 32 + 31 - __clz((int)m) : -1;   // last k of this half word
        // the four lanes of a step: counts of the lanes before this one, the step's total and last k
        const uint32_t c1 = (uint32_t)__shfl_xor((int)cnt, 1, 64);
        const uint32_t pair = cnt + c1;
        const uint32_t c2 = (uint32_t)__shfl_xor((int)pair, 2, 64);
        const uint32_t live = pair + c2;
        const uint32_t before = ((q & 1) ? c1 : 0u) + ((q & 2) ? c2 : 0u);
        int last = max(top, __shfl_xor(top, 1, 64));
        last = max(last, __shfl_xor(last, 2, 64));
        const uint32_t PT = (live + (uint32_t)BATCH - 1u) & ~((uint32_t)BATCH - 1u);
        uint32_t incl = q == 0 ? PT : 0u;   // the first lane of a step carries its padded length
#pragma unroll
        for (int d = 1; d < HSEG; d <<= 1) {
            const uint32_t o = __shfl_up(incl, d, 64);
            if (hi >= d) incl += o;
        }
        const uint32_t step_start = incl - PT;   // all lanes of a step see the same inclusive sum
        lpos = step_start + before;
        ltot = live;
        uint8_t *lst = &lists[wave][g * REGION];
        uint8_t *dst = lst + lpos;
        const uint32_t base = (uint32_t)q * 32u;
        while (m != 0) {   // as many rounds as the fullest half word of the wave has bits
            *dst++ = (uint8_t)(base + (uint32_t)__ffs((int)m) - 1u);
            m &= m - 1;
        }
        if (q == 3 && live != 0)
            for (uint32_t i = live; i < PT; ++i) lst[step_start + i] = (uint8_t)last;
    };
    // first list slot and number of live k of step ci for group g
    auto step_range = [&](int ci, int g, int &start, int &n) __attribute__((always_inline)) {
        start = (int)__builtin_amdgcn_readlane(lpos, g * HSEG + ci * 4);
        n = (int)__builtin_amdgcn_readlane(ltot, g * HSEG + ci * 4);
    };

    // B operands.  Every load is in bounds: list slots past a step's last quad are not read (the
    // last quad is read again instead), the slots that pad the last quad repeat the last listed
    // row (their A operand is the zero column of the slab, so the product vanishes), and lanes
    // past column N re-read column N-1 (their results are never written).
    const int64_t wcol0 = ((int64_t)tile_n * NG + wave * GW) * 16;   // first column of this wave
    const int64_t wcolb = min(wcol0, p.N - 1);                       // the column the wave-uniform base points at
    uint32_t coffb[GW];   // byte offset of this lane's column of group g from that base
#pragma unroll
    for (int g = 0; g < GW; ++g) coffb[g] = (uint32_t)(min(wcol0 + g * 16 + c, p.N - 1) - wcolb) * ESZ;
    const char *Ywave = static_cast<const char *>(p.Y) + wcolb * ESZ;
    const uint32_t c16 = (uint32_t)c * 16u;
    auto load_b = [&](const char *Yst, int64_t k0, uint32_t kb, int g) __attribute__((always_inline)) -> float {
        float v = to_f32<T>(*reinterpret_cast<const T *>(Yst + (__umul24(kb, ldyb) + coffb[g])));
        if (BW8) {   // a group spans two blocks: take only this lane's own block
            const int64_t blk = (wcolb + coffb[g] / ESZ) >> 3, kk = k0 + kb;
            if (!((p.bt_bits[blk * p.WA + (kk >> 6)] >> (kk & 63)) & 1ull)) v = 0.f;
        }
        return v;
    };
    // One batch of a step's list: for each of its quads the B operand of this lane's slot and the
    // slab offset of the matching A operand (the zero column for the slots that pad the list).
    // lst_s: this lane's first slot of the batch; left: live k from the batch's first slot on.
    uint32_t slotv[QB];
#pragma unroll
    for (int u = 0; u < QB; ++u) slotv[u] = (uint32_t)(4 * u + s);
    const uint32_t zero_off = (uint32_t)KC * COLB + c16;
    auto fetch_batch = [&](const char *Yst, int64_t k0, const uint8_t *lst_s, int left, int g, float (&b)[QB],
                           uint32_t (&aoff)[QB]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < QB; ++u) {
            const uint32_t kk = lst_s[4 * u];
            b[u] = load_b(Yst, k0, kk, g);
            aoff[u] = (int)slotv[u] < left ? __umul24(kk, COLB) + c16 : zero_off;
        }
    };
    // First batch of B operands of one step, per group of this wave.
    struct BFirst {
        float b[GW][QB];
        uint32_t aoff[GW][QB];   // where the matching A operands sit in a slab
        int n[GW], start[GW];
    };
    BFirst BP, BQ;
    // Yst: row k0 of Y at the wave's base column (wave-uniform)
    auto issue_b_first = [&](int ci, const char *Yst, BFirst &f) __attribute__((always_inline)) {
        const int64_t k0 = (int64_t)(wbegin + ci) * KC;
#pragma unroll
        for (int g = 0; g < GW; ++g) {
            step_range(ci, g, f.start[g], f.n[g]);
            if (f.n[g] > 0) fetch_batch(Yst, k0, &lists[wave][g * REGION + f.start[g]] + s, f.n[g], g, f.b[g], f.aoff[g]);
        }
    };

    // ---- multiply step ci from the slab at byte address S: 4 listed k per MFMA.  `between`
    // runs after the first batch.  Yst: row k0 of Y of this step at the wave's base column.
    auto mfma_quad = [&](int g, const avec &a, float b) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < RT; ++r) acc[g][r] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r], b, acc[g][r], 0, 0, 0);
    };
    // the quads of one batch that hold a live k: `left` live k from the batch's first slot on
    auto mfma_batch = [&](int g, const avec (&a)[QB], const float (&b)[QB], int left) __attribute__((always_inline)) {
        if constexpr (sizeof(T) == 2) {
            // One 16x16x16 instruction per row tile takes the whole batch: element u of a lane's operand
            // is list slot 4 * u + s, for A and B alike.  Slots without a live k hold the slab's zero
            // column on the A side and a re-read row on the B side, so they add nothing.
            const uint2 bp = make_uint2(Narrow<T>::pack(b[0], b[1]), Narrow<T>::pack(b[2], b[3]));
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const uint2 ap = make_uint2(Narrow<T>::pack(a[0][r], a[1][r]), Narrow<T>::pack(a[2][r], a[3][r]));
                acc[g][r] = Narrow<T>::mfma(ap, bp, acc[g][r]);
            }
            return;
        }
        mfma_quad(g, a[0], b[0]);
        if (left > 4) {
            mfma_quad(g, a[1], b[1]);
            if (left > 8) {
                mfma_quad(g, a[2], b[2]);
                if (left > 12) mfma_quad(g, a[3], b[3]);
            }
        }
    };
    static_assert(QB == 4, "mfma_batch is written out for four quads");
    auto multiply = [&](int ci, const BFirst &f, const char *S, const char *Yst, auto &&between) __attribute__((always_inline)) {
        // First batch of every group: the slab offsets are already in registers, so all A operands
        // are requested at once (those of quads without a live k too: they are in bounds, and a
        // branch costs more than the read), then multiplied.
        {
            avec a[GW][QB];
#pragma unroll
            for (int g = 0; g < GW; ++g) {
                if (f.n[g] > 0) {
#pragma unroll
                    for (int u = 0; u < QB; ++u) a[g][u] = *reinterpret_cast<const avec *>(S + f.aoff[g][u]);
                }
            }
#pragma unroll
            for (int g = 0; g < GW; ++g)
                if (f.n[g] > 0) mfma_batch(g, a[g], f.b[g], f.n[g]);
            between();
        }
        // further batches of long lists: B operands one batch ahead
#pragma unroll
        for (int g = 0; g < GW; ++g) {
            const int n = f.n[g];
            if (n <= BATCH) continue;
            const int64_t k0 = (int64_t)(wbegin + ci) * KC;
            const uint8_t *lst_s = &lists[wave][g * REGION + f.start[g]] + s;
            float b[QB];
            uint32_t ao[QB];
            fetch_batch(Yst, k0, lst_s + BATCH, n - BATCH, g, b, ao);
            for (int t = BATCH; t < n; t += BATCH) {   // t: first slot of the batch in b / ao
                float bn[QB];
                uint32_t aon[QB];
                if (t + BATCH < n) {
                    fetch_batch(Yst, k0, lst_s + t + BATCH, n - t - BATCH, g, bn, aon);
                } else {
#pragma unroll
                    for (int u = 0; u < QB; ++u) {
                        bn[u] = 0.f;
                        aon[u] = zero_off;
                    }
                }
                avec a[QB];
#pragma unroll
                for (int u = 0; u < QB; ++u) a[u] = *reinterpret_cast<const avec *>(S + ao[u]);
                mfma_batch(g, a, b, n - t);
#pragma unroll
                for (int u = 0; u < QB; ++u) {
                    b[u] = bn[u];
                    ao[u] = aon[u];
                }
            }
        }
    };

    const int64_t ystride = (int64_t)KC * ldyb;   // bytes of Y per step
    // start of a window: map words -> LDS -> k lists, and the first B operands of its first step
    auto open_window = [&](int wb, BFirst &f) __attribute__((always_inline)) {
        wbegin = wb;
        wchunks = min(p.window_chunks, chunk_end - wb);
        build_lists(wb, wchunks);
        issue_b_first(0, Ywave + wb * ystride, f);
    };

    // Step ch multiplies from slab (ch - chunk_begin) & 1, which holds block ch.  Meanwhile the other
    // slab, which held block ch-1, loses that block and receives block ch+1: one barrier per step.
    // prev / cur / next hold the lists of blocks ch-1 / ch / ch+1 (cur only waits for its turn as
    // prev), load receives that of block ch+2; use / next hold the first B operands of steps ch / ch+1.
    const char *Ycur = Ywave + chunk_begin * ystride;   // row ch * KC of Y at the wave's base column
    auto step = [&](int ch, int par, Entries &prev, Entries &next, Entries &load, const BFirst &use, BFirst &nextb) __attribute__((always_inline)) {
        const int ci = ch - wbegin;
        __syncthreads();   // block ch is complete in its slab; nobody reads the other slab any more
        issue_entries(ch + 2, load);
        if (ci + 1 < wchunks) issue_b_first(ci + 1, Ycur + ystride, nextb);
        const char *S = reinterpret_cast<const char *>(As) + par * SLAB_BYTES;
        char *other = reinterpret_cast<char *>(As) + (par ^ 1) * SLAB_BYTES;
        const int cprev = padded_count(prev, ch - 1), cnext = padded_count(next, ch + 1);
        multiply(ci, use, S, Ycur, [&]() {
            apply_round(other, prev, cprev, false);
            apply_round(other, next, cnext, true);
        });
        if (cprev > ROUND) apply_rest(other, ch - 1, cprev, false);
        if (cnext > ROUND) apply_rest(other, ch + 1, cnext, true);
        Ycur += ystride;
    };

    if constexpr (DUMP) {
        // Inspection only: write out the k lists exactly as build_lists makes them, window by window, and
        // multiply nothing.  Record of (row tile, 16-column group, step): 4-byte count, then 128 list bytes.
        for (int wb = chunk_begin; wb < chunk_end; wb += p.window_chunks) {
            wbegin = wb;
            wchunks = min(p.window_chunks, chunk_end - wb);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();   // the previous window's lists have been copied out
            build_lists(wb, wchunks);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int g = 0; g < GW; ++g) {
                const int64_t G = (int64_t)tile_n * NG + wave * GW + g;
                for (int ci = 0; ci < wchunks; ++ci) {
                    int start, n;
                    step_range(ci, g, start, n);
                    uint8_t *rec = p.dump + ((((int64_t)tile_m * p.tiles_n * NG + G) * p.chunks_total) + wb + ci) * 132;
                    if (lane == 0) *reinterpret_cast<uint32_t *>(rec) = (uint32_t)n;
                    for (int e = lane; e < n; e += 64) rec[4 + e] = lists[wave][g * REGION + start + e];
                }
            }
        }
        return;
    }
    if (chunk_begin < chunk_end) {
        issue_entries(chunk_begin, E1);
        issue_entries(chunk_begin + 1, E2);
        open_window(chunk_begin, BP);
        __syncthreads();   // the slabs are all zero
        const int cnt = padded_count(E1, chunk_begin);
        apply_round(reinterpret_cast<char *>(As), E1, cnt, true);
        if (cnt > ROUND) apply_rest(reinterpret_cast<char *>(As), chunk_begin, cnt, true);
    }
    // Four steps per trip, so that the roles of the register sets rotate by name.  A window that is
    // not the last one holds a multiple of four steps (the host picks 4, 8 or 16).
    for (int ch = chunk_begin; ch < chunk_end; ch += 4) {
        if (ch == wbegin + wchunks) open_window(ch, BP);
        step(ch, 0, E0, E2, E3, BP, BQ);
        if (ch + 1 < chunk_end) step(ch + 1, 1, E1, E3, E0, BQ, BP);
        if (ch + 2 < chunk_end) step(ch + 2, 0, E2, E0, E1, BP, BQ);
        if (ch + 3 < chunk_end) step(ch + 3, 1, E3, E1, E2, BQ, BP);
    }
    __syncthreads();   // the slabs are free: the epilogue reuses them

    // ---- write C (or this split's partial sums): every element exactly once.
    // Accumulator layout of the 16x16x4 MFMA: lane holds rows 4*s + v (v = 0..3) of column c.
    // Each wave first lays its 16*RT x 16*GW tile out row-major in its own piece of the (now
    // free) slab, then stores whole rows with 16-byte lanes, so full cache lines leave the CU.
    float *out = p.split_k > 1 ? p.P + (int64_t)split * p.M * p.N : p.C;
    const int64_t ldo = p.split_k > 1 ? p.N : p.ldc;
    const bool add = p.split_k == 1 && p.accumulate;
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
    matmul_kernel_fn f32, bf16, f16, f32_bw8, bf16_bw8, f16_bw8;
};

#define MMM_VARIANT(RT, GW, NW)                                                                             \
    {                                                                                                       \
        {"R" #RT "x16_TN" #GW "x" #NW "x16", TM, 16 * GW * NW, KC, NW * 64, NW * GW, 16 * RT},                 \
            mmm_matmul_kernel<RT, GW, NW, float, false>, mmm_matmul_kernel<RT, GW, NW, uint16_t, false>,     \
            mmm_matmul_kernel<RT, GW, NW, _Float16, false>, mmm_matmul_kernel<RT, GW, NW, float, true>,      \
            mmm_matmul_kernel<RT, GW, NW, uint16_t, true>, mmm_matmul_kernel<RT, GW, NW, _Float16, true>     \
    }

const VariantEntry g_variants[] = {
    MMM_VARIANT(4, 1, 8),    // 0: 64 x 128, eight waves
    MMM_VARIANT(4, 1, 16),   // 1: 64 x 256, sixteen waves
    MMM_VARIANT(4, 1, 4),    // 2: 64 x 64, four waves
    MMM_VARIANT(4, 2, 8),    // 3: 64 x 256, eight waves
    MMM_VARIANT(4, 2, 4),    // 4: 64 x 128, four waves
    MMM_VARIANT(2, 1, 8),    // 5: 32 x 128, eight waves   (matrices of at most 32 rows)
    MMM_VARIANT(2, 1, 4),    // 6: 32 x 64
    MMM_VARIANT(2, 2, 4),    // 7: 32 x 128, four waves
};
constexpr int32_t kVariants = (int32_t)(sizeof(g_variants) / sizeof(g_variants[0]));

}   // namespace

// Partial sums of the split-K multiplication for callers that cannot bring (or let the library
// carve out of a workspace) a buffer of their own: one array per GPU, held until the process
// ends.  Host code never uses the array's name as an address: the device address is looked up
// once per device and that pointer is what kernels and copies get.
static __device__ __align__(256) unsigned char scratch[MMM_STATIC_SCRATCH_BYTES];

hipError_t mmm_static_scratch(float **ptr)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *addr[kMaxDevices];   // zero-initialised: not looked up yet
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (addr[dev] == nullptr) {   // the current device's own copy of the array
        void *q = nullptr;
        e = hipGetSymbolAddress(&q, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (q == nullptr) return hipErrorInvalidSymbol;
        addr[dev] = q;
    }
    *ptr = static_cast<float *>(addr[dev]);
    return hipSuccess;
}

int32_t mmm_variant_count() { return kVariants; }
const mmm_variant_info &mmm_variant(int32_t i) { return g_variants[i].info; }

// The k lists of the default tile shape (64 x 256, sixteen waves), written out for inspection.
hipError_t mmm_launch_dump_lists(const mmm_maps *m, uint8_t *out, size_t out_bytes, size_t *need, hipStream_t s)
{
    constexpr int NG = 16;
    MatmulParams p{};
    p.a_colany = m->b_compact ? m->a_colany_c : m->a_colany;
    p.bt_bits = m->b_compact ? m->btc_bits : m->bt_bits;
    p.kinfo = m->b_compact ? m->kinfo : nullptr;
    p.M = m->M;
    p.K = m->K;
    p.N = m->N;
    p.NB = m->NB;
    p.WA = m->WA;
    p.WB = m->WB;
    p.MT = m->MT;
    p.KBA = m->KBA;
    p.bw = m->bw;
    p.tiles_m = (int32_t)((m->M + TM - 1) / TM);
    p.tiles_n = (int32_t)((m->N + 16 * NG - 1) / (16 * NG));
    p.split_k = 1;
    p.chunks_total = (int32_t)((m->K + KC - 1) / KC);
    p.chunks_per_split = p.chunks_total;
    p.window_chunks = (int32_t)(list_words(NG) / WPC);
    p.dump = out;
    const size_t bytes = (size_t)p.tiles_m * (size_t)p.tiles_n * NG * (size_t)p.chunks_total * 132;
    if (need) *need = bytes;
    if (out == nullptr || out_bytes < bytes) return hipErrorInvalidValue;
    (void)hipGetLastError();
    hipLaunchKernelGGL((mmm_matmul_kernel<4, 1, 16, float, false, true>), dim3((uint32_t)(p.tiles_m * p.tiles_n)), dim3(1024), 0, s, p);
    return hipGetLastError();
}

hipError_t mmm_launch_matmul(const mmm_maps *m, const mmm_plan &pl, int32_t dtype, const void *X, int64_t ldx,
                             const void *Y, int64_t ldy, float *C, int64_t ldc, int32_t accumulate, float *partials,
                             size_t partial_bytes, hipStream_t s)
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
    p.P = partials;
    p.a_cnt = m->a_cnt;
    p.a_ent = reinterpret_cast<const uint2 *>(m->a_ent);
    p.a_colany = m->a_colany;
    p.b_bits = m->b_bits;
    p.bt_bits = m->bt_bits;
    if (m->b_compact) {   // everything the kernel walks is over the live rows k'
        p.Y = m->Bc;
        p.ldy = m->N;
        p.a_colany = m->a_colany_c;
        p.bt_bits = m->btc_bits;
        p.kinfo = m->kinfo;
    }
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
    if (pl.split_k > 1 && (size_t)pl.split_k * (size_t)m->M * (size_t)m->N * sizeof(float) > partial_bytes)
        return hipErrorInvalidValue;
    const int64_t gw = v.info.groups / (v.info.threads / 64);
    int64_t window = list_words(v.info.threads / 64) / (gw * WPC);   // one map word per lane
    if (window > pl.chunks_per_split) window = pl.chunks_per_split;
    if (window < 1) return hipErrorInvalidValue;
    p.window_chunks = (int32_t)window;
    matmul_kernel_fn fn = m->bw == 8 ? (dtype == MMM_BF16 ? v.bf16_bw8 : dtype == MMM_F16 ? v.f16_bw8 : v.f32_bw8)
                                     : (dtype == MMM_BF16 ? v.bf16 : dtype == MMM_F16 ? v.f16 : v.f32);
    (void)hipGetLastError();   // drop any stale error another library left on this thread
    hipLaunchKernelGGL(fn, dim3((uint32_t)pl.workgroups), dim3((uint32_t)v.info.threads), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (pl.split_k > 1) {
        const int64_t total = m->M * m->N;
        int64_t blocks = (total + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(mmm_splitk_reduce_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, partials, C, ldc,
                           m->M, m->N, pl.split_k, accumulate);
        e = hipGetLastError();
    }
    return e;
}
