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
// block sparsity is skipped exactly (no unoccupied block is ever loaded or
// multiplied); A's element sparsity is honoured by zeroing masked elements when
// the A slab is staged, and by dropping every k whose whole column of the row
// tile is zero (column-any words).  The iteration over the list is uniform
// across the wave: no lane-divergent branch exists in the inner loop.
//
// Data movement.  K is walked in chunks of KC.  The masked A slab of a chunk
// (TM rows x KC columns) is staged once per workgroup in LDS and shared by all
// of its waves; occupied B blocks go straight from global memory into the MFMA
// operand register and are reused for all TM/16 row sub-tiles of the wave.  The
// loop is software-pipelined by one chunk: while chunk c is multiplied, the A
// slab of chunk c+1 is already in flight into registers, the lists of chunk c+1
// are built, and its first B operands are in flight too; inside a list the B
// operands of the next batch are requested before the current batch is
// multiplied.  The map words a workgroup needs are copied to LDS in windows of
// many chunks, so building a list never waits on global memory.
#include "mmm_internal.h"

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

struct MatmulParams {
    const void *X;
    int64_t ldx;
    const void *Y;
    int64_t ldy;
    float *C;
    int64_t ldc;
    float *P;   // split-K partial sums, [split][M][N]
    const uint8_t *a_bytes;
    const uint64_t *a_colany;
    const uint64_t *b_bits;
    const uint64_t *bt_bits;
    int64_t M, K, N, NB, WA, WB, MT;
    int32_t bw;
    int32_t tiles_m, tiles_n, split_k, chunks_total, chunks_per_split;
    int32_t window_chunks;   // chunks whose map words are held in LDS at a time
    int32_t accumulate;
    int32_t fast_x;   // X rows are 16-byte (f32) / 8-byte (bf16) aligned: vector loads allowed
};

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<uint16_t>(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

template <typename T> __device__ __forceinline__ floatx4 load4(const T *p);
template <> __device__ __forceinline__ floatx4 load4<float>(const float *p)
{
    return *reinterpret_cast<const floatx4 *>(p);
}
template <> __device__ __forceinline__ floatx4 load4<uint16_t>(const uint16_t *p)
{
    const uint2 r = *reinterpret_cast<const uint2 *>(p);
    floatx4 v;
    v.x = __uint_as_float(r.x << 16);
    v.y = __uint_as_float(r.x & 0xffff0000u);
    v.z = __uint_as_float(r.y << 16);
    v.w = __uint_as_float(r.y & 0xffff0000u);
    return v;
}

// Workgroups are dealt round-robin to the 8 XCDs.  Re-number them so that each
// XCD works on a contiguous range of logical tiles: neighbours in that range
// share the same rows of X, which then stay in that XCD's L2.
__device__ __forceinline__ uint32_t xcd_contiguous_id(uint32_t b, uint32_t n)
{
    const uint32_t x = b & 7u, i = b >> 3, q = n >> 3, rem = n & 7u;
    return x * q + (x < rem ? x : rem) + i;
}

__device__ __forceinline__ uint64_t uniform64(uint64_t v)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

extern __shared__ uint64_t mmm_dyn_words[];   // [NG + 1][nwords]: transposed-B words per group, then column-any words

// TM  rows of C per workgroup (shared by all its waves), multiple of 32
// GW  16-column groups per wave, NW waves per workgroup: TN = 16*GW*NW columns
// KC  columns of A staged per step, multiple of 64
template <int TM, int GW, int NW, int KC, typename T>
__global__ __launch_bounds__(NW * 64) void mmm_matmul_kernel(const MatmulParams p)
{
    constexpr int RT = TM / 16;      // 16-row MFMA sub-tiles per wave
    constexpr int KCP = KC + 4;      // padded LDS row; columns KC..KC+3 stay zero (list sentinel)
    constexpr int NG = NW * GW;
    constexpr int QB = 4;            // list quads per batch
    constexpr int LPAD = 4 * QB;
    constexpr int C4 = KC / 4;
    constexpr int NT = NW * 64;
    constexpr int APT = TM * C4 / NT;   // float4 items of the A slab per thread
    constexpr int WPC = KC / 64;        // map words per chunk
    static_assert(TM * C4 % NT == 0, "A slab must divide evenly over the threads");

    __shared__ __align__(16) float As[TM * KCP];
    __shared__ uint16_t lists[2][NG][KC + LPAD];

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

    const T *X = static_cast<const T *>(p.X);
    const T *Y = static_cast<const T *>(p.Y);

    floatx4 acc[GW][RT];
#pragma unroll
    for (int g = 0; g < GW; ++g)
#pragma unroll
        for (int r = 0; r < RT; ++r) acc[g][r] = floatx4{0.f, 0.f, 0.f, 0.f};

    for (int r = tid; r < TM; r += NT) *reinterpret_cast<floatx4 *>(&As[r * KCP + KC]) = floatx4{0.f, 0.f, 0.f, 0.f};

    // map words of the chunks [wbegin, wbegin + window_chunks) -> LDS
    auto load_words = [&](int wbegin) {
        for (int idx = tid; idx < (NG + 1) * nwords; idx += NT) {
            const int gi = idx / nwords, wi = idx % nwords;
            const int64_t widx = (int64_t)wbegin * WPC + wi;
            uint64_t m = 0;
            if (widx < p.WA) {
                if (gi < NG) {
                    const int64_t G = (int64_t)tile_n * NG + gi;   // global 16-column group
                    if (G * 16 < p.N) {
                        if (p.bw == 16) {
                            m = p.bt_bits[G * p.WA + widx];
                        } else if (p.bw == 32) {
                            m = p.bt_bits[(G >> 1) * p.WA + widx];
                        } else {
                            m = p.bt_bits[(2 * G) * p.WA + widx];
                            if (2 * G + 1 < p.NB) m |= p.bt_bits[(2 * G + 1) * p.WA + widx];
                        }
                    }
                } else {
#pragma unroll
                    for (int t = 0; t < TM / MMM_COLANY_ROWS; ++t) {
                        const int64_t tt = row0 / MMM_COLANY_ROWS + t;
                        if (tt < p.MT) m |= p.a_colany[tt * p.WA + widx];
                    }
                }
            }
            mmm_dyn_words[idx] = m;
        }
    };

    int wbegin = chunk_begin;   // first chunk of the current window
    floatx4 areg[APT];
    uint32_t anib[APT];
    float bcur[GW][QB], bnext[GW][QB];
    int cnt_cur[GW], cnt_next[GW];

    // request the A slab of chunk ci (relative) into registers
    auto issue_a = [&](int ci) {
        const int64_t k0 = (int64_t)(wbegin + ci) * KC;
#pragma unroll
        for (int i = 0; i < APT; ++i) {
            const int idx = tid + i * NT;
            const int r = idx / C4, c4 = idx % C4;
            const int64_t row = row0 + r, k = k0 + 4 * c4;
            floatx4 v = {0.f, 0.f, 0.f, 0.f};
            uint32_t nib = 0;
            if (row < p.M && k < p.K) {
                nib = (p.a_bytes[row * p.WA * 8 + (k >> 3)] >> (k & 4)) & 0xFu;
                const T *src = X + row * p.ldx + k;
                if (p.fast_x && k + 3 < p.K) {
                    v = load4<T>(src);
                } else {   // pad bits of the map are zero, so a set bit implies k+e < K
                    if (nib & 1u) v.x = to_f32<T>(src[0]);
                    if (nib & 2u) v.y = to_f32<T>(src[1]);
                    if (nib & 4u) v.z = to_f32<T>(src[2]);
                    if (nib & 8u) v.w = to_f32<T>(src[3]);
                }
            }
            areg[i] = v;
            anib[i] = nib;
        }
    };
    // As[r][kk] = a_bits[row0+r, k0+kk] ? X[row0+r, k0+kk] : 0
    auto store_a = [&]() {
#pragma unroll
        for (int i = 0; i < APT; ++i) {
            const int idx = tid + i * NT;
            const int r = idx / C4, c4 = idx % C4;
            floatx4 v = areg[i];
            const uint32_t nib = anib[i];
            if (!(nib & 1u)) v.x = 0.f;
            if (!(nib & 2u)) v.y = 0.f;
            if (!(nib & 4u)) v.z = 0.f;
            if (!(nib & 8u)) v.w = 0.f;
            *reinterpret_cast<floatx4 *>(&As[r * KCP + 4 * c4]) = v;
        }
    };
    // per 16-column group: compacted list of the live k of chunk ci (chunk-relative, ascending)
    auto build_lists = [&](int ci, int buf, int (&cnt)[GW]) {
#pragma unroll
        for (int g = 0; g < GW; ++g) {
            const int gi = wave * GW + g;
            int base = 0;
#pragma unroll
            for (int wd = 0; wd < WPC; ++wd) {
                const int wi = ci * WPC + wd;
                const uint64_t m = uniform64(mmm_dyn_words[gi * nwords + wi] & mmm_dyn_words[NG * nwords + wi]);
                const uint32_t pos = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                if ((m >> lane) & 1ull) lists[buf][gi][base + pos] = (uint16_t)(wd * 64 + lane);
                base += __popcll(m);
            }
            if (lane < LPAD) lists[buf][gi][base + lane] = (uint16_t)KC;
            cnt[g] = base;
        }
    };
    // one B operand: row k0+kk of Y at this lane's column, or 0 for a list sentinel
    auto load_b = [&](int64_t k0, int kk, int64_t col, bool col_ok) -> float {
        bool ok = col_ok && kk < KC;
        if (p.bw == 8 && ok) {   // a group spans two blocks: take only this lane's own block
            const int64_t blk = col >> 3;
            ok = (p.b_bits[(k0 + kk) * p.WB + (blk >> 6)] >> (blk & 63)) & 1ull;
        }
        return ok ? to_f32<T>(Y[(k0 + kk) * p.ldy + col]) : 0.f;
    };
    auto issue_b_first = [&](int ci, int buf, float (&b)[GW][QB]) {
        const int64_t k0 = (int64_t)(wbegin + ci) * KC;
#pragma unroll
        for (int g = 0; g < GW; ++g) {
            const int gi = wave * GW + g;
            const int64_t col = ((int64_t)tile_n * NG + gi) * 16 + c;
#pragma unroll
            for (int u = 0; u < QB; ++u) b[g][u] = load_b(k0, lists[buf][gi][4 * u + s], col, col < p.N);
        }
    };

    // K range of this workgroup, in windows whose map words fit in LDS; inside a window the
    // chunk loop is pipelined by one chunk
    for (wbegin = chunk_begin; wbegin < chunk_end; wbegin += p.window_chunks) {
        const int nchunks = min(p.window_chunks, chunk_end - wbegin);
        __syncthreads();   // previous window fully consumed (A slab and map words)
        load_words(wbegin);
        __syncthreads();
        build_lists(0, 0, cnt_cur);
        issue_a(0);
        issue_b_first(0, 0, bcur);
        store_a();
        __syncthreads();


        for (int ci = 0; ci < nchunks; ++ci) {
            const int buf = ci & 1;
            const bool has_next = ci + 1 < nchunks;
            const int64_t k0 = (int64_t)(wbegin + ci) * KC;
            if (has_next) {
                build_lists(ci + 1, buf ^ 1, cnt_next);
                issue_a(ci + 1);
                issue_b_first(ci + 1, buf ^ 1, bnext);
            }

            // ---- multiply chunk ci: 4 listed k per MFMA
    #pragma unroll
            for (int g = 0; g < GW; ++g) {
                const int n = cnt_cur[g];
                const int gi = wave * GW + g;
                const int64_t col = ((int64_t)tile_n * NG + gi) * 16 + c;
                const bool col_ok = col < p.N;
                const uint16_t *lst = lists[buf][gi];
                float b[QB];
    #pragma unroll
                for (int u = 0; u < QB; ++u) b[u] = bcur[g][u];
                for (int q = 0; q < n; q += LPAD) {
                    float bn[QB];
                    if (q + LPAD < n) {   // request the next batch of B operands before multiplying this one
    #pragma unroll
                        for (int u = 0; u < QB; ++u) bn[u] = load_b(k0, lst[q + LPAD + 4 * u + s], col, col_ok);
                    } else {
    #pragma unroll
                        for (int u = 0; u < QB; ++u) bn[u] = 0.f;
                    }
                    int kk[QB];
    #pragma unroll
                    for (int u = 0; u < QB; ++u) kk[u] = lst[q + 4 * u + s];
    #pragma unroll
                    for (int u = 0; u < QB; ++u) {
                        if (q + 4 * u < n) {
    #pragma unroll
                            for (int r = 0; r < RT; ++r) {
                                const float a = As[(r * 16 + c) * KCP + kk[u]];
                                acc[g][r] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b[u], acc[g][r], 0, 0, 0);
                            }
                        }
                    }
    #pragma unroll
                    for (int u = 0; u < QB; ++u) b[u] = bn[u];
                }
            }

            __syncthreads();   // every wave is done reading the A slab of chunk ci
            if (has_next) {
                store_a();
    #pragma unroll
                for (int g = 0; g < GW; ++g) {
                    cnt_cur[g] = cnt_next[g];
    #pragma unroll
                    for (int u = 0; u < QB; ++u) bcur[g][u] = bnext[g][u];
                }
            }
            __syncthreads();   // the A slab of chunk ci+1 is complete
        }
    }

    // ---- write C (or this split's partial sums): every element exactly once
    // accumulator layout of the 16x16x4 MFMA: lane holds rows 4*s + v (v = 0..3) of column c
#pragma unroll
    for (int g = 0; g < GW; ++g) {
        const int64_t col = ((int64_t)tile_n * NG + wave * GW + g) * 16 + c;
        if (col >= p.N) continue;
#pragma unroll
        for (int r = 0; r < RT; ++r) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int64_t row = row0 + r * 16 + s * 4 + v;
                if (row >= p.M) continue;
                const float val = acc[g][r][v];
                if (p.split_k > 1) {
                    p.P[((int64_t)split * p.M + row) * p.N + col] = val;
                } else {
                    float *dst = p.C + row * p.ldc + col;
                    *dst = p.accumulate ? *dst + val : val;
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
    matmul_kernel_fn f32, bf16;
};

#define MMM_VARIANT(TM, GW, NW, KC)                                                                        \
    {                                                                                                      \
        {"TM" #TM "_TN" #GW "x" #NW "x16_KC" #KC, TM, 16 * GW * NW, KC, NW * 64, NW * GW},                 \
            mmm_matmul_kernel<TM, GW, NW, KC, float>, mmm_matmul_kernel<TM, GW, NW, KC, uint16_t>          \
    }

const VariantEntry g_variants[] = {
    MMM_VARIANT(64, 4, 4, 128),    // 0: 64 x 256
    MMM_VARIANT(64, 2, 4, 128),    // 1: 64 x 128
    MMM_VARIANT(32, 4, 4, 128),    // 2: 32 x 256
    MMM_VARIANT(32, 2, 4, 256),    // 3: 32 x 128, long chunk
    MMM_VARIANT(128, 2, 4, 64),    // 4: 128 x 128, short chunk
    MMM_VARIANT(64, 2, 4, 64),     // 5: 64 x 128, short chunk
    MMM_VARIANT(64, 1, 8, 128),    // 6: 64 x 128, eight waves
    MMM_VARIANT(32, 1, 4, 256),    // 7: 32 x 64
};
constexpr int32_t kVariants = (int32_t)(sizeof(g_variants) / sizeof(g_variants[0]));

}   // namespace

int32_t mmm_variant_count() { return kVariants; }
const mmm_variant_info &mmm_variant(int32_t i) { return g_variants[i].info; }

hipError_t mmm_launch_matmul(const mmm_maps *m, const mmm_plan &pl, int32_t dtype, const void *X, int64_t ldx,
                             const void *Y, int64_t ldy, float *C, int64_t ldc, int32_t accumulate, hipStream_t s)
{
    if (pl.variant < 0 || pl.variant >= kVariants) return hipErrorInvalidValue;
    const VariantEntry &v = g_variants[pl.variant];
    MatmulParams p{};
    p.X = X;
    p.ldx = ldx;
    p.Y = Y;
    p.ldy = ldy;
    p.C = C;
    p.ldc = ldc;
    p.P = m->partials;
    p.a_bytes = reinterpret_cast<const uint8_t *>(m->a_bits);
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
    p.bw = m->bw;
    p.tiles_m = pl.tiles_m;
    p.tiles_n = pl.tiles_n;
    p.split_k = pl.split_k;
    p.chunks_total = pl.chunks_total;
    p.chunks_per_split = pl.chunks_per_split;
    p.accumulate = accumulate;
    const size_t esz = dtype == MMM_BF16 ? 2 : 4;
    p.fast_x = ((reinterpret_cast<uintptr_t>(X) % (4 * esz)) == 0 && (ldx % 4) == 0) ? 1 : 0;
    if (pl.workgroups <= 0 || pl.workgroups > 0x7fffffffLL) return hipErrorInvalidValue;
    if (pl.split_k > 1 && (size_t)pl.split_k * (size_t)m->M * (size_t)m->N * sizeof(float) > m->partial_bytes)
        return hipErrorInvalidValue;
    const int64_t wpc = v.info.KC / 64;
    int64_t window = MMM_MAX_DYN_LDS / (int64_t)((v.info.groups + 1) * wpc * sizeof(uint64_t));
    if (window > pl.chunks_per_split) window = pl.chunks_per_split;
    if (window < 1) return hipErrorInvalidValue;
    p.window_chunks = (int32_t)window;
    const size_t dyn = (size_t)(v.info.groups + 1) * (size_t)window * (size_t)wpc * sizeof(uint64_t);
    matmul_kernel_fn fn = dtype == MMM_BF16 ? v.bf16 : v.f32;
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
