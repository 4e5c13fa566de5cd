// Host side of the C ABI declared in include/mmm.h: argument checks, workspace
// layout, launch planning.  All checks run before any device call, so they can
// be exercised on a machine without a GPU.
#include <atomic>
#include <cstdio>
#include <cstring>
#include <new>

#include "mmm_internal.h"

namespace {

constexpr size_t kAlign = 256;
constexpr int64_t kMaxLd = (1LL << 22) - 1;   // largest leading dimension of X and Y the masked GEMM addresses
constexpr size_t kPartialCap = (size_t)64 << 20;   // split-K partial sums: at most 64 MiB

thread_local char g_detail[160] = "";

void note_device_error(const char *where, hipError_t e)
{
    std::snprintf(g_detail, sizeof(g_detail), "%s: %s (%d)", where, hipGetErrorName(e), (int)e);
}

std::atomic<int64_t> g_opt_variant{-1};
std::atomic<int64_t> g_opt_split{0};
std::atomic<int64_t> g_opt_path{-1};

inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Layout {
    size_t a_bits, a_colany, a_cnt, a_ent, b_bits, bt_bits, stats, kinfo, kmap, a_colany_c, btc_bits, Bc, partials, partial_bytes, total;
};

bool shape_ok(int64_t M, int64_t K, int64_t N, int32_t bw)
{
    if (M < 1 || K < 1 || N < 1) return false;
    if (bw != 8 && bw != 16 && bw != 32) return false;
    if (N % bw != 0) return false;
    // 31-bit grids and 32-bit tile-relative offsets are used throughout
    if (M > (1LL << 30) || K > (1LL << 30) || N > (1LL << 30)) return false;
    return true;
}

Layout make_layout(int64_t M, int64_t K, int64_t N, int32_t bw)
{
    const int64_t NB = N / bw, WA = (K + 63) / 64, WB = (NB + 63) / 64, MT = (M + MMM_COLANY_ROWS - 1) / MMM_COLANY_ROWS;
    Layout l{};
    size_t off = 0;
    l.a_bits = off;
    off += align_up((size_t)M * WA * 8);
    l.a_colany = off;
    off += align_up((size_t)MT * WA * 8);
    const size_t blocks = (size_t)((M + MMM_AB_ROWS - 1) / MMM_AB_ROWS) * (size_t)((K + MMM_AB_COLS - 1) / MMM_AB_COLS);
    l.a_cnt = off;
    off += align_up(blocks * 4);
    l.a_ent = off;
    off += align_up(blocks * MMM_AB_CAP * 8);
    l.b_bits = off;
    off += align_up((size_t)K * WB * 8);
    l.bt_bits = off;
    off += align_up((size_t)NB * WA * 8);
    l.stats = off;
    off += align_up(4 * 8);
    // row-compacted mode: numbering of the live rows, maps over it, and room for every row of Y in its widest type
    l.kinfo = off;
    off += align_up(64);
    l.kmap = off;
    off += align_up((size_t)K * 4);
    l.a_colany_c = off;
    off += align_up((size_t)MT * WA * 8);
    l.btc_bits = off;
    off += align_up((size_t)NB * WA * 8);
    l.Bc = off;
    off += align_up((size_t)K * (size_t)N * 4);
    l.partials = off;
    // room for up to 32 splits of C, capped
    size_t want = (size_t)M * (size_t)N * sizeof(float) * 32;
    if (want > kPartialCap) want = kPartialCap;
    l.partial_bytes = align_up(want);
    off += l.partial_bytes;
    l.total = off;
    return l;
}

bool dtype_ok(int32_t dt) { return dt == MMM_F32 || dt == MMM_BF16 || dt == MMM_F16 || dt == MMM_F64; }
size_t elem_size(int32_t dt) { return dt == MMM_F64 ? 8 : dt == MMM_F32 ? 4 : 2; }
size_t c_elem_size(int32_t dt) { return dt == MMM_F64 ? 8 : 4; }

mmm_plan make_plan(const mmm_maps *m, int32_t dt)
{
    (void)dt;
    mmm_plan p{};
    int64_t v = m->plan_variant >= 0 ? m->plan_variant : g_opt_variant.load();
    if (v >= 0 && v < mmm_variant_count() && mmm_variant((int32_t)v).rows < MMM_AB_ROWS && m->M > mmm_variant((int32_t)v).rows)
        v = -1;   // that kernel computes too few rows for this matrix
    if (v < 0 || v >= mmm_variant_count()) {
        // automatic: the shapes that put sixteen waves on a compute unit.  32-row kernel for short
        // matrices; otherwise the 256-column tile (one workgroup of sixteen waves per CU) when that
        // still gives every CU a workgroup, else the 128-column tile (eight waves); matrices too small
        // to fill the machine that way, and too short in K for a split to pay, take the 64-column tile
        if (m->M <= 32) {
            v = 5;
        } else {
            const int64_t tm = (m->M + 63) / 64, chunks = (m->K + MMM_AB_COLS - 1) / MMM_AB_COLS;
            const int64_t t256 = tm * ((m->N + 255) / 256), t128 = tm * ((m->N + 127) / 128);
            v = t256 >= 256 ? 1 : (t128 >= 192 || chunks >= 16) ? 0 : 2;
        }
    }
    const mmm_variant_info &vi = mmm_variant((int32_t)v);
    p.variant = (int32_t)v;
    p.tiles_m = (int32_t)((m->M + vi.TM - 1) / vi.TM);
    p.tiles_n = (int32_t)((m->N + vi.TN - 1) / vi.TN);
    p.chunks_total = (int32_t)((m->K + vi.KC - 1) / vi.KC);
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    int64_t split = m->plan_split > 0 ? m->plan_split : g_opt_split.load();
    if (split <= 0) {
        split = 1;
        if (tiles < 256) {   // fewer tiles than CUs: split K to give every CU work, if every part keeps 8 steps
            split = (512 + tiles - 1) / tiles;
            if (split > p.chunks_total / 8) split = p.chunks_total / 8;
        }
    }
    const int64_t max_by_ws = (int64_t)(m->partial_bytes / ((size_t)m->M * (size_t)m->N * sizeof(float)));
    if (split > max_by_ws) split = max_by_ws;
    if (split > p.chunks_total) split = p.chunks_total;
    if (split < 1) split = 1;
    p.chunks_per_split = (int32_t)((p.chunks_total + split - 1) / split);
    split = (p.chunks_total + p.chunks_per_split - 1) / p.chunks_per_split;   // drop empty splits
    p.split_k = (int32_t)split;
    p.workgroups = tiles * split;
    return p;
}

// Which kernel multiplies.  The matrix-instruction kernel issues work in proportion to B's block
// density (every listed row of B meets all rows of a tile of A); the pair kernel does work in
// proportion to the product of both densities but pays two gathers per product and a fixed cost
// per row and 64 columns.  Fitted to measurements on an MI355X (4096^3, 2048 x 16384 x 4096 and
// 32 ... 512 x 8192 x 4096, densities 0.02 ... 0.4):
//     pairs  ~ 110 us + 24500 us * p_A * p_B      matrix ~ 95 us + 1000 us * p_B      (per 4096^3)
// so for matrices of many rows the pair kernel is ahead iff p_B * (1 - 24.5 * p_A) > 0.015, which
// needs p_A below 0.04; for matrices of at most 64 rows (one tile of the matrix kernel, mostly
// empty, and a latency-bound launch) it is ahead up to p_A * p_B of about 0.02, and for small problems
// (256^3) with short lists as well.  Densities are
// known only after a mmm_maps_stats call (the counts of the most recent one are kept as the
// estimate, also across rebuilds: emergent sparsity levels are stable from step to step); without
// one the shape decides alone.
int32_t choose_path(const mmm_maps *m)
{
    int64_t path = m->plan_path >= 0 ? m->plan_path : g_opt_path.load();
    if (path == MMM_PATH_MATRIX || path == MMM_PATH_PAIRS) return (int32_t)path;
    if (m->plan_variant >= 0 || g_opt_variant.load() >= 0) return MMM_PATH_MATRIX;   // a tile variant was asked for
    const bool known = m->stats_a_valid && m->stats_b_valid;
    const double p_a = known ? (double)m->stats_nnz_a / ((double)m->M * (double)m->K) : 0.0;
    const double p_b = known ? (double)m->stats_occ_b / ((double)m->K * (double)m->NB) : 0.0;
    if (m->M <= 64) return !known || p_a * p_b <= 0.02 ? MMM_PATH_PAIRS : MMM_PATH_MATRIX;
    // small problems (the matrix kernel would fill less than half the machine) with short lists are bound by
    // latency, of which the pair kernel has less
    const int64_t tiles = ((m->M + 63) / 64) * ((m->N + 127) / 128);
    if (known && tiles < 128 && p_a * p_b * (double)m->K <= 64.0) return MMM_PATH_PAIRS;
    return known && p_b * (1.0 - 24.5 * p_a) > 0.015 ? MMM_PATH_PAIRS : MMM_PATH_MATRIX;
}

}   // namespace

extern "C" {

const char *mmm_status_string(mmm_status st)
{
    switch (st) {
    case MMM_OK: return "ok";
    case MMM_ERR_INVALID_ARG: return "invalid argument";
    case MMM_ERR_SHAPE: return "invalid shape";
    case MMM_ERR_DTYPE: return "invalid element type or alignment";
    case MMM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case MMM_ERR_MAPS_MISMATCH: return "maps not built or built for different inputs";
    case MMM_ERR_DEVICE: return "device error";
    }
    return "unknown status";
}

mmm_status mmm_maps_workspace_bytes(int64_t M, int64_t K, int64_t N, int32_t block_width, size_t *bytes)
{
    if (bytes == nullptr) return MMM_ERR_INVALID_ARG;
    if (!shape_ok(M, K, N, block_width)) return MMM_ERR_SHAPE;
    *bytes = make_layout(M, K, N, block_width).total;
    return MMM_OK;
}

mmm_status mmm_maps_init(void *dev_workspace, size_t workspace_bytes, int64_t M, int64_t K, int64_t N,
                         int32_t block_width, mmm_maps **out)
{
    if (out == nullptr) return MMM_ERR_INVALID_ARG;
    if (!shape_ok(M, K, N, block_width)) return MMM_ERR_SHAPE;
    const Layout l = make_layout(M, K, N, block_width);
    if (dev_workspace == nullptr || reinterpret_cast<uintptr_t>(dev_workspace) % kAlign != 0 ||
        workspace_bytes < l.total)
        return MMM_ERR_WORKSPACE;
    mmm_maps *m = new (std::nothrow) mmm_maps();
    if (m == nullptr) return MMM_ERR_INVALID_ARG;
    m->M = M;
    m->K = K;
    m->N = N;
    m->bw = block_width;
    m->NB = N / block_width;
    m->WA = (K + 63) / 64;
    m->WB = (m->NB + 63) / 64;
    m->MT = (M + MMM_COLANY_ROWS - 1) / MMM_COLANY_ROWS;
    char *base = static_cast<char *>(dev_workspace);
    m->a_bits = reinterpret_cast<uint64_t *>(base + l.a_bits);
    m->a_colany = reinterpret_cast<uint64_t *>(base + l.a_colany);
    m->MBA = (M + MMM_AB_ROWS - 1) / MMM_AB_ROWS;
    m->KBA = (K + MMM_AB_COLS - 1) / MMM_AB_COLS;
    m->a_cnt = reinterpret_cast<uint32_t *>(base + l.a_cnt);
    m->a_ent = reinterpret_cast<uint64_t *>(base + l.a_ent);
    m->b_bits = reinterpret_cast<uint64_t *>(base + l.b_bits);
    m->bt_bits = reinterpret_cast<uint64_t *>(base + l.bt_bits);
    m->stats = reinterpret_cast<uint64_t *>(base + l.stats);
    m->kinfo = reinterpret_cast<uint32_t *>(base + l.kinfo);
    m->kmap = reinterpret_cast<uint32_t *>(base + l.kmap);
    m->a_colany_c = reinterpret_cast<uint64_t *>(base + l.a_colany_c);
    m->btc_bits = reinterpret_cast<uint64_t *>(base + l.btc_bits);
    m->Bc = base + l.Bc;
    m->partials = reinterpret_cast<float *>(base + l.partials);
    m->partial_bytes = l.partial_bytes;
    m->ws = dev_workspace;
    m->ws_bytes = workspace_bytes;
    m->a_built = m->b_built = false;
    m->a_compact = m->b_compact = false;
    m->a_dtype = m->b_dtype = -1;
    m->a_src = nullptr;
    m->a_src_ld = 0;
    m->plan_variant = -1;
    m->plan_split = 0;
    m->plan_path = -1;
    m->stats_a_valid = m->stats_b_valid = false;
    m->stats_nnz_a = m->stats_occ_b = 0;
    *out = m;
    return MMM_OK;
}

void mmm_maps_release(mmm_maps *maps) { delete maps; }

mmm_status mmm_build_maps(mmm_maps *maps, mmm_dtype dt, const void *X, int64_t ldx, const mmm_mask_a *ma,
                          const void *Y, int64_t ldy, const mmm_mask_b *mb, void *hip_stream)
{
    if (maps == nullptr || (X == nullptr && Y == nullptr)) return MMM_ERR_INVALID_ARG;
    if (!dtype_ok(dt)) return MMM_ERR_DTYPE;
    const size_t esz = elem_size(dt);
    mmm_build_args a{};
    a.dtype = dt;
    if (X != nullptr) {
        if (ma == nullptr) return MMM_ERR_INVALID_ARG;
        if (ma->pred < MMM_PRED_NONZERO || ma->pred > MMM_PRED_ABS_GT) return MMM_ERR_INVALID_ARG;
        if (ldx < maps->K || ldx > kMaxLd) return MMM_ERR_SHAPE;
        if (reinterpret_cast<uintptr_t>(X) % esz != 0) return MMM_ERR_DTYPE;
        if (ma->keep_bits != nullptr && reinterpret_cast<uintptr_t>(ma->keep_bits) % 8 != 0) return MMM_ERR_INVALID_ARG;
        a.X = X;
        a.ldx = ldx;
        a.pred = ma->pred;
        a.threshold = ma->threshold;
        a.keep_a = ma->keep_bits;
    }
    if (Y != nullptr) {
        if (mb == nullptr) return MMM_ERR_INVALID_ARG;
        if (mb->block_width != maps->bw) return MMM_ERR_SHAPE;
        if (ldy < maps->N || ldy > kMaxLd) return MMM_ERR_SHAPE;
        if (reinterpret_cast<uintptr_t>(Y) % esz != 0) return MMM_ERR_DTYPE;
        if ((mb->keep_rows != nullptr && reinterpret_cast<uintptr_t>(mb->keep_rows) % 8 != 0) ||
            (mb->keep_blocks != nullptr && reinterpret_cast<uintptr_t>(mb->keep_blocks) % 8 != 0))
            return MMM_ERR_INVALID_ARG;
        a.Y = Y;
        a.ldy = ldy;
        a.keep_rows = mb->keep_rows;
        a.keep_blocks = mb->keep_blocks;
    }
    // Row-compacted mode: when keep_rows switches whole rows of B off, the live rows are numbered k' and the
    // matrix kernel walks k' (steps of 128 live rows instead of 128 rows of which few are live).  The lists of
    // A are then made over k', so they are only good for the numbering they were made for.
    a.b_compact = Y != nullptr && mb->keep_rows != nullptr && dt != MMM_F64;
    const bool compact_after = Y != nullptr ? a.b_compact : maps->b_compact;
    a.a_compact = X != nullptr && compact_after;
    if (hipError_t e = dt == MMM_F64 ? mmm_launch_build64(maps, a, static_cast<hipStream_t>(hip_stream))
                                      : mmm_launch_build(maps, a, static_cast<hipStream_t>(hip_stream));
        e != hipSuccess) {
        note_device_error("map builder launch", e);
        return MMM_ERR_DEVICE;
    }
    if (Y != nullptr) {
        // lists of A made for another numbering of k (or for none) do not fit the new B side
        if (X == nullptr && (maps->b_compact || a.b_compact)) maps->a_built = false;
        maps->b_compact = a.b_compact;
    }
    if (X != nullptr) {
        maps->a_compact = a.a_compact;
        maps->a_built = true;
        maps->a_dtype = dt;
        maps->a_src = X;   // compared, never dereferenced
        maps->a_src_ld = ldx;
    }
    if (Y != nullptr) {
        maps->b_built = true;
        maps->b_dtype = dt;
    }
    return MMM_OK;
}

mmm_status mmm_maps_view(const mmm_maps *maps, const uint64_t **a_bits, int64_t *a_row_words,
                         const uint64_t **b_bits, int64_t *b_row_words)
{
    if (maps == nullptr) return MMM_ERR_INVALID_ARG;
    if (a_bits) *a_bits = maps->a_bits;
    if (a_row_words) *a_row_words = maps->WA;
    if (b_bits) *b_bits = maps->b_bits;
    if (b_row_words) *b_row_words = maps->WB;
    return MMM_OK;
}

mmm_status mmm_maps_view_derived(const mmm_maps *maps, const uint64_t **a_colany, const uint64_t **bt_bits,
                                 int64_t *k_words)
{
    if (maps == nullptr) return MMM_ERR_INVALID_ARG;
    if (a_colany) *a_colany = maps->a_colany;
    if (bt_bits) *bt_bits = maps->bt_bits;
    if (k_words) *k_words = maps->WA;
    return MMM_OK;
}

mmm_status mmm_maps_view_compacted(const mmm_maps *maps, int32_t *on, const uint32_t **live_count, const uint32_t **kmap,
                                   const uint64_t **a_colany_c, const uint64_t **btc_bits)
{
    if (maps == nullptr) return MMM_ERR_INVALID_ARG;
    if (on) *on = maps->b_compact ? 1 : 0;
    if (live_count) *live_count = maps->kinfo;
    if (kmap) *kmap = maps->kmap;
    if (a_colany_c) *a_colany_c = maps->a_colany_c;
    if (btc_bits) *btc_bits = maps->btc_bits;
    return MMM_OK;
}

mmm_status mmm_debug_k_lists(const mmm_maps *maps, void *out, size_t out_bytes, size_t *bytes_needed, void *hip_stream)
{
    if (maps == nullptr) return MMM_ERR_INVALID_ARG;
    if (!maps->a_built || !maps->b_built) return MMM_ERR_MAPS_MISMATCH;
    if (maps->a_dtype == MMM_F64) return MMM_ERR_DTYPE;   // double inputs have no matrix kernel
    size_t need = 0;
    const hipError_t e = mmm_launch_dump_lists(maps, static_cast<uint8_t *>(out), out_bytes, &need,
                                               static_cast<hipStream_t>(hip_stream));
    if (bytes_needed) *bytes_needed = need;
    if (e == hipErrorInvalidValue) return out == nullptr && bytes_needed != nullptr ? MMM_OK : MMM_ERR_WORKSPACE;
    if (e != hipSuccess) {
        note_device_error("k list dump launch", e);
        return MMM_ERR_DEVICE;
    }
    return MMM_OK;
}

mmm_status mmm_maps_view_lists(const mmm_maps *maps, const uint32_t **counts, const uint64_t **entries,
                               int64_t *blocks_m, int64_t *blocks_k, int64_t *capacity)
{
    if (maps == nullptr) return MMM_ERR_INVALID_ARG;
    if (counts) *counts = maps->a_cnt;
    if (entries) *entries = maps->a_ent;
    if (blocks_m) *blocks_m = maps->MBA;
    if (blocks_k) *blocks_k = maps->KBA;
    if (capacity) *capacity = MMM_AB_CAP;
    return MMM_OK;
}

mmm_status mmm_maps_stats(const mmm_maps *maps, uint64_t *nnz_a, uint64_t *occupied_blocks_b,
                          uint64_t *useful_macs, void *hip_stream)
{
    if (maps == nullptr) return MMM_ERR_INVALID_ARG;
    if (!maps->a_built || !maps->b_built) return MMM_ERR_MAPS_MISMATCH;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipError_t e = mmm_launch_stats(maps, s);
    uint64_t host[4] = {0, 0, 0, 0};
    if (e == hipSuccess) e = hipMemcpyAsync(host, maps->stats, sizeof(host), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
        note_device_error("statistics", e);
        return MMM_ERR_DEVICE;
    }
    maps->stats_nnz_a = host[0];
    maps->stats_occ_b = host[1];
    maps->stats_a_valid = maps->stats_b_valid = true;
    if (nnz_a) *nnz_a = host[0];
    if (occupied_blocks_b) *occupied_blocks_b = host[1];
    if (useful_macs) *useful_macs = host[2];
    return MMM_OK;
}

mmm_status mmm_matmul_plan(const mmm_maps *maps, mmm_dtype dt, int32_t *variant, int32_t *split_k, int64_t *workgroups)
{
    if (maps == nullptr) return MMM_ERR_INVALID_ARG;
    if (!dtype_ok(dt)) return MMM_ERR_DTYPE;
    const mmm_plan p = make_plan(maps, dt);
    if (variant) *variant = p.variant;
    if (split_k) *split_k = p.split_k;
    if (workgroups) *workgroups = p.workgroups;
    return MMM_OK;
}

}   // extern "C"

static mmm_status matmul_common(const mmm_maps *maps, mmm_dtype dt, const void *X, int64_t ldx, const void *Y, int64_t ldy,
                                void *C, int64_t ldc, int32_t accumulate, void *hip_stream, bool static_scratch)
{
    if (maps == nullptr || X == nullptr || Y == nullptr || C == nullptr) return MMM_ERR_INVALID_ARG;
    if (!dtype_ok(dt)) return MMM_ERR_DTYPE;
    if (ldx < maps->K || ldy < maps->N || ldc < maps->N) return MMM_ERR_SHAPE;
    if (ldx > kMaxLd || ldy > kMaxLd) return MMM_ERR_SHAPE;   // tile-relative offsets are 32-bit
    const size_t esz = elem_size(dt);
    if (reinterpret_cast<uintptr_t>(X) % esz != 0 || reinterpret_cast<uintptr_t>(Y) % esz != 0 ||
        reinterpret_cast<uintptr_t>(C) % c_elem_size(dt) != 0)
        return MMM_ERR_DTYPE;
    if (dt == MMM_F64 && !mmm_pairs_supports(dt, ldy)) return MMM_ERR_SHAPE;   // double inputs have the pair kernel only
    if (!maps->a_built || !maps->b_built) return MMM_ERR_MAPS_MISMATCH;
    if (maps->a_dtype != dt || maps->b_dtype != dt) return MMM_ERR_MAPS_MISMATCH;
    // the values of A travel in the lists that were copied from X at build time: another X is another A
    if (maps->a_src != X || maps->a_src_ld != ldx) return MMM_ERR_MAPS_MISMATCH;
    if (dt == MMM_F64 || (choose_path(maps) == MMM_PATH_PAIRS && mmm_pairs_supports(dt, ldy))) {   // no scratch at all on this path
        if (hipError_t e = mmm_launch_pairs(maps, dt, X, ldx, Y, ldy, C, ldc, accumulate ? 1 : 0, false, 0, 0.f, nullptr,
                                            static_cast<hipStream_t>(hip_stream));
            e != hipSuccess) {
            note_device_error("masked GEMM (pairs) launch", e);
            return MMM_ERR_DEVICE;
        }
        return MMM_OK;
    }
    const mmm_plan p = make_plan(maps, dt);
    float *partials = maps->partials;
    size_t partial_bytes = maps->partial_bytes;
    if (static_scratch) {
        const size_t need = p.split_k > 1 ? (size_t)p.split_k * (size_t)maps->M * (size_t)maps->N * sizeof(float) : 0;
        if (need > (size_t)MMM_STATIC_SCRATCH_BYTES) {
            std::snprintf(g_detail, sizeof(g_detail),
                          "mmm_matmul_static_scratch: %d partial sums of C need %zu bytes, the static scratch holds %zu",
                          (int)p.split_k, need, (size_t)MMM_STATIC_SCRATCH_BYTES);
            return MMM_ERR_WORKSPACE;
        }
        if (hipError_t e = mmm_static_scratch(&partials); e != hipSuccess) {
            note_device_error("address of the static scratch", e);
            return MMM_ERR_DEVICE;
        }
        partial_bytes = (size_t)MMM_STATIC_SCRATCH_BYTES;
    }
    if (hipError_t e = mmm_launch_matmul(maps, p, dt, X, ldx, Y, ldy, static_cast<float *>(C), ldc, accumulate ? 1 : 0, partials,
                                         partial_bytes, static_cast<hipStream_t>(hip_stream));
        e != hipSuccess) {
        note_device_error("masked GEMM launch", e);
        return MMM_ERR_DEVICE;
    }
    return MMM_OK;
}

extern "C" {

mmm_status mmm_matmul(const mmm_maps *maps, mmm_dtype dt, const void *X, int64_t ldx, const void *Y, int64_t ldy,
                      void *C, int64_t ldc, int32_t accumulate, void *hip_stream)
{
    return matmul_common(maps, dt, X, ldx, Y, ldy, C, ldc, accumulate, hip_stream, false);
}

mmm_status mmm_matmul_fused(const mmm_maps *maps, mmm_dtype dt, const void *X, int64_t ldx, const mmm_mask_a *ma,
                            const void *Y, int64_t ldy, void *C, int64_t ldc, int32_t accumulate, void *hip_stream)
{
    if (maps == nullptr || X == nullptr || Y == nullptr || C == nullptr || ma == nullptr) return MMM_ERR_INVALID_ARG;
    if (ma->pred < MMM_PRED_NONZERO || ma->pred > MMM_PRED_ABS_GT) return MMM_ERR_INVALID_ARG;
    if (ma->keep_bits != nullptr && reinterpret_cast<uintptr_t>(ma->keep_bits) % 8 != 0) return MMM_ERR_INVALID_ARG;
    if (!dtype_ok(dt)) return MMM_ERR_DTYPE;
    if (ldx < maps->K || ldy < maps->N || ldc < maps->N) return MMM_ERR_SHAPE;
    if (ldx > kMaxLd || ldy > kMaxLd) return MMM_ERR_SHAPE;
    const size_t esz = elem_size(dt);
    if (reinterpret_cast<uintptr_t>(X) % esz != 0 || reinterpret_cast<uintptr_t>(Y) % esz != 0 ||
        reinterpret_cast<uintptr_t>(C) % c_elem_size(dt) != 0)
        return MMM_ERR_DTYPE;
    if (!mmm_pairs_supports(dt, ldy)) return MMM_ERR_SHAPE;
    if (!maps->b_built || maps->b_dtype != dt) return MMM_ERR_MAPS_MISMATCH;
    if (hipError_t e = mmm_launch_pairs(maps, dt, X, ldx, Y, ldy, C, ldc, accumulate ? 1 : 0, true, ma->pred,
                                        ma->threshold, ma->keep_bits, static_cast<hipStream_t>(hip_stream));
        e != hipSuccess) {
        note_device_error("fused masked GEMM launch", e);
        return MMM_ERR_DEVICE;
    }
    return MMM_OK;
}

mmm_status mmm_matmul_static_scratch(const mmm_maps *maps, mmm_dtype dt, const void *X, int64_t ldx, const void *Y,
                                     int64_t ldy, void *C, int64_t ldc, int32_t accumulate, void *hip_stream)
{
    return matmul_common(maps, dt, X, ldx, Y, ldy, C, ldc, accumulate, hip_stream, true);
}

mmm_status mmm_maps_set_plan(mmm_maps *maps, int32_t variant, int32_t split_k)
{
    if (maps == nullptr) return MMM_ERR_INVALID_ARG;
    if (variant < -1 || variant >= mmm_variant_count()) return MMM_ERR_INVALID_ARG;
    if (split_k < 0 || split_k > 4096) return MMM_ERR_INVALID_ARG;
    maps->plan_variant = variant;
    maps->plan_split = split_k;
    return MMM_OK;
}

mmm_status mmm_maps_set_path(mmm_maps *maps, int32_t path)
{
    if (maps == nullptr) return MMM_ERR_INVALID_ARG;
    if (path < -1 || path > MMM_PATH_PAIRS) return MMM_ERR_INVALID_ARG;
    maps->plan_path = path;
    return MMM_OK;
}

mmm_status mmm_matmul_path(const mmm_maps *maps, int32_t *path)
{
    if (maps == nullptr || path == nullptr) return MMM_ERR_INVALID_ARG;
    *path = (maps->a_built && maps->a_dtype == MMM_F64) || (maps->b_built && maps->b_dtype == MMM_F64) ? MMM_PATH_PAIRS : choose_path(maps);
    return MMM_OK;
}

mmm_status mmm_set_option(const char *name, int64_t value)
{
    if (name == nullptr) return MMM_ERR_INVALID_ARG;
    if (std::strcmp(name, "matmul_path") == 0) {
        if (value < -1 || value > MMM_PATH_PAIRS) return MMM_ERR_INVALID_ARG;
        g_opt_path.store(value);
        return MMM_OK;
    }
    if (std::strcmp(name, "matmul_variant") == 0) {
        if (value < -1 || value >= mmm_variant_count()) return MMM_ERR_INVALID_ARG;
        g_opt_variant.store(value);
        return MMM_OK;
    }
    if (std::strcmp(name, "split_k") == 0) {
        if (value < 0 || value > 4096) return MMM_ERR_INVALID_ARG;
        g_opt_split.store(value);
        return MMM_OK;
    }
    return MMM_ERR_INVALID_ARG;
}

const char *mmm_last_device_error(void) { return g_detail; }

int32_t mmm_matmul_variant_count(void) { return mmm_variant_count(); }

const char *mmm_matmul_variant_name(int32_t i)
{
    if (i < 0 || i >= mmm_variant_count()) return nullptr;
    return mmm_variant(i).name;
}

}   // extern "C"
