// Internal declarations shared by the host API and the kernel launchers.
// Not part of the public ABI (that is include/mmm.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "mmm.h"

// Rows of A summarised by one column-any word.
constexpr int MMM_COLANY_ROWS = 32;
// Rows of B (values of k) one workgroup of the B-side map builder covers; the
// transposed map is written in pieces of this many bits.
constexpr int MMM_BT_PIECE = 16;
// Geometry of the blocks of A whose non-zero elements are listed (count, offsets, values).
constexpr int MMM_AB_ROWS = 64;
constexpr int MMM_AB_COLS = 128;
constexpr int MMM_AB_CAP = MMM_AB_ROWS * MMM_AB_COLS;   // list capacity per block: the worst case
// The LDS slab a block is scattered into is column-major: a column takes MMM_SLAB_COL_BYTES, its
// first 256 bytes hold the 64 rows with the rows r, r+16, r+32, r+48 next to each other, so one
// 16-byte read yields the A operands of all four 16-row MFMA tiles for one k and the 16 lanes of an
// operand read 256 contiguous bytes.  The 16 spare bytes per column shift neighbouring columns by
// four LDS banks, which spreads the entries of one row of a block (neighbours in its list) over
// the banks.  Column MMM_AB_COLS is spare and always zero.
constexpr uint32_t MMM_SLAB_COL_BYTES = 272;
constexpr int MMM_SLAB_FLOATS = (MMM_AB_COLS + 1) * (int)(MMM_SLAB_COL_BYTES / 4);
__host__ __device__ constexpr uint32_t mmm_slab_pos(uint32_t row, uint32_t col)   // byte offset of element (row, col)
{
    return col * MMM_SLAB_COL_BYTES + (row & 15u) * 16u + (row >> 4) * 4u;
}
constexpr uint32_t MMM_SLAB_SPARE = mmm_slab_pos(0, MMM_AB_COLS);
struct mmm_maps {
    int64_t M, K, N;
    int32_t bw;
    int64_t NB;        // N / bw
    int64_t WA;        // ceil(K/64): words per row of a_bits, a_colany and bt_bits
    int64_t WB;        // ceil(NB/64): words per row of b_bits
    int64_t MT;        // ceil(M/32): rows of a_colany
    int64_t MBA, KBA;  // blocks of A: ceil(M/64) x ceil(K/128)
    // device pointers into the caller's workspace
    uint64_t *a_bits;
    uint64_t *a_colany;
    uint32_t *a_cnt;   // [MBA][KBA] non-zeros per block
    uint64_t *a_ent;   // [MBA*KBA][MMM_AB_CAP] entries {byte offset mmm_slab_pos(row, column) in the slab, value bits},
                       // padded to a multiple of 64 with {spare cell, 0}
    uint64_t *b_bits;
    uint64_t *bt_bits;
    uint64_t *stats;   // 4 words
    // Row-compacted mode (B side built with keep_rows): k' numbers the rows keep_rows leaves on, and the
    // matrix kernel walks k' instead of k.
    uint32_t *kinfo;       // [0] = number of live k (device)
    uint32_t *kmap;        // [K]: k' -> k
    uint64_t *a_colany_c;  // [MT][WA]: column-any words of A over k'
    uint64_t *btc_bits;    // [NB][WA]: the B map transposed, over k'
    void *Bc;              // [K][N] elements: the kept blocks of live row k' of Y at row k'
    float *partials;   // split-K partial sums
    size_t partial_bytes;
    void *ws;
    size_t ws_bytes;
    // state
    bool a_built, b_built;
    bool b_compact;   // the B side was built in row-compacted mode
    bool a_compact;   // the lists of A were built over k' (for the numbering of the current B side)
    int32_t a_dtype, b_dtype;
    const void *a_src;   // address and leading dimension of the X the A side was built from (identity only)
    int64_t a_src_ld;
    // launch plan fixed for this handle (-1 / 0: none, follow the process-wide options)
    int32_t plan_variant, plan_split, plan_path;
    // what the most recent mmm_maps_stats call counted: the density estimate behind the choice of kernel
    mutable bool stats_a_valid, stats_b_valid;
    mutable uint64_t stats_nnz_a, stats_occ_b;
};

struct mmm_build_args {
    // A side (X == nullptr: skip)
    const void *X;
    int64_t ldx;
    int32_t pred;
    float threshold;
    const uint64_t *keep_a;
    // B side (Y == nullptr: skip)
    const void *Y;
    int64_t ldy;
    const uint64_t *keep_rows;
    const uint64_t *keep_blocks;
    int32_t dtype;
    bool a_compact;   // list the blocks of A over the live k (the numbering exists or is made in this call)
    bool b_compact;   // number the live rows (keep_rows given) and write the compacted B side too
};

struct mmm_plan {
    int32_t variant;
    int32_t split_k;
    int32_t tiles_m, tiles_n;
    int32_t chunks_total;      // ceil(K / KC)
    int32_t chunks_per_split;
    int64_t workgroups;
};

struct mmm_variant_info {
    const char *name;
    int32_t TM, TN, KC, threads, groups, rows;   // rows: rows of C actually computed (64, or 32 for short matrices)
};

hipError_t mmm_launch_build(const mmm_maps *m, const mmm_build_args &a, hipStream_t s);
// double-precision inputs: bitmaps, column-any words and the transposed map only (no lists)
hipError_t mmm_launch_build64(const mmm_maps *m, const mmm_build_args &a, hipStream_t s);
uint64_t mmm_threshold_key64(int32_t pred, float threshold);
hipError_t mmm_launch_stats(const mmm_maps *m, hipStream_t s);
int32_t mmm_variant_count();
const mmm_variant_info &mmm_variant(int32_t i);
// partials / partial_bytes: where the split-K partial sums go (used only when p.split_k > 1)
hipError_t mmm_launch_matmul(const mmm_maps *m, const mmm_plan &p, int32_t dtype, const void *X, int64_t ldx,
                             const void *Y, int64_t ldy, float *C, int64_t ldc, int32_t accumulate, float *partials,
                             size_t partial_bytes, hipStream_t s);
// The multiplication over exactly the surviving products, on the vector ALUs.  fused: evaluate M
// (pred, threshold, keep_a) on X inside the kernel; otherwise a_bits of the maps are used.
hipError_t mmm_launch_pairs(const mmm_maps *m, int32_t dtype, const void *X, int64_t ldx, const void *Y, int64_t ldy,
                            void *C, int64_t ldc, int32_t accumulate, bool fused, int32_t pred, float threshold,
                            const uint64_t *keep_a, hipStream_t s);
// whether that kernel can address a Y of this leading dimension (it forms 32-bit offsets inside 4096 rows)
bool mmm_pairs_supports(int32_t dtype, int64_t ldy);
// the k lists the matrix kernel's default tile shape walks, written out (need: bytes required)
hipError_t mmm_launch_dump_lists(const mmm_maps *m, uint8_t *out, size_t out_bytes, size_t *need, hipStream_t s);
// device address of the library's own scratch array on the current device (MMM_STATIC_SCRATCH_BYTES bytes)
hipError_t mmm_static_scratch(float **ptr);
