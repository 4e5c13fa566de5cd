/*
 * mmm.h -- C ABI of the MI355X (gfx950) Masked Matrix Multiplication engine.
 *
 *   C = M(X) x N(Y)
 *
 * X (M x K) and Y (K x N) are dense, row-major and live in device memory.  M and
 * N are masks evaluated at run time: M zeroes single elements of X, N zeroes
 * whole aligned 1 x block_width pieces of the rows of Y (paper, sections 1 and
 * 3: A = M(X) has random element sparsity, B = N(Y) block-random sparsity; Fig.
 * "Types of sparsity").  The work is split the way the paper splits it
 * (section 3, "Preprocessing" and "Matrix Multiplication"): one pass builds
 * sparsity maps, the multiplication then consumes the maps and skips every
 * product whose A element is zero or whose B block is empty.
 *
 * Conventions for every call
 *   - Pointers named X, Y, C, keep_*, dev_workspace are DEVICE pointers owned by
 *     the caller.  The library never allocates or frees device memory and never
 *     reads X, Y or C after the work of a call has run; the handle remembers the
 *     address and leading dimension of the X its A side was built from, only to
 *     compare them with what mmm_matmul is given.
 *   - Row-major; leading dimensions (ldx, ldy, ldc) are in elements and must be
 *     >= the row length; ldx and ldy must be below 2^22 (MMM_ERR_SHAPE
 *     otherwise, from mmm_build_maps and from mmm_matmul alike).  C is float
 *     (double for MMM_F64 inputs), passed as void*.
 *   - Bitmaps: LSB-first little-endian 64-bit words, row-major, every row padded
 *     to whole words, pad bits zero: bit (c mod 64) of word (c div 64) of row r
 *     describes column c of row r.  (The paper prints patterns first-vector-
 *     leftmost; the layout here is this library's own.)
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls enqueue work and return; only mmm_maps_stats waits for the stream.
 *   - Errors are return codes.  Arguments are checked on the host before any
 *     device work is enqueued; on error nothing is launched and no output is
 *     touched.  No call aborts or prints.
 *   - Masked-out elements of X and switched-off blocks of Y never reach the
 *     arithmetic, whatever they hold.  Values inside occupied blocks of Y are
 *     expected to be finite.  If Y[k,j] inside an occupied block is Inf or NaN,
 *     column j of C is affected and no other column: C[i,j] is non-finite for
 *     every row i whose a_bits[i,k] is set (as the definition gives), and for the
 *     remaining rows it is either the value of the definition or NaN (the matrix
 *     instruction path multiplies an occupied block by explicit zeros for rows
 *     whose element of A is zero).
 */
#ifndef MMM_H
#define MMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MMM_OK = 0,
    MMM_ERR_INVALID_ARG = 1,   /* NULL where a pointer is required, bad enum value                */
    MMM_ERR_SHAPE = 2,         /* M, K, N < 1, ld too small, N not a multiple of block_width      */
    MMM_ERR_DTYPE = 3,         /* unknown element type, or misaligned pointer for that type       */
    MMM_ERR_WORKSPACE = 4,     /* workspace NULL, misaligned (256 B) or too small                 */
    MMM_ERR_MAPS_MISMATCH = 5, /* maps not built yet, or built for another shape / element type   */
    MMM_ERR_DEVICE = 6         /* a HIP call failed (launch error)                                */
} mmm_status;

/* Element type of X and Y.  BF16 is the upper half of an IEEE float, F16 the IEEE
 * half format; both are widened to float exactly, products are accumulated in
 * float and C is float.  F64: X, Y and C are double, products are accumulated in
 * double (the paper reports float and double runs, section 4).  Double inputs
 * are multiplied by the MMM_PATH_PAIRS kernel only, and mmm_build_maps writes the
 * bitmaps and derived maps for them but no blocked lists (mmm_maps_view_lists is
 * then meaningless) and does not use the row-compacted mode. */
typedef enum { MMM_F32 = 0, MMM_BF16 = 1, MMM_F16 = 2, MMM_F64 = 3 } mmm_dtype;

/* Element predicate of M.  An element of A is non-zero iff the predicate holds,
 * the optional keep bit is set, and the value is not +-0.  (Zero test by value:
 * paper Fig. "skip computation when A is sparse".  ReLU sparsity, section 1, is
 * MMM_PRED_GT with threshold 0.)  NaN fails MMM_PRED_GT and MMM_PRED_ABS_GT;
 * denormals are non-zero. */
typedef enum {
    MMM_PRED_NONZERO = 0, /* x != 0        */
    MMM_PRED_GT = 1,      /* x >  threshold */
    MMM_PRED_ABS_GT = 2   /* |x| > threshold */
} mmm_pred;

/* M: element mask over X. */
typedef struct {
    int32_t pred;              /* mmm_pred */
    float threshold;
    const uint64_t *keep_bits; /* optional device bitmap, M x ceil(K/64) words, AND-ed with pred */
} mmm_mask_a;

/* N: block mask over Y.  A block is the aligned piece [jb*bw, jb*bw+bw) of one
 * row.  A kept block is *occupied* iff it holds any non-zero value (paper,
 * section 3, "Block-Random Sparsity in B"; caption of Fig. "Preprocessing
 * patterns": bit 1 = some non-zero value). */
typedef struct {
    int32_t block_width;         /* 8, 16 or 32; must equal the width given to mmm_maps_init     */
    const uint64_t *keep_rows;   /* optional device bitmap, ceil(K/64) words: whole rows of Y    */
    const uint64_t *keep_blocks; /* optional device bitmap, K x ceil(NB/64) words, NB = N / bw   */
} mmm_mask_b;

/* Host-side handle describing maps that live in caller-provided device memory. */
typedef struct mmm_maps mmm_maps;

/* Bytes of device workspace that maps for this shape need: the maps and their
 * derived forms, the blocked lists of A at their worst-case size (8 bytes per
 * element of X), room for the row-compacted copy of Y (4 bytes per element of
 * Y, used only when keep_rows is given), and the partial-sum area of the split-K
 * multiplication (at most 64 MiB).
 * Errors: MMM_ERR_SHAPE, MMM_ERR_INVALID_ARG (bytes NULL). */
mmm_status mmm_maps_workspace_bytes(int64_t M, int64_t K, int64_t N, int32_t block_width, size_t *bytes);

/* Create the handle.  `dev_workspace` must be 256-byte aligned device memory of
 * at least mmm_maps_workspace_bytes(); it stays owned by the caller and must
 * outlive the handle.  No device work is done here.  *out is written only on
 * success.  Errors: MMM_ERR_SHAPE, MMM_ERR_WORKSPACE, MMM_ERR_INVALID_ARG. */
mmm_status mmm_maps_init(void *dev_workspace, size_t workspace_bytes, int64_t M, int64_t K, int64_t N,
                         int32_t block_width, mmm_maps **out);

/* Frees the host handle only (NULL is allowed). */
void mmm_maps_release(mmm_maps *maps);

/* Evaluate the masks on the device and write the sparsity maps into the
 * workspace (paper, section 3 "Preprocessing": one sequential, aligned pass per
 * matrix; Fig. "Preprocessing function pointer arrays" for B, Fig. "Blocked
 * sparse row preprocessing" for A -- here both become bitmaps):
 *     a_bits[i,k]  = pred(X[i,k]) & keep_bits[i,k] & (X[i,k] != 0)
 *     b_bits[k,jb] = keep_rows[k] & keep_blocks[k,jb] & (some Y[k, jb*bw .. jb*bw+bw) != 0)
 * plus derived forms the multiplication reads: column-any words of A per 32-row
 * tile, the B map transposed to one bit-row per block column, and, for every
 * 64 x 128 block of A, the count and a compacted list of its non-zero elements
 * with their values (the count-and-offsets form of Fig. "Blocked sparse row
 * preprocessing", with the value stored beside the offset).
 * Either side may be skipped by passing X == NULL (then ma is ignored) or
 * Y == NULL: that side's maps from an earlier call are kept -- the B side of a
 * weight matrix is built once and reused (section 3: rows of B are preprocessed
 * once and used many times).  Lanes of Y whose block is switched off by the keep
 * bitmaps are not read.  With mb->keep_rows the B side is built in row-compacted
 * mode (see mmm_maps_view_compacted), which ties the lists of A to this B side.
 * Errors: MMM_ERR_INVALID_ARG (maps NULL, both X and Y NULL, mask struct NULL for
 * a present side, bad pred), MMM_ERR_SHAPE (ld too small, block_width differs
 * from the handle's), MMM_ERR_DTYPE, MMM_ERR_DEVICE. */
mmm_status mmm_build_maps(mmm_maps *maps, mmm_dtype dt,
                          const void *X, int64_t ldx, const mmm_mask_a *ma,
                          const void *Y, int64_t ldy, const mmm_mask_b *mb,
                          void *hip_stream);

/* Device pointers to the two primary maps, for inspection.  a_bits is
 * M x *a_row_words words, b_bits is K x *b_row_words words.  Any out pointer may
 * be NULL.  Valid once the side has been built and the stream has reached that
 * point.  Errors: MMM_ERR_INVALID_ARG. */
mmm_status mmm_maps_view(const mmm_maps *maps, const uint64_t **a_bits, int64_t *a_row_words,
                         const uint64_t **b_bits, int64_t *b_row_words);

/* Device pointers to the derived maps, for inspection:
 *   a_colany: ceil(M/32) x ceil(K/64) words; bit k of row t = OR of a_bits[i,k], i in [32t, 32t+32)
 *   bt_bits : NB x ceil(K/64) words; bit k of row jb = b_bits[k,jb]   (the B map transposed)
 * Errors: MMM_ERR_INVALID_ARG. */
mmm_status mmm_maps_view_derived(const mmm_maps *maps, const uint64_t **a_colany, const uint64_t **bt_bits,
                                 int64_t *k_words);

/* Row-compacted mode.  When mmm_build_maps is given mb->keep_rows (whole rows of Y switched off:
 * the contextual selection of neurons of section 4 "Matrices from ML workloads"), the rows that
 * keep_rows leaves on are numbered k' = 0 .. K'-1 in ascending k, and the matrix kernel walks k'
 * in steps of 128 live rows instead of walking k in steps of 128 rows of which few are live.  The
 * builder then also writes, for the multiplication and for inspection here:
 *   *live_count : device pointer to K' (one uint32)
 *   kmap        : K' entries, kmap[k'] = k
 *   a_colany_c  : ceil(M/32) x ceil(K/64) words; bit k' of row t = OR of a_bits[i, kmap[k']], i in [32t, 32t+32)
 *   btc_bits    : NB x ceil(K/64) words; bit k' of row jb = b_bits[kmap[k'], jb]
 *   (bits k' >= K' up to the next multiple of 128 are zero; words beyond are unspecified)
 * and keeps a copy of the kept blocks of the live rows of Y (row k' of the copy = row kmap[k'] of
 * Y), from which the matrix kernel takes B; Y itself is still what MMM_PATH_PAIRS and
 * mmm_matmul_fused read.  The blocked lists of A (mmm_maps_view_lists) are then over k' as well.
 * *on says whether the B side was last built this way.  Because the lists of A depend on the
 * numbering, building the B side alone (X == NULL) with keep_rows, or after it had been built with
 * keep_rows, leaves the A side unbuilt: build A in the same call or afterwards.
 * Any out pointer may be NULL.  Errors: MMM_ERR_INVALID_ARG. */
mmm_status mmm_maps_view_compacted(const mmm_maps *maps, int32_t *on, const uint32_t **live_count,
                                   const uint32_t **kmap, const uint64_t **a_colany_c,
                                   const uint64_t **btc_bits);

/* The per-tile active-k lists, for inspection.  The matrix kernel walks, for every row tile
 * of 64 rows, every group of 16 columns and every step of 128 values of k (of k' in
 * row-compacted mode), the ascending list of the k in that step for which the group's
 * block(s) of B are occupied and some row of the tile has a non-zero element of A; it makes
 * these lists itself, a window of steps at a time, from the transposed B map and the
 * column-any words.  This call runs exactly that list construction (for the default tile
 * shape) and writes the lists to `out` (device memory) instead of multiplying:
 *     record (tile t, group G, step c) at byte ((t * groups + G) * steps + c) * 132, where
 *     groups = 16 * ceil(N / 256), steps = ceil(K / 128):
 *     uint32 count, then `count` bytes k - 128 c (ascending), then unspecified bytes.
 *     Records of steps past the last live step (row-compacted mode) are not written.
 * Call with out == NULL to learn the size in *bytes_needed.  Both sides must be built.
 * Errors: MMM_ERR_INVALID_ARG, MMM_ERR_MAPS_MISMATCH, MMM_ERR_DTYPE (double inputs),
 * MMM_ERR_WORKSPACE (out too small), MMM_ERR_DEVICE. */
mmm_status mmm_debug_k_lists(const mmm_maps *maps, void *out, size_t out_bytes, size_t *bytes_needed,
                             void *hip_stream);

/* Device pointers to the blocked non-zero lists of A, for inspection.  A is cut
 * into *blocks_m x *blocks_k blocks of 64 rows x 128 columns (ragged at the far
 * edges); block (bm, bk) has index bm * *blocks_k + bk.
 *   counts [block]            : number of non-zero elements of A in the block
 *   entries[block][*capacity] : the first counts[block] words describe those
 *       elements, each exactly once, in an order that is fixed for a given A:
 *       low 32 bits  = 272 * column_in_block + 16 * (row_in_block % 16) + 4 * (row_in_block / 16)
 *       high 32 bits = the value as IEEE float bits (16-bit types widened)
 *     then words {34816, 0} up to the next multiple of 64 (none if the count
 *     is one already); words beyond that are unspecified.
 * In row-compacted mode (see mmm_maps_view_compacted) the columns are the live columns k': block
 * (bm, bk) holds k' in [128 bk, 128 bk + 128), column_in_block = k' - 128 bk, and only the blocks
 * with 128 bk < K' are written.
 * Errors: MMM_ERR_INVALID_ARG. */
mmm_status mmm_maps_view_lists(const mmm_maps *maps, const uint32_t **counts, const uint64_t **entries,
                               int64_t *blocks_m, int64_t *blocks_k, int64_t *capacity);

/* Counts taken from the maps (runs a small reduction on `hip_stream`, then
 * WAITS for the stream): non-zeros of A, occupied blocks of B, and useful
 * multiply-adds  sum_k nnz(A[:,k]) * bw * occupied(B[k,:])  -- the products the
 * loop of Fig. "MMM Pseudocode" performs.  Any out pointer may be NULL.
 * Errors: MMM_ERR_INVALID_ARG, MMM_ERR_MAPS_MISMATCH (a side not built),
 * MMM_ERR_DEVICE. */
mmm_status mmm_maps_stats(const mmm_maps *maps, uint64_t *nnz_a, uint64_t *occupied_blocks_b,
                          uint64_t *useful_macs, void *hip_stream);

/* C = A x B (accumulate == 0) or C += A x B (accumulate != 0) using the maps:
 *     C[i,j] (+)= sum over k with a_bits[i,k] & b_bits[k, j div bw] of X[i,k] * Y[k,j]
 * (paper, section 3 "Matrix Multiplication", Fig. "MMM Pseudocode").  X and Y
 * must hold the same values the maps were built from: the values of A are taken
 * from the lists mmm_build_maps wrote (X is not read again), those of B from Y.
 * WARNING: after X has been changed in place the A side must be rebuilt
 * (mmm_build_maps with Y == NULL) before the next mmm_matmul; otherwise C is
 * computed from the old values without any error.  What can be checked is: X
 * and ldx must be the ones the A side was built from (MMM_ERR_MAPS_MISMATCH).
 * Products the maps skip contribute exactly 0, whatever the skipped operands
 * hold (see the conventions above for non-finite kept values).  Every element
 * of C is written exactly once, zeros included.  float accumulation; the
 * result is bitwise reproducible from run to run for the same inputs and shape.
 * Errors: MMM_ERR_INVALID_ARG, MMM_ERR_SHAPE, MMM_ERR_DTYPE,
 * MMM_ERR_MAPS_MISMATCH (a side not built, dt differs from the build, or X / ldx
 * are not those of the build), MMM_ERR_DEVICE. */
mmm_status mmm_matmul(const mmm_maps *maps, mmm_dtype dt,
                      const void *X, int64_t ldx, const void *Y, int64_t ldy,
                      void *C, int64_t ldc, int32_t accumulate, void *hip_stream);

/* Which kernel mmm_matmul uses.
 *   MMM_PATH_MATRIX: matrix instructions over the compacted k lists of each 16-column group; skips
 *       B's empty blocks exactly and A's zeros only where a whole column of a 64-row tile is zero.
 *       Work grows with B's density alone.
 *   MMM_PATH_PAIRS : vector FMAs over exactly the products that survive both maps (the loop of
 *       Fig. "MMM Pseudocode": skip when the element of A is zero, skip the empty blocks of the row
 *       of B), found by AND-ing the bitmap row of A with the transposed B map.  Work grows with
 *       the product of both densities, at a higher cost per product.  Reads X itself (not the
 *       lists of the maps).  Needs ldy * sizeof(element) below 2^20 bytes; beyond that mmm_matmul
 *       uses MATRIX whatever was asked for.
 * Automatic choice (path -1): MATRIX if a tile variant has been fixed (mmm_maps_set_plan or the
 * "matmul_variant" option).  Else, with p_A and p_B the densities of A's elements and B's
 * blocks counted by the most recent mmm_maps_stats call on the handle (kept as the estimate
 * across rebuilds): for matrices of at most 64 rows PAIRS unless p_A * p_B is known to exceed
 * 0.02; for larger ones PAIRS iff the densities are known and p_B * (1 - 24.5 * p_A) > 0.015
 * (A keeps fewer than 4 % of its elements and B is not nearly empty), or the problem is small
 * (fewer than 128 tiles of 64 x 128 in C) with at most 64 surviving k per element of C; else MATRIX.  The
 * thresholds are fitted to timings on an MI355X.  The paper leaves this
 * per-workload choice of method to the caller (section 6, choosing between methods by
 * sparsity). */
#define MMM_PATH_MATRIX 0
#define MMM_PATH_PAIRS 1
/* Fix the kernel for one handle (-1: automatic).  Errors: MMM_ERR_INVALID_ARG. */
mmm_status mmm_maps_set_path(mmm_maps *maps, int32_t path);
/* The kernel mmm_matmul would use now.  Errors: MMM_ERR_INVALID_ARG. */
mmm_status mmm_matmul_path(const mmm_maps *maps, int32_t *path);

/* C (+)= M(X) x B with the mask M evaluated inside the multiplication: the A-side pass of
 * mmm_build_maps is not needed and X is read once (section 3 "Preprocessing": the cost of
 * preprocessing matters for small matrices; rows of B are preprocessed once and reused).  Only
 * the B side of the maps must have been built (for this Y, with element type dt); the A side of
 * the maps is neither read nor written, so mmm_maps_view / mmm_maps_stats keep describing
 * whatever mmm_build_maps last built.  Same definition of A as mmm_build_maps:
 *     a_bits[i,k] = pred(X[i,k]) & keep_bits[i,k] & (X[i,k] != 0).
 * Always uses the MMM_PATH_PAIRS kernel; meant for activations of few rows (decode), correct for
 * any shape with ldy * sizeof(element) below 2^20 bytes.  Errors: MMM_ERR_INVALID_ARG (NULL
 * pointer, bad pred, misaligned keep_bits), MMM_ERR_SHAPE (also: ldy beyond that), MMM_ERR_DTYPE, MMM_ERR_MAPS_MISMATCH (B side not built, or built for another
 * element type), MMM_ERR_DEVICE. */
mmm_status mmm_matmul_fused(const mmm_maps *maps, mmm_dtype dt,
                            const void *X, int64_t ldx, const mmm_mask_a *ma,
                            const void *Y, int64_t ldy,
                            void *C, int64_t ldc, int32_t accumulate, void *hip_stream);

/* The same multiplication for callers that cannot allocate and must not have
 * memory allocated on their behalf while they run: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  mmm_matmul keeps the
 * partial sums of a K-split multiplication (few tiles of C, long K: the decode
 * shape) in the caller's workspace; this entry point keeps them in an array that
 * is part of the library's own device image instead (MMM_STATIC_SCRATCH_BYTES
 * bytes on every GPU the library runs on, held until the process ends), so the
 * call touches no allocator at all.  Same arguments, same launch plan, same
 * kernels and bit-identical results as mmm_matmul.
 * Limit: split_k * M * N * 4 bytes of partial sums must fit the array, else
 * MMM_ERR_WORKSPACE (mmm_last_device_error() then says how many bytes were
 * needed); a plan that does not split K needs no scratch and is always accepted.
 * The partial sums are fully overwritten before they are read, so nothing is
 * cleared between calls.  All calls on one GPU share that GPU's array: two calls
 * that may run at the same time on one GPU (different streams) race; calls on
 * one stream do not.
 * Errors: as mmm_matmul, plus MMM_ERR_WORKSPACE as described. */
#define MMM_STATIC_SCRATCH_BYTES (16u << 20)
mmm_status mmm_matmul_static_scratch(const mmm_maps *maps, mmm_dtype dt,
                                     const void *X, int64_t ldx, const void *Y, int64_t ldy,
                                     void *C, int64_t ldc, int32_t accumulate, void *hip_stream);

/* Process-wide tuning knobs (for benchmarking; the defaults choose by shape).
 *   "matmul_variant": -1 = automatic, else index of a compiled tile variant
 *   "split_k"       :  0 = automatic, else the number of K splits to use
 *   "matmul_path"   : -1 = automatic, else MMM_PATH_MATRIX or MMM_PATH_PAIRS
 * Errors: MMM_ERR_INVALID_ARG (unknown name or value out of range). */
mmm_status mmm_set_option(const char *name, int64_t value);

/* Fix the launch plan of one handle: tile variant (-1 = leave it to the options
 * above / the automatic choice) and number of K splits (0 = likewise).  A
 * variant that computes too few rows for the matrix, or more splits than K has
 * steps or the workspace has room for, is adjusted as in the automatic choice;
 * mmm_matmul_plan reports what will be used.  This is the tuning knob the paper
 * leaves to an autotuner (section 3, "Optimizations": the base vector multiple).
 * Errors: MMM_ERR_INVALID_ARG (maps NULL, values out of range). */
mmm_status mmm_maps_set_plan(mmm_maps *maps, int32_t variant, int32_t split_k);

/* Number of compiled tile variants and a short description of variant i
 * (NULL if i is out of range). */
int32_t mmm_matmul_variant_count(void);
const char *mmm_matmul_variant_name(int32_t i);

/* The launch plan mmm_matmul would use for these maps: variant index, K splits,
 * grid size.  Any out pointer may be NULL.  Errors: MMM_ERR_INVALID_ARG. */
mmm_status mmm_matmul_plan(const mmm_maps *maps, mmm_dtype dt, int32_t *variant, int32_t *split_k,
                           int64_t *workgroups);

const char *mmm_status_string(mmm_status st);

/* Text describing the HIP failure behind the most recent MMM_ERR_DEVICE returned
 * on the calling thread ("" if none).  The pointer stays valid for the thread. */
const char *mmm_last_device_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MMM_H */
