/*
 * CPU oracle for Masked Matrix Multiplication, C = M(X) x N(Y).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP path is checked against.  It shares no code with the HIP path and must
 * never be called from it.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may use it.
 *
 * What it follows (paper: "Masked Matrix Multiplication for Emergent
 * Sparsity", arXiv 2402.14118):
 *   - Problem statement, sections 1 and 3: A = M(X), B = N(Y), C = A x B with
 *     X, Y dense and M, N masks evaluated at run time; A has random element
 *     sparsity, B has block-random sparsity in aligned, contiguous 1 x bw
 *     pieces of each row (Fig. "Types of sparsity").
 *   - Dense definition: Fig. "Simple dense matrix multiplication"
 *     (i-k-j loops, C[i,j] += A[i,k]*B[k,j]).
 *   - A-side skipping: Fig. "A simple optimization to skip computation when A
 *     is sparse" (skip the whole row of B when A[i,k] == 0).
 *   - B-side pattern bits: section 3 "Block-Random Sparsity in B" and Fig.
 *     "Preprocessing patterns": one bit per vector, 1 = some non-zero value,
 *     0 = all zero.
 *   - A-side map: section 3 "Optimizations", Fig. "Blocked sparse row
 *     preprocessing": which elements of a row are non-zero.
 *
 * MMM only skips products that are zero, so it reaches exactly the plain
 * result; the oracle therefore is the plain definition written out, with a
 * double-precision accumulator so that it spends none of the error budget.
 * The paper also reports double-precision runs (section 4, table of the server
 * machines: float and double); the *_f64 functions are the same definitions on
 * double inputs, accumulated in long double (64-bit significand on x86) for
 * the same reason.
 *
 * Readings taken where the paper is silent or at odds with itself:
 *   - bit = 1 means occupied / non-zero (text and caption; the pseudocode of
 *     Fig. "Preprocessing function pointer arrays" tests "== 0", a slip);
 *   - bit order is ours: LSB-first little-endian 64-bit words, rows padded
 *     with zero bits (the paper prints patterns MSB-first: "01010000" selects
 *     the 2nd and 4th vector);
 *   - zero means IEEE equality with 0: +0 and -0 are zero, denormals and NaN
 *     are not;
 *   - a map bit is (mask keeps it) AND (value is non-zero); the B mask acts on
 *     whole aligned blocks only;
 *   - C is overwritten (C = A x B); the listings' "+=" is the optional
 *     accumulate mode;
 *   - masked-out products contribute exactly nothing (they are skipped, never
 *     multiplied).
 *
 * Pins: tests/test_oracle_pins.py (brute force on tiny inputs, textbook GEMM
 * in the all-keep case, identity and zero-mask invariants, exact integer
 * inputs, numpy.packbits for the bit layout, closed-form keep fractions, the
 * paper's printed pattern example).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_PRED_NONZERO = 0, ORACLE_PRED_GT = 1, ORACLE_PRED_ABS_GT = 2 };

static inline int get_bit(const uint64_t *words, int64_t idx)
{
    return (int)((words[idx >> 6] >> (idx & 63)) & 1u);
}

static inline void set_bit(uint64_t *words, int64_t idx)
{
    words[idx >> 6] |= (uint64_t)1 << (idx & 63);
}

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* How many threads the row loops may use from now on (timing on one core and on all). */
void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* M evaluated element by element (sections 1, 3: masks evaluated at run time;
 * zero test as in Fig. "skip computation when A is sparse").
 * a_bits: M x ceil(K/64) words, cleared here. */
void oracle_a_bits(const float *X, int64_t M, int64_t K, int64_t ldx, int pred, float threshold,
                   const uint64_t *keep_bits, uint64_t *a_bits)
{
    const int64_t W = (K + 63) / 64;
    memset(a_bits, 0, (size_t)(M * W) * sizeof(uint64_t));
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t k = 0; k < K; ++k) {
            const float x = X[i * ldx + k];
            int keep;
            if (pred == ORACLE_PRED_GT)
                keep = x > threshold;
            else if (pred == ORACLE_PRED_ABS_GT)
                keep = fabsf(x) > threshold;
            else
                keep = 1;
            if (keep_bits && !get_bit(keep_bits + i * W, k))
                keep = 0;
            if (keep && x != 0.0f)
                set_bit(a_bits + i * W, k);
        }
    }
}

/* N evaluated on whole aligned 1 x bw blocks; a kept block is occupied iff it
 * holds any non-zero (section 3, "Block-Random Sparsity in B"; caption of Fig.
 * "Preprocessing patterns").  b_bits: K x ceil(NB/64) words, cleared here. */
void oracle_b_bits(const float *Y, int64_t K, int64_t N, int64_t ldy, int64_t bw,
                   const uint64_t *keep_rows, const uint64_t *keep_blocks, uint64_t *b_bits)
{
    const int64_t NB = N / bw;
    const int64_t W = (NB + 63) / 64;
    memset(b_bits, 0, (size_t)(K * W) * sizeof(uint64_t));
    for (int64_t k = 0; k < K; ++k) {
        if (keep_rows && !get_bit(keep_rows, k))
            continue;
        for (int64_t jb = 0; jb < NB; ++jb) {
            if (keep_blocks && !get_bit(keep_blocks + k * W, jb))
                continue;
            int any = 0;
            for (int64_t j = jb * bw; j < (jb + 1) * bw; ++j)
                if (Y[k * ldy + j] != 0.0f)
                    any = 1;
            if (any)
                set_bit(b_bits + k * W, jb);
        }
    }
}

/* A = M(X), B = N(Y) written out densely (sections 1, 3). */
void oracle_materialize_a(const float *X, int64_t M, int64_t K, int64_t ldx,
                          const uint64_t *a_bits, float *A)
{
    const int64_t W = (K + 63) / 64;
    for (int64_t i = 0; i < M; ++i)
        for (int64_t k = 0; k < K; ++k)
            A[i * K + k] = get_bit(a_bits + i * W, k) ? X[i * ldx + k] : 0.0f;
}

void oracle_materialize_b(const float *Y, int64_t K, int64_t N, int64_t ldy, int64_t bw,
                          const uint64_t *b_bits, float *B)
{
    const int64_t NB = N / bw;
    const int64_t W = (NB + 63) / 64;
    for (int64_t k = 0; k < K; ++k)
        for (int64_t j = 0; j < N; ++j)
            B[k * N + j] = get_bit(b_bits + k * W, j / bw) ? Y[k * ldy + j] : 0.0f;
}

/* Fig. "Simple dense matrix multiplication" on already materialised A and B:
 * no skipping at all, double accumulator, double result.  Tiny sizes only. */
void oracle_dense_ref(const float *A, const float *B, int64_t M, int64_t K, int64_t N, double *C64)
{
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k)
                s += (double)A[i * K + k] * (double)B[k * N + j];
            C64[i * N + j] = s;
        }
}

/* The masked product in the loop order of Fig. "skip computation when A is
 * sparse" (i, then k, then j), skipping zero A[i,k] and unoccupied blocks of
 * B[k,:] (Fig. "MMM Pseudocode").  One row of double accumulators; a single
 * rounding to float at the end.  absAB (optional) receives
 * sum_k |A[i,k]|*|B[k,j]|, the magnitude term of the acceptance bound.
 * With accumulate != 0 the previous C[i,j] is added (in double) first.
 * Rows [row0, row1) only, so a bounded sample can be timed. */
void oracle_mmm_rows(const float *X, int64_t ldx, const float *Y, int64_t ldy,
                     const uint64_t *a_bits, const uint64_t *b_bits,
                     int64_t M, int64_t K, int64_t N, int64_t bw,
                     int64_t row0, int64_t row1,
                     float *C, int64_t ldc, double *absAB, int accumulate)
{
    const int64_t WA = (K + 63) / 64;
    const int64_t NB = N / bw;
    const int64_t WB = (NB + 63) / 64;
    (void)M;
#pragma omp parallel
    {
        double *acc = (double *)malloc((size_t)N * sizeof(double));
        double *mag = (double *)malloc((size_t)N * sizeof(double));
#pragma omp for schedule(dynamic, 4)
        for (int64_t i = row0; i < row1; ++i) {
            for (int64_t j = 0; j < N; ++j) {
                acc[j] = accumulate ? (double)C[i * ldc + j] : 0.0;
                mag[j] = accumulate ? fabs((double)C[i * ldc + j]) : 0.0;
            }
            for (int64_t k = 0; k < K; ++k) {
                if (!get_bit(a_bits + i * WA, k))
                    continue;
                const double a = (double)X[i * ldx + k];
                for (int64_t jb = 0; jb < NB; ++jb) {
                    if (!get_bit(b_bits + k * WB, jb))
                        continue;
                    for (int64_t j = jb * bw; j < (jb + 1) * bw; ++j) {
                        const double b = (double)Y[k * ldy + j];
                        acc[j] += a * b;
                        mag[j] += fabs(a) * fabs(b);
                    }
                }
            }
            for (int64_t j = 0; j < N; ++j) {
                C[i * ldc + j] = (float)acc[j];
                if (absAB)
                    absAB[i * N + j] = mag[j];
            }
        }
        free(acc);
        free(mag);
    }
}

void oracle_mmm(const float *X, int64_t ldx, const float *Y, int64_t ldy,
                const uint64_t *a_bits, const uint64_t *b_bits,
                int64_t M, int64_t K, int64_t N, int64_t bw,
                float *C, int64_t ldc, double *absAB, int accumulate)
{
    oracle_mmm_rows(X, ldx, Y, ldy, a_bits, b_bits, M, K, N, bw, 0, M, C, ldc, absAB, accumulate);
}

/* One output element, by the definition, for sampled checks at full size. */
void oracle_mmm_element(const float *X, int64_t ldx, const float *Y, int64_t ldy,
                        const uint64_t *a_bits, const uint64_t *b_bits,
                        int64_t K, int64_t N, int64_t bw, int64_t i, int64_t j,
                        double *c, double *mag)
{
    const int64_t WA = (K + 63) / 64;
    const int64_t WB = (N / bw + 63) / 64;
    double s = 0.0, m = 0.0;
    for (int64_t k = 0; k < K; ++k) {
        if (!get_bit(a_bits + i * WA, k) || !get_bit(b_bits + k * WB, j / bw))
            continue;
        const double a = (double)X[i * ldx + k], b = (double)Y[k * ldy + j];
        s += a * b;
        m += fabs(a) * fabs(b);
    }
    *c = s;
    *mag = m;
}

/* Counts: non-zeros of A, occupied blocks of B, and useful multiply-adds
 * sum_k (#non-zeros in column k of A) * bw * (#occupied blocks in row k of B),
 * i.e. the number of products the loop of Fig. "MMM Pseudocode" performs. */
void oracle_counts(const uint64_t *a_bits, const uint64_t *b_bits,
                   int64_t M, int64_t K, int64_t N, int64_t bw,
                   uint64_t *nnz_a, uint64_t *occ_b, uint64_t *useful_macs)
{
    const int64_t WA = (K + 63) / 64;
    const int64_t NB = N / bw;
    const int64_t WB = (NB + 63) / 64;
    uint64_t na = 0, nb = 0, macs = 0;
    for (int64_t k = 0; k < K; ++k) {
        uint64_t col = 0, row = 0;
        for (int64_t i = 0; i < M; ++i)
            col += (uint64_t)get_bit(a_bits + i * WA, k);
        for (int64_t jb = 0; jb < NB; ++jb)
            row += (uint64_t)get_bit(b_bits + k * WB, jb);
        na += col;
        nb += row;
        macs += col * row * (uint64_t)bw;
    }
    *nnz_a = na;
    *occ_b = nb;
    *useful_macs = macs;
}

/* ---- double-precision inputs (section 4, table of the server machines) ------------------------
 * The same definitions as above with X, Y and C in double. */
void oracle_a_bits_f64(const double *X, int64_t M, int64_t K, int64_t ldx, int pred, float threshold,
                       const uint64_t *keep_bits, uint64_t *a_bits)
{
    const int64_t W = (K + 63) / 64;
    memset(a_bits, 0, (size_t)(M * W) * sizeof(uint64_t));
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t k = 0; k < K; ++k) {
            const double x = X[i * ldx + k];
            int keep;
            if (pred == ORACLE_PRED_GT)
                keep = x > (double)threshold;
            else if (pred == ORACLE_PRED_ABS_GT)
                keep = fabs(x) > (double)threshold;
            else
                keep = 1;
            if (keep_bits && !get_bit(keep_bits + i * W, k))
                keep = 0;
            if (keep && x != 0.0)
                set_bit(a_bits + i * W, k);
        }
    }
}

void oracle_b_bits_f64(const double *Y, int64_t K, int64_t N, int64_t ldy, int64_t bw,
                       const uint64_t *keep_rows, const uint64_t *keep_blocks, uint64_t *b_bits)
{
    const int64_t NB = N / bw;
    const int64_t W = (NB + 63) / 64;
    memset(b_bits, 0, (size_t)(K * W) * sizeof(uint64_t));
    for (int64_t k = 0; k < K; ++k) {
        if (keep_rows && !get_bit(keep_rows, k))
            continue;
        for (int64_t jb = 0; jb < NB; ++jb) {
            if (keep_blocks && !get_bit(keep_blocks + k * W, jb))
                continue;
            int any = 0;
            for (int64_t j = jb * bw; j < (jb + 1) * bw; ++j)
                if (Y[k * ldy + j] != 0.0)
                    any = 1;
            if (any)
                set_bit(b_bits + k * W, jb);
        }
    }
}

/* Fig. "skip computation when A is sparse" / Fig. "MMM Pseudocode" on doubles: i, k, j loops that
 * skip zero A[i,k] and unoccupied blocks; one row of long double accumulators, one rounding to
 * double at the end; absAB as above. */
void oracle_mmm_rows_f64(const double *X, int64_t ldx, const double *Y, int64_t ldy,
                         const uint64_t *a_bits, const uint64_t *b_bits,
                         int64_t M, int64_t K, int64_t N, int64_t bw,
                         int64_t row0, int64_t row1,
                         double *C, int64_t ldc, double *absAB, int accumulate)
{
    const int64_t WA = (K + 63) / 64;
    const int64_t NB = N / bw;
    const int64_t WB = (NB + 63) / 64;
    (void)M;
#pragma omp parallel
    {
        long double *acc = (long double *)malloc((size_t)N * sizeof(long double));
        long double *mag = (long double *)malloc((size_t)N * sizeof(long double));
#pragma omp for schedule(dynamic, 4)
        for (int64_t i = row0; i < row1; ++i) {
            for (int64_t j = 0; j < N; ++j) {
                acc[j] = accumulate ? (long double)C[i * ldc + j] : 0.0L;
                mag[j] = accumulate ? fabsl((long double)C[i * ldc + j]) : 0.0L;
            }
            for (int64_t k = 0; k < K; ++k) {
                if (!get_bit(a_bits + i * WA, k))
                    continue;
                const long double a = (long double)X[i * ldx + k];
                for (int64_t jb = 0; jb < NB; ++jb) {
                    if (!get_bit(b_bits + k * WB, jb))
                        continue;
                    for (int64_t j = jb * bw; j < (jb + 1) * bw; ++j) {
                        const long double b = (long double)Y[k * ldy + j];
                        acc[j] += a * b;
                        mag[j] += fabsl(a) * fabsl(b);
                    }
                }
            }
            for (int64_t j = 0; j < N; ++j) {
                C[i * ldc + j] = (double)acc[j];
                if (absAB)
                    absAB[i * N + j] = (double)mag[j];
            }
        }
        free(acc);
        free(mag);
    }
}
