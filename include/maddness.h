/*
 * maddness.h - C ABI of the MADDNESS inference path on one AMD MI355X (gfx950).
 *
 * The method approximates A B for A (N x D, rows are samples) and B (D x M) as
 * alpha f(g(A), h(B)) + beta (paper, Section 1.1):
 *   g  encodes every row of A with C hashing trees (Section 4.1, Algorithm 1),
 *   h  turns B into C tables of K = 16 entries per output column and quantises
 *      them to 8 bits (Section 3 "Table Construction"; Appendix A),
 *   f  sums, for every row and output column, the C table entries the codes
 *      select (Section 4.4), and alpha, beta undo the quantisation.
 * Learning the trees and prototypes (Sections 4.2-4.3) is set-up work, done once per
 * problem; its result is passed in through maddness_params.  It may run anywhere (the
 * package ships a CPU learner); maddness_learn_trees / maddness_learn_prototypes at the
 * end of this header run it on the GPU.
 *
 * Conventions common to every call
 *   - Unless a parameter says "host", every pointer is a DEVICE pointer to
 *     memory owned by the caller.  The library allocates nothing, keeps no
 *     state between calls (apart from one-time per-process kernel attributes
 *     and the switches of maddness_set_option) and never modifies an input.
 *     Outputs must not alias inputs.
 *   - Work is enqueued on the HIP stream given as `stream` (a hipStream_t cast
 *     to void*; NULL is the null stream) and the call returns without
 *     synchronising.
 *   - Matrices are row-major; ld* is the row stride in ELEMENTS.
 *   - The return value is a maddness_status; argument errors are detected on
 *     the host before anything is launched, and maddness_last_error() gives a
 *     text for the last failure on the calling thread.
 *   - N = 0 is valid and does nothing.
 *   - Fixed by the paper: K = 16 leaves/prototypes per codebook, tree depth 4.
 *     Limits of this implementation: 1 <= C <= 256 (255 C must fit the 16-bit
 *     accumulators of the exact sum, Section 4.4), D, M >= 1.
 */
#ifndef MADDNESS_H
#define MADDNESS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MADDNESS_K 16
#define MADDNESS_MAX_C 256

typedef enum {
    MADDNESS_OK = 0,
    MADDNESS_E_INVAL = -1,       /* null pointer, negative size, ld too small */
    MADDNESS_E_UNSUPPORTED = -2, /* C outside 1..MADDNESS_MAX_C, workspace too small,
                                    averaged aggregation with C not a multiple of 16 */
    MADDNESS_E_ALIGN = -3,       /* pointer not aligned to its element size */
    MADDNESS_E_HIP = -4          /* the HIP runtime refused a launch */
} maddness_status;

/*
 * Learned parameters (Sections 4.1-4.3).  The struct itself lives in HOST
 * memory; the three arrays it points to live in DEVICE memory.
 *
 * split_dims[c][t]   column of A that level t+1 (t = 0..3) of tree c tests
 *                    (Algorithm 1's j^1..j^4), an absolute index in [0, D).
 *                    An index outside [0, D) is clamped into it by the kernels,
 *                    so a corrupt array gives wrong codes, never a bad access.
 * thresholds[c][s]   Algorithm 1's v^t_i for tree c, the four arrays stored one
 *                    after the other: level t (1..4), node i (1..2^(t-1)) is at
 *                    s = 2^(t-1) - 1 + (i - 1).  s = 15 is padding, never read.
 * prototypes[c][k][d] row k of codebook c of the dense prototype matrix P of
 *                    Section 4.3 (K C x D, row-major).  Only read by
 *                    maddness_build_luts; may be NULL for the other calls.
 */
typedef struct {
    int32_t D;
    int32_t C;
    const int32_t *split_dims; /* [C][4]     */
    const float *thresholds;   /* [C][16]    */
    const float *prototypes;   /* [C][16][D] */
} maddness_params;

/*
 * g(A): Algorithm 1 for every row and every codebook (Section 4.1).
 * For t = 1..4: b = (A[n][j^t] >= v^t_i), i <- 2i - 1 + b, starting at i = 1.
 * The comparison is an ordered >=: equal goes right, a NaN goes left.
 *
 * A      [N][lda] fp32, lda >= D.
 * codes  [N][(C+1)/2] bytes, no row padding.  Byte b of a row holds the code of
 *        codebook 2b in bits 0..3 and that of codebook 2b+1 in bits 4..7 (zero
 *        when C is odd and 2b+1 == C).  A code is the leaf index minus 1, 0..15;
 *        its most significant bit is the level-1 decision.
 */
int maddness_encode(const maddness_params *params, const float *A, int64_t N, int64_t lda,
                    uint8_t *codes, void *stream);

/*
 * h(B): tables and their 8-bit quantisation (Section 3; Appendix A).
 *   T[c][k][m]  = sum_d prototypes[c][k][d] * B[d][m]      (fp64 matrix cores)
 *   delta[c][m] = min_k T[c][k][m]
 *   r[m]        = max_{c,k} (T[c][k][m] - delta[c][m])
 *   l[m]        = the largest integer with r[m] 2^l <= 255, kept in [-126, 126];
 *                 0 when r[m] is 0 or not finite
 *   luts[c][k][m] = clamp(round-half-even((T - delta) 2^l), 0, 255)
 *   scale[m]    = 2^-l[m]             (alpha of Section 1.1, one per column)
 *   offset[m]   = (float) sum_c delta[c][m]   (beta)
 * The scale is a power of two as in Appendix A, chosen from the widest table of
 * the column so that no entry exceeds 255, here per output column.
 *
 * B         [D][ldb] fp32, ldb >= M.
 * luts      [C][16][M] bytes (m contiguous).
 * scale, offset  [M] fp32.
 * workspace device scratch of at least maddness_build_luts_workspace(D, C, M)
 *           bytes, 8-byte aligned; contents undefined afterwards.
 * Results for non-finite prototypes or B are unspecified (no fault).
 */
size_t maddness_build_luts_workspace(int32_t D, int32_t C, int32_t M);
int maddness_build_luts(const maddness_params *params, const float *B, int32_t M, int64_t ldb,
                        uint8_t *luts, float *scale, float *offset, void *workspace,
                        size_t workspace_bytes, void *stream);

/*
 * h(B) with the quantisation of Appendix A as printed: offsets per codebook and
 * one scale, both pooled over the output columns,
 *   delta[c] = min_{m,k} T[c][k][m]
 *   r        = max_{c,m,k} (T[c][k][m] - delta[c])
 *   l        = the largest integer with r 2^l <= 255 (kept in [-126, 126]; 0 when r
 *              is 0 or not finite)
 *   luts[c][k][m] = clamp(round-half-even((T - delta[c]) 2^l), 0, 255)
 *   scale[m] = 2^-l and offset[m] = (float) sum_c delta[c] for every m
 * (alpha and beta are written per column so that maddness_scan and
 * maddness_encode_scan take either variant).  Arguments, workspace and error
 * behaviour as for maddness_build_luts.
 */
int maddness_build_luts_pooled(const maddness_params *params, const float *B, int32_t M, int64_t ldb,
                               uint8_t *luts, float *scale, float *offset, void *workspace,
                               size_t workspace_bytes, void *stream);

/*
 * maddness_build_luts for callers that cannot allocate device memory (code under HIP
 * graph capture, serving loops, harnesses that forbid hipMalloc): the workspace is an
 * array of MADDNESS_STATIC_WORKSPACE_BYTES bytes inside the library, one per GPU,
 * held from the first use on that GPU until the process ends.  The call allocates
 * nothing; same kernels, same results as maddness_build_luts, bit for bit.
 * Shapes whose workspace (maddness_build_luts_workspace) exceeds that size are
 * refused with MADDNESS_E_UNSUPPORTED before anything is launched (C = 64, M = 512
 * needs 4.3 MiB).  Every call on one GPU uses the same array: calls that overlap in
 * time on one GPU (different streams, different threads) race and must be ordered by
 * the caller.  Nothing in the array has to be cleared between calls: every word a
 * call reads it has written itself before.
 */
#define MADDNESS_STATIC_WORKSPACE_BYTES 8388608
int maddness_build_luts_static(const maddness_params *params, const float *B, int32_t M, int64_t ldb,
                               uint8_t *luts, float *scale, float *offset, void *stream);

/*
 * f and alpha f + beta (Section 4.4 as an exact sum; Section 1.1):
 *   acc[n][m] = sum_c luts[c][code(n, c)][m]        exact, unsigned
 *   out[n][m] = fma((float)acc[n][m], scale[m], offset[m])
 *
 * codes  as written by maddness_encode.
 * out    [N][ldo] fp32, ldo >= M; may be NULL if only acc is wanted.  Any ldo >= M and
 *        any alignment is accepted; the kernels for many rows write whole 128-byte
 *        lines when the rows of out start on them (out 128-byte aligned, ldo a
 *        multiple of 32) and are slower otherwise (measured: N = 2^20, C = 32,
 *        M = 1000: 1.43 ms with ldo = 1000, 1.29 ms with ldo = 1024).
 * acc    [N][M] uint16 (dense), may be NULL.  At least one of out/acc non-NULL.
 */
int maddness_scan(int32_t C, int32_t M, const uint8_t *codes, int64_t N, const uint8_t *luts,
                  const float *scale, const float *offset, float *out, int64_t ldo,
                  uint16_t *acc, void *stream);

/*
 * maddness_encode followed by maddness_scan in one kernel: the codes stay in
 * registers and on-chip memory.  Results are bit-identical to the two calls.
 * acc and codes are optional extra outputs (NULL to skip); out may be NULL only
 * if acc is not.
 */
int maddness_encode_scan(const maddness_params *params, const float *A, int64_t N, int64_t lda,
                         int32_t M, const uint8_t *luts, const float *scale,
                         const float *offset, float *out, int64_t ldo, uint16_t *acc,
                         uint8_t *codes, void *stream);

/*
 * f by pairwise averages instead of an exact sum (Section 4.4; Appendix D), with
 * the paper's block size U = 16: the codebooks are taken in blocks of 16
 * consecutive ones, and within a block the 16 looked-up bytes are reduced by a
 * balanced tree of rounding averages avg(a, b) = floor((a + b + 1) / 2), pairing
 * neighbours (0,1), (2,3), ... at every level, each result again 8 bits wide.
 *   S[n][m]   = sum over blocks of the block's average          exact, unsigned
 *   acc[n][m] = 16 S[n][m]
 *   out[n][m] = fma((float)(16 S[n][m] - C), scale[m], offset[m])
 * 16 S overestimates the exact sum by C log2(16) / 4 = C in expectation for
 * uniformly distributed low bits (Theorem D.1), which the formula takes off
 * before alpha and beta are applied.
 * Arguments as for maddness_scan / maddness_encode_scan; C must be a multiple
 * of 16 (MADDNESS_E_UNSUPPORTED otherwise).  The codes written by
 * maddness_encode_scan_averaged are those of maddness_encode.
 */
int maddness_scan_averaged(int32_t C, int32_t M, const uint8_t *codes, int64_t N, const uint8_t *luts,
                           const float *scale, const float *offset, float *out, int64_t ldo,
                           uint16_t *acc, void *stream);
int maddness_encode_scan_averaged(const maddness_params *params, const float *A, int64_t N, int64_t lda,
                                  int32_t M, const uint8_t *luts, const float *scale,
                                  const float *offset, float *out, int64_t ldo, uint16_t *acc,
                                  uint8_t *codes, void *stream);

/*
 * g(A), and g followed by f, for inputs that are not fp32 or that are stored by
 * columns.  The tree walk only compares single elements of a row with thresholds,
 * so narrow data are encoded as they are (Appendix E.6: 8-bit image data used
 * directly), and it touches four columns per codebook, so a matrix stored by
 * columns is read at O(C) instead of O(D) elements per row (Section 4.1,
 * Section 5.2).  Every element is widened to the fp32 number of the same value
 * (exact for all three narrow types) and Algorithm 1 runs on those values with the
 * fp32 thresholds of maddness_params; results are those of maddness_encode /
 * maddness_encode_scan on the widened, row-major matrix, bit for bit.
 *
 * A       device pointer to elements of `dtype`, aligned to the element size.
 * dtype   a maddness_dtype: IEEE binary32, IEEE binary16, bfloat16, unsigned byte.
 * layout  MADDNESS_ROW_MAJOR: element (n, d) at index n * lda + d, lda >= D;
 *         MADDNESS_COL_MAJOR: at index d * lda + n, lda >= N.
 * The remaining arguments, the outputs and the error behaviour are those of
 * maddness_encode and maddness_encode_scan (exact sum).  An unknown dtype or
 * layout gives MADDNESS_E_INVAL.
 */
typedef enum { MADDNESS_F32 = 0, MADDNESS_F16 = 1, MADDNESS_BF16 = 2, MADDNESS_U8 = 3 } maddness_dtype;
typedef enum { MADDNESS_ROW_MAJOR = 0, MADDNESS_COL_MAJOR = 1 } maddness_layout;

int maddness_encode_typed(const maddness_params *params, const void *A, int32_t dtype, int32_t layout,
                          int64_t N, int64_t lda, uint8_t *codes, void *stream);
int maddness_encode_scan_typed(const maddness_params *params, const void *A, int32_t dtype,
                               int32_t layout, int64_t N, int64_t lda, int32_t M, const uint8_t *luts,
                               const float *scale, const float *offset, float *out, int64_t ldo,
                               uint16_t *acc, uint8_t *codes, void *stream);

/*
 * The learning step on the GPU (set-up, once per problem).
 *
 * maddness_learn_trees builds the C hashing trees from a training matrix (Section 4.2,
 * Algorithm 2, with the subroutines of Appendix C, Algorithms 3 and 4).  Tree c only looks
 * at the columns [subspace_bounds[c][0], subspace_bounds[c][1]) of A_train.  Level by level
 * (four levels), for the buckets B_1..B_n of the level (the rows that reach each node):
 *   - the candidate columns are the min(4, width) columns with the largest
 *     sum_i L(j, B_i), L(j, B) = sum_{x in B} (x_j - mean_B(x_j))^2 (the loss equation of
 *     Section 4.2), largest first, equal sums in column order;
 *   - for a candidate j every bucket gets the threshold that minimises the summed loss
 *     L(B_below) + L(B_above) of its two children over all columns of the subspace
 *     (Algorithm 3: rows sorted by x_j, equal values in row order; Algorithm 4's running
 *     sums of x and x^2 from both ends; only positions between two different values of x_j
 *     count; the first minimum wins).  The threshold is the fp32 midpoint v of the two
 *     neighbouring values with lower < v <= upper.  A bucket that cannot be split (empty,
 *     one row, x_j constant) keeps its loss L(B) and gets that value (0 if empty);
 *   - the candidate with the smallest loss summed over the buckets is taken (the first of
 *     equal ones), and every bucket is split: x_j >= v goes to the upper child.
 * All sums are fp64 and run in the order the algorithms state them (rows of a bucket in
 * sorted or row order, columns in column order), so the result does not depend on the
 * launch and is reproducible to the bit.
 *
 * A_train          [N][lda] fp32, lda >= D, 1 <= N < 2^29 rows (MADDNESS_E_UNSUPPORTED beyond: a sort key
 *                  holds bucket, value and row number in 64 bits).
 * subspace_bounds  HOST array [C][2]: first and one-past-last column of every codebook,
 *                  0 <= first < last <= D.  A subspace may be at most 128 columns wide
 *                  (MADDNESS_E_UNSUPPORTED beyond; the running sums of a bucket live in
 *                  on-chip memory).
 * split_dims       out [C][4], thresholds out [C][16] (slot 15 = 0): as maddness_params
 *                  takes them.
 * train_codes      out [N][C], ONE BYTE per code (not packed): the leaf minus 1 of every
 *                  training row in every tree; may be NULL.
 * workspace        device scratch of at least maddness_learn_trees_workspace(...) bytes,
 *                  256-byte aligned (maddness_learn_trees_workspace returns 0 for arguments
 *                  it cannot size).
 *
 * maddness_learn_prototypes computes the prototype matrix P from the training codes:
 *   ridge != 0   P = (G^T G + lambda I)^-1 G^T A_train (Section 4.3), G the one-hot matrix of
 *                the codes, by Cholesky factorisation in fp64; lambda > 0 (the paper: 1);
 *   ridge == 0   P[c][k] = mean of the training rows with code k in tree c on the codebook's
 *                own columns and 0 elsewhere (an empty bucket: 0) - the prototypes before the
 *                ridge step, the variant Section 5.1 calls MADDNESS-PQ.
 * prototypes       out [C][16][D] fp32, as maddness_params takes them.
 * workspace        at least maddness_learn_prototypes_workspace(D, C) bytes, 256-byte aligned.
 *
 * Both calls are enqueued on `stream` and return without synchronising; errors as everywhere.
 */
size_t maddness_learn_trees_workspace(int64_t N, int32_t D, int32_t C, const int32_t *subspace_bounds);
int maddness_learn_trees(const float *A_train, int64_t N, int64_t lda, int32_t D, int32_t C,
                         const int32_t *subspace_bounds, int32_t *split_dims, float *thresholds,
                         uint8_t *train_codes, void *workspace, size_t workspace_bytes, void *stream);
size_t maddness_learn_prototypes_workspace(int32_t D, int32_t C);
int maddness_learn_prototypes(const uint8_t *train_codes, const float *A_train, int64_t N, int64_t lda,
                              int32_t D, int32_t C, const int32_t *subspace_bounds, int32_t ridge,
                              double lambda, float *prototypes, void *workspace, size_t workspace_bytes,
                              void *stream);

/*
 * Process-wide switches for tests and measurements (Section 4.4 describes f as table
 * lookups and integer additions; MADDNESS_OPT_KERNELS = 1 keeps the library to kernels
 * of exactly that form).  Normal use needs none of them: every switch starts at 0, "the
 * library chooses", and no switch changes a result - every kernel gives the same bits.
 * They select WHICH kernel computes it, so that each kernel can be held against the
 * CPU reference and timed on the same inputs.  The environment is never read.
 *
 * MADDNESS_OPT_KERNELS      0  automatic.
 *                           1  no matrix-core kernels: the table scan runs as LDS
 *                              lookups and packed integer additions on the vector ALUs
 *                              (the exact scan otherwise runs, for many rows, as the
 *                              product of the one-hot code matrix of Section 4.3 with
 *                              the tables on the int8 matrix cores).
 *                           2  only the general kernels (any shape, no specialisation).
 * MADDNESS_OPT_PHASED_ROWS  n >= 2: at most n rows per wavefront and region (rounded up to
 *                           a multiple of 256 for A stored by columns) in the kernels that
 *                           work in phases, so that few rows already make many regions;
 *                           0: as many as on-chip memory holds.
 * MADDNESS_OPT_COLS_RUN     1, 2 or 4 rows per lane in the by-columns kernels; 0: automatic.
 * MADDNESS_OPT_MAX_WORKGROUPS  n >= 1: the phased kernels launch at most n workgroups, so
 *                           that each takes several regions in turn; 0: one per compute unit.
 *
 * maddness_set_option returns MADDNESS_E_INVAL for an unknown option or a value outside
 * the ranges above; maddness_get_option returns the current value, or -1 for an unknown
 * option.  A call that runs concurrently with maddness_set_option sees the old or the new
 * value.
 */
typedef enum {
    MADDNESS_OPT_KERNELS = 0,
    MADDNESS_OPT_PHASED_ROWS = 1,
    MADDNESS_OPT_COLS_RUN = 2,
    MADDNESS_OPT_MAX_WORKGROUPS = 3
} maddness_option;
enum { MADDNESS_KERNELS_AUTO = 0, MADDNESS_KERNELS_NO_MATRIX_CORES = 1, MADDNESS_KERNELS_GENERAL = 2 };

int maddness_set_option(int32_t option, int32_t value);
int32_t maddness_get_option(int32_t option);

/* Text of the last error on this thread (host string owned by the library). */
const char *maddness_last_error(void);

/*
 * Diagnostic for tests and benchmarks: which kernel the last launching call on this
 * thread selected, as "<kernel name> [<template arguments of the instance>]", e.g.
 * "rows_kernel [MODE = 0, C = 32, ...]"; for a call that launches several kernels, the
 * first (the one that does the bulk of the work); "" if the call launched nothing.
 * Host string owned by the library, valid until the next call on this thread.
 */
const char *maddness_last_kernel(void);

#ifdef __cplusplus
}
#endif
#endif /* MADDNESS_H */
