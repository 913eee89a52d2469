/*
 * CPU oracle for the LEARNING step of MADDNESS ("Multiplying Matrices Without
 * Multiplying", arXiv 2106.10860): the greedy construction of the hashing trees
 * (Section 4.2, Algorithm 2; Appendix C, Algorithms 3 and 4) and the prototypes
 * (bucket means, Section 4; ridge regression, Section 4.3).
 *
 * THIS IS TEST INFRASTRUCTURE, like maddness_oracle.c beside it: a plain, slow,
 * single-threaded statement of the algorithms in the paper's order and notation,
 * in fp64, for the tests to hold the product's learners against.  The product
 * shares no code with it and never calls it.
 *
 * Learning is a heuristic, so the oracle is the algorithm's steps, not a closed
 * form.  Readings of the passages that are silent or garbled:
 *   - Algorithm 4's inner loop adds row n of X (the printed X_{1,d} is a slip), and
 *     the reversed pass is turned back, so that tail_n is the SSE of rows n..N;
 *   - the loss a split position is judged by is Algorithm 4's: the SSE summed over
 *     ALL columns of the codebook's subspace (Section 4.2: "minimizes the sum of
 *     the losses in the buckets produced");
 *   - Algorithm 3's argmin runs over n = 1..N-1 (a split after the last row makes
 *     no child), and only over positions whose two neighbours differ in column j:
 *     Algorithm 1 sends x_j >= v right, so rows with equal x_j cannot be
 *     separated.  The first minimum wins.  The threshold is the midpoint of the two
 *     neighbours rounded to fp32, moved up to the upper neighbour if rounding
 *     brought it down to the lower one (lower < v <= upper must hold);
 *   - a bucket that cannot be split (fewer than two rows, or column j constant)
 *     keeps its loss L(B) (the loss equation of Section 4.2, two passes) and gets
 *     the column's value as threshold (0 if the bucket is empty);
 *   - heuristic_select_idxs (Section 4.2): the n = min(4, |J|) columns of the
 *     subspace with the largest L(j, B) summed over the buckets of the level,
 *     largest first, equal sums in index order; Algorithm 2 tries them in that
 *     order and keeps the first of equal losses (its "<" is strict);
 *   - ridge: P = (G^T G + lambda I)^-1 G^T A~ literally, by Cholesky
 *     factorisation, in fp64; an empty bucket's row of P comes out 0.
 *
 * Pins (tests/test_oracle_learn_pins.py): the loss equation against a library
 * variance; Algorithm 4 against two-pass sums of every prefix and suffix;
 * Algorithm 3 against brute force over all thresholds; the tree against brute
 * force over its candidate columns level by level, against Algorithm 1 run on the
 * training rows, and against data whose 16 clusters it must recover; ridge
 * against the closed form for one codebook, the normal equations, a library
 * solver and the singular-value bound of Lemma F.3; G against the row the paper
 * prints in Section 4.3.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_K 16
#define ORACLE_DEPTH 4
#define ORACLE_CANDIDATES 4

/* ------------------------------------------------------------------------
 * L(j, B) of Section 4.2: sum over the bucket of (x_j - mean_j)^2, two passes.
 * X is N x d (row stride ld); rows[0..n) are the bucket's rows in row order.
 * ---------------------------------------------------------------------- */
double oracle_bucket_loss(const float *X, int64_t ld, const int64_t *rows, int64_t n, int32_t j)
{
    if (n == 0) return 0.0;
    double sum = 0.0;
    for (int64_t r = 0; r < n; ++r) sum += (double)X[rows[r] * ld + j];
    const double mean = sum / (double)n;
    double loss = 0.0;
    for (int64_t r = 0; r < n; ++r) {
        const double e = (double)X[rows[r] * ld + j] - mean;
        loss += e * e;
    }
    return loss;
}

/* ------------------------------------------------------------------------
 * Algorithm 4 (Cumulative SSE).  X is n x d, contiguous.  out[i] (i = 0..n-1):
 * reverse = 0: SSE, summed over the columns, of rows 0..i;
 * reverse = 1: of rows i..n-1 (the rows are taken last to first and the result is
 * turned back).
 * ---------------------------------------------------------------------- */
void oracle_cumulative_sse(const float *X, int64_t n, int32_t d, int32_t reverse, double *out)
{
    if (n == 0) return;
    double *cumX = (double *)malloc(sizeof(double) * (size_t)d);
    double *cumX2 = (double *)malloc(sizeof(double) * (size_t)d);
    for (int64_t step = 0; step < n; ++step) {
        const int64_t row = reverse ? n - 1 - step : step;
        const double count = (double)(step + 1);
        double o = 0.0;
        for (int32_t c = 0; c < d; ++c) {
            const double x = (double)X[row * d + c];
            if (step == 0) {
                cumX[c] = x;
                cumX2[c] = x * x;
            } else {
                cumX[c] = cumX[c] + x;
                cumX2[c] = cumX2[c] + x * x;
                o = o + (cumX2[c] - (cumX[c] * cumX[c] / count));
            }
        }
        out[row] = o;   /* step 0: a single row has SSE 0 */
    }
    free(cumX);
    free(cumX2);
}

/* stable order of the bucket's rows by column j (equal values keep row order) */
typedef struct { float key; int64_t row; } sort_item;

static void merge_sort(sort_item *a, sort_item *tmp, int64_t n)
{
    if (n < 2) return;
    const int64_t h = n / 2;
    merge_sort(a, tmp, h);
    merge_sort(a + h, tmp, n - h);
    int64_t i = 0, k = h, o = 0;
    while (i < h && k < n) tmp[o++] = (a[k].key < a[i].key) ? a[k++] : a[i++];
    while (i < h) tmp[o++] = a[i++];
    while (k < n) tmp[o++] = a[k++];
    memcpy(a, tmp, sizeof(sort_item) * (size_t)n);
}

/* ------------------------------------------------------------------------
 * Algorithm 3 (Optimal Split Threshold Within a Bucket).
 * X N x d (row stride ld), bucket = rows[0..n) in row order, column j.
 * Writes the threshold and the loss of the two children.
 * ---------------------------------------------------------------------- */
void oracle_optimal_split_threshold(const float *X, int64_t ld, int32_t d, const int64_t *rows, int64_t n,
                                    int32_t j, float *v_out, double *loss_out)
{
    if (n == 0) { *v_out = 0.0f; *loss_out = 0.0; return; }
    sort_item *items = (sort_item *)malloc(sizeof(sort_item) * (size_t)n);
    sort_item *tmp = (sort_item *)malloc(sizeof(sort_item) * (size_t)n);
    for (int64_t r = 0; r < n; ++r) { items[r].key = X[rows[r] * ld + j]; items[r].row = rows[r]; }
    merge_sort(items, tmp, n);
    free(tmp);
    if (!(items[0].key < items[n - 1].key)) {
        /* column j is constant in this bucket (or the bucket has one row): no split */
        double loss = 0.0;
        for (int32_t c = 0; c < d; ++c) loss += oracle_bucket_loss(X, ld, rows, n, c);
        *v_out = items[0].key;
        *loss_out = loss;
        free(items);
        return;
    }
    float *Xsort = (float *)malloc(sizeof(float) * (size_t)n * (size_t)d);
    for (int64_t r = 0; r < n; ++r) memcpy(Xsort + r * d, X + items[r].row * ld, sizeof(float) * (size_t)d);
    double *head = (double *)malloc(sizeof(double) * (size_t)n);
    double *tail = (double *)malloc(sizeof(double) * (size_t)n);
    oracle_cumulative_sse(Xsort, n, d, 0, head);
    oracle_cumulative_sse(Xsort, n, d, 1, tail);
    int64_t best = -1;
    double best_loss = 0.0;
    for (int64_t r = 0; r + 1 < n; ++r) {           /* split between sorted rows r and r + 1 */
        if (!(items[r].key < items[r + 1].key)) continue;
        const double loss = head[r] + tail[r + 1];
        if (best < 0 || loss < best_loss) { best = r; best_loss = loss; }
    }
    const float lo = items[best].key, hi = items[best + 1].key;
    float v = (float)(((double)lo + (double)hi) / 2.0);
    if (!(v > lo)) v = hi;
    *v_out = v;
    *loss_out = best_loss;
    free(head); free(tail); free(Xsort); free(items);
}

/* ------------------------------------------------------------------------
 * heuristic_select_idxs (Section 4.2): writes the n_cand = min(4, d) columns with the
 * largest loss summed over the level's buckets, largest first; returns n_cand.
 * bucket_rows / bucket_start: the rows of bucket i are
 * bucket_rows[bucket_start[i] .. bucket_start[i + 1]).
 * ---------------------------------------------------------------------- */
int32_t oracle_select_idxs(const float *X, int64_t ld, int32_t d, const int64_t *bucket_rows,
                           const int64_t *bucket_start, int32_t n_buckets, int32_t *cand)
{
    double *total = (double *)malloc(sizeof(double) * (size_t)d);
    for (int32_t j = 0; j < d; ++j) {
        total[j] = 0.0;
        for (int32_t i = 0; i < n_buckets; ++i)
            total[j] += oracle_bucket_loss(X, ld, bucket_rows + bucket_start[i], bucket_start[i + 1] - bucket_start[i], j);
    }
    const int32_t n_cand = d < ORACLE_CANDIDATES ? d : ORACLE_CANDIDATES;
    for (int32_t q = 0; q < n_cand; ++q) {
        int32_t pick = -1;
        for (int32_t j = 0; j < d; ++j) {
            int taken = 0;
            for (int32_t p = 0; p < q; ++p) taken |= cand[p] == j;
            if (!taken && (pick < 0 || total[j] > total[pick])) pick = j;
        }
        cand[q] = pick;
    }
    free(total);
    return n_cand;
}

/* ------------------------------------------------------------------------
 * Algorithm 2, applied four times: the tree of one codebook.
 * X N x d (row stride ld): the codebook's columns of the training matrix.
 * split_cols[t]  column (0..d-1) chosen at level t + 1
 * thresholds     16 floats in the order Algorithm 1 reads them (level t, node i at
 *                2^(t-1) - 1 + (i - 1); slot 15 = 0)
 * leaf[n]        leaf of training row n minus 1 (0..15)
 * level_loss[t]  l^min of level t + 1
 * ---------------------------------------------------------------------- */
void oracle_learn_tree(const float *X, int64_t N, int64_t ld, int32_t d, int32_t *split_cols,
                       float *thresholds, uint8_t *leaf, double *level_loss)
{
    int64_t *bucket_rows = (int64_t *)malloc(sizeof(int64_t) * (size_t)(N > 0 ? N : 1));
    int64_t *next_rows = (int64_t *)malloc(sizeof(int64_t) * (size_t)(N > 0 ? N : 1));
    int64_t start[ORACLE_K + 1], next_start[ORACLE_K + 1];
    for (int64_t n = 0; n < N; ++n) bucket_rows[n] = n;   /* B^0_1 holds every row */
    start[0] = 0; start[1] = N;
    for (int s = 0; s < ORACLE_K; ++s) thresholds[s] = 0.0f;
    for (int32_t t = 0; t < ORACLE_DEPTH; ++t) {
        const int32_t n_buckets = 1 << t;
        int32_t cand[ORACLE_CANDIDATES];
        const int32_t n_cand = oracle_select_idxs(X, ld, d, bucket_rows, start, n_buckets, cand);
        double l_min = INFINITY;
        int32_t j_min = cand[0];
        float v_min[ORACLE_K / 2], v[ORACLE_K / 2];
        int have = 0;
        for (int32_t q = 0; q < n_cand; ++q) {
            double l = 0.0;
            for (int32_t i = 0; i < n_buckets; ++i) {
                double l_i;
                oracle_optimal_split_threshold(X, ld, d, bucket_rows + start[i], start[i + 1] - start[i], cand[q],
                                               &v[i], &l_i);
                l += l_i;
            }
            if (!have || l < l_min) {
                have = 1;
                l_min = l; j_min = cand[q];
                memcpy(v_min, v, sizeof(v));
            }
        }
        split_cols[t] = j_min;
        level_loss[t] = l_min;
        for (int32_t i = 0; i < n_buckets; ++i) thresholds[n_buckets - 1 + i] = v_min[i];
        /* apply_split: below first, then above; both keep the row order */
        int64_t o = 0;
        for (int32_t i = 0; i < n_buckets; ++i) {
            next_start[2 * i] = o;
            for (int64_t r = start[i]; r < start[i + 1]; ++r)
                if (!(X[bucket_rows[r] * ld + j_min] >= v_min[i])) next_rows[o++] = bucket_rows[r];
            next_start[2 * i + 1] = o;
            for (int64_t r = start[i]; r < start[i + 1]; ++r)
                if (X[bucket_rows[r] * ld + j_min] >= v_min[i]) next_rows[o++] = bucket_rows[r];
        }
        next_start[2 * n_buckets] = o;
        memcpy(bucket_rows, next_rows, sizeof(int64_t) * (size_t)N);
        memcpy(start, next_start, sizeof(int64_t) * (size_t)(2 * n_buckets + 1));
    }
    for (int32_t i = 0; i < ORACLE_K; ++i)
        for (int64_t r = start[i]; r < start[i + 1]; ++r) leaf[bucket_rows[r]] = (uint8_t)i;
    free(bucket_rows);
    free(next_rows);
}

/* ------------------------------------------------------------------------
 * All C trees.  A N x D (row stride lda); codebook c owns the columns
 * [bounds[2c], bounds[2c+1]).  split_dims [C][4] are absolute columns of A,
 * thresholds [C][16], codes [N][C], level_loss [C][4].
 * ---------------------------------------------------------------------- */
void oracle_learn_trees(const float *A, int64_t N, int64_t lda, int32_t C, const int32_t *bounds,
                        int32_t *split_dims, float *thresholds, uint8_t *codes, double *level_loss)
{
    uint8_t *leaf = (uint8_t *)malloc((size_t)(N > 0 ? N : 1));
    for (int32_t c = 0; c < C; ++c) {
        const int32_t lo = bounds[2 * c], hi = bounds[2 * c + 1];
        int32_t cols[ORACLE_DEPTH];
        oracle_learn_tree(A + lo, N, lda, hi - lo, cols, thresholds + 16 * c, leaf, level_loss + 4 * c);
        for (int t = 0; t < ORACLE_DEPTH; ++t) split_dims[4 * c + t] = lo + cols[t];
        for (int64_t n = 0; n < N; ++n) codes[n * C + c] = leaf[n];
    }
    free(leaf);
}

/* ------------------------------------------------------------------------
 * G of Section 4.3: row n is the concatenation over the codebooks of the one-hot
 * encoding (n_protos wide) of codes[n][c] (0-based).  G is N x (C n_protos).
 * ---------------------------------------------------------------------- */
void oracle_one_hot(const uint8_t *codes, int64_t N, int32_t C, int32_t n_protos, double *G)
{
    memset(G, 0, sizeof(double) * (size_t)N * (size_t)C * (size_t)n_protos);
    for (int64_t n = 0; n < N; ++n)
        for (int32_t c = 0; c < C; ++c)
            G[n * C * n_protos + c * n_protos + codes[n * C + c]] = 1.0;
}

/* ------------------------------------------------------------------------
 * Prototypes as bucket means (Section 4; the variant the paper calls MADDNESS-PQ in
 * Section 5.1): P[c][k] holds, on the codebook's own columns, the mean of the
 * training rows with code k in codebook c, and 0 elsewhere; an empty bucket gives 0.
 * P is [C][16][D] in fp64.
 * ---------------------------------------------------------------------- */
void oracle_bucket_means(const uint8_t *codes, const float *A, int64_t N, int64_t lda, int32_t D, int32_t C,
                         const int32_t *bounds, double *P)
{
    memset(P, 0, sizeof(double) * (size_t)C * ORACLE_K * (size_t)D);
    for (int32_t c = 0; c < C; ++c)
        for (int32_t k = 0; k < ORACLE_K; ++k) {
            int64_t count = 0;
            for (int64_t n = 0; n < N; ++n) count += codes[n * C + c] == k;
            if (count == 0) continue;
            for (int32_t j = bounds[2 * c]; j < bounds[2 * c + 1]; ++j) {
                double sum = 0.0;
                for (int64_t n = 0; n < N; ++n)
                    if (codes[n * C + c] == k) sum += (double)A[n * lda + j];
                P[((size_t)c * ORACLE_K + k) * D + j] = sum / (double)count;
            }
        }
}

/* ------------------------------------------------------------------------
 * Section 4.3: P = (G^T G + lambda I)^-1 G^T A~, with G the one-hot matrix of the
 * training codes.  Cholesky factorisation of the (16 C) x (16 C) matrix, then a
 * forward and a backward substitution per column of A~.  P is [16 C][D] in fp64.
 * Returns 0, or -1 if the matrix is not positive definite (lambda <= 0 with an
 * empty bucket).
 * ---------------------------------------------------------------------- */
int32_t oracle_ridge_prototypes(const uint8_t *codes, const float *A, int64_t N, int64_t lda, int32_t D,
                                int32_t C, double lambda, double *P)
{
    const int64_t Q = (int64_t)C * ORACLE_K;
    double *S = (double *)calloc((size_t)(Q * Q), sizeof(double));   /* G^T G + lambda I, then its factor L */
    /* G^T G: (q, q') counts the rows whose one-hot row has ones in both places */
    for (int64_t n = 0; n < N; ++n)
        for (int32_t c = 0; c < C; ++c)
            for (int32_t c2 = 0; c2 < C; ++c2)
                S[(c * ORACLE_K + codes[n * C + c]) * Q + (c2 * ORACLE_K + codes[n * C + c2])] += 1.0;
    for (int64_t q = 0; q < Q; ++q) S[q * Q + q] += lambda;
    /* G^T A~: row q = sum of the training rows whose code in codebook q / 16 is q % 16 */
    memset(P, 0, sizeof(double) * (size_t)Q * (size_t)D);
    for (int64_t n = 0; n < N; ++n)
        for (int32_t c = 0; c < C; ++c) {
            double *dst = P + (size_t)(c * ORACLE_K + codes[n * C + c]) * D;
            for (int32_t j = 0; j < D; ++j) dst[j] += (double)A[n * lda + j];
        }
    /* Cholesky: S = L L^T, L kept in the lower triangle */
    for (int64_t j = 0; j < Q; ++j) {
        double diag = S[j * Q + j];
        for (int64_t k = 0; k < j; ++k) diag -= S[j * Q + k] * S[j * Q + k];
        if (!(diag > 0.0)) { free(S); return -1; }
        const double ljj = sqrt(diag);
        S[j * Q + j] = ljj;
        for (int64_t i = j + 1; i < Q; ++i) {
            double s = S[i * Q + j];
            for (int64_t k = 0; k < j; ++k) s -= S[i * Q + k] * S[j * Q + k];
            S[i * Q + j] = s / ljj;
        }
    }
    /* L y = G^T A~, then L^T P = y, for all columns of A~ side by side: y_i = (b_i - sum_{k<i} L_ik y_k) / L_ii
       with k ascending, then P_i = (y_i - sum_{k>i} L_ki P_k) / L_ii with k ascending */
    for (int64_t i = 0; i < Q; ++i) {
        for (int64_t k = 0; k < i; ++k)
            for (int32_t col = 0; col < D; ++col) P[i * D + col] -= S[i * Q + k] * P[k * D + col];
        for (int32_t col = 0; col < D; ++col) P[i * D + col] /= S[i * Q + i];
    }
    for (int64_t i = Q - 1; i >= 0; --i) {
        for (int64_t k = i + 1; k < Q; ++k)
            for (int32_t col = 0; col < D; ++col) P[i * D + col] -= S[k * Q + i] * P[k * D + col];
        for (int32_t col = 0; col < D; ++col) P[i * D + col] /= S[i * Q + i];
    }
    free(S);
    return 0;
}
