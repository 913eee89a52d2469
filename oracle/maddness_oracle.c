/*
 * CPU oracle for the MADDNESS inference path ("Multiplying Matrices Without
 * Multiplying", arXiv 2106.10860).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded statement
 * of what the path computes, written from the paper so that a reader can check
 * it by eye.  Only the test-suite, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the product (the HIP library) shares no code
 * with it and never routes through it.  No blocking, no SIMD, no reordering.
 *
 * All pointers are HOST pointers.  Fixed by the paper: K = 16 prototypes per
 * codebook, trees of depth 4 (Section 4.1), 8-bit table entries (Section 3,
 * "Table Construction"; Appendix A).
 *
 * Parity pins (tests/test_oracle_pins.py): every function below is pinned to
 * something other than itself - closed forms, library routines, brute force,
 * the paper's worked example for the one-hot matrix G, and the half-level
 * quantisation error bound from the proof of Lemma F.5.  The approximation
 * quality itself (NMSE of the method on some matrix) is "parity unpinned": the
 * paper prints no such value.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>

#define ORACLE_K 16
#define ORACLE_DEPTH 4

/* ------------------------------------------------------------------------
 * Algorithm 1 (MaddnessHash), Section 4.1.
 *
 * x           one row of A (D floats)
 * j[t-1]      split index of level t = 1..4 (absolute column of A)
 * v           the 15 thresholds of this tree.  The paper gives four arrays
 *             v^1..v^4 with len(v^t) = 2^(t-1); they are stored one after the
 *             other: v^t_i (i = 1..2^(t-1)) sits at slot 2^(t-1) - 1 + (i - 1).
 *             Slot 15 is padding.
 * returns     the leaf index i in 1..16 exactly as the algorithm does.
 *
 * Comparison: b = (x_j >= v).  A NaN on either side compares false -> left.
 * ---------------------------------------------------------------------- */
int oracle_hash_row(const float *x, const int32_t *j, const float *v)
{
    int i = 1;                                   /* node index within level */
    for (int t = 1; t <= ORACLE_DEPTH; ++t) {
        int first_slot_of_level = (1 << (t - 1)) - 1;
        float thr = v[first_slot_of_level + (i - 1)];   /* v^t_i */
        int b = (x[j[t - 1]] >= thr) ? 1 : 0;
        i = 2 * i - 1 + b;                       /* left or right child */
    }
    return i;
}

/* g(A): Algorithm 1 on every row for each of the C codebooks (Section 3,
 * "Encoding Function"; Section 4.1).  codes[n*C + c] = leaf - 1, in 0..15
 * (the leaf is one of 16, so it fits the 4 bits Appendix B speaks of). */
void oracle_encode(const float *A, int64_t N, int64_t lda,
                   int32_t C, const int32_t *split_dims /*[C][4]*/,
                   const float *thresholds /*[C][16]*/,
                   uint8_t *codes /*[N][C]*/)
{
    for (int64_t n = 0; n < N; ++n)
        for (int32_t c = 0; c < C; ++c) {
            int leaf = oracle_hash_row(A + n * lda, split_dims + 4 * c,
                                       thresholds + 16 * c);
            codes[n * C + c] = (uint8_t)(leaf - 1);
        }
}

/* ------------------------------------------------------------------------
 * Inputs that are not fp32, and inputs stored by columns.
 *
 * The tree walk only compares one element of the row with a threshold, so it
 * applies to narrower data as it is (Appendix E.6: 8-bit image data are used
 * directly), and it touches four columns per codebook, which is cheapest when
 * the matrix is stored by columns (Section 4.1; Section 5.2: the cost per row
 * is O(C), not O(D)).  The definition used here: every element is widened to
 * the fp32 number of the same value - exact for IEEE binary16, for bfloat16 (the
 * upper half of an fp32) and for unsigned bytes - and Algorithm 1 then runs on
 * those values with the fp32 thresholds.
 *
 * dtype: 0 fp32, 1 binary16, 2 bfloat16, 3 uint8.
 * --------------------------------------------------------------------- */
static float widen_f16(uint16_t h)
{
    const int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
    float mag;
    if (e == 0)
        mag = ldexpf((float)m, -24);                 /* zero and subnormals: m 2^-24 */
    else if (e == 31)
        mag = m ? NAN : INFINITY;
    else
        mag = ldexpf((float)(1024 + m), e - 25);     /* (1 + m / 1024) 2^(e - 15) */
    return sign ? -mag : mag;
}

static float widen_bf16(uint16_t b)
{
    const uint32_t u = (uint32_t)b << 16;            /* the 16 dropped mantissa bits are zero */
    float f;
    memcpy(&f, &u, 4);
    return f;
}

int oracle_widen(const void *src, int32_t dtype, int64_t count, float *dst)
{
    for (int64_t i = 0; i < count; ++i) {
        switch (dtype) {
        case 0: dst[i] = ((const float *)src)[i]; break;
        case 1: dst[i] = widen_f16(((const uint16_t *)src)[i]); break;
        case 2: dst[i] = widen_bf16(((const uint16_t *)src)[i]); break;
        case 3: dst[i] = (float)((const uint8_t *)src)[i]; break;
        default: return -1;
        }
    }
    return 0;
}

/* g(A) for an input of any of the four types, stored by rows (col_major = 0:
 * element (n, d) at index n * lda + d) or by columns (col_major = 1: at index
 * d * lda + n).  One row at a time: gather the row, widen it, walk the trees. */
int oracle_encode_typed(const void *A, int32_t dtype, int32_t col_major, int64_t N, int32_t D,
                        int64_t lda, int32_t C, const int32_t *split_dims, const float *thresholds,
                        uint8_t *codes /*[N][C]*/, float *row /* scratch, D floats */)
{
    static const int size_of[4] = {4, 2, 2, 1};
    if (dtype < 0 || dtype > 3) return -1;
    const unsigned char *base = (const unsigned char *)A;
    for (int64_t n = 0; n < N; ++n) {
        for (int32_t d = 0; d < D; ++d) {
            const int64_t idx = col_major ? (int64_t)d * lda + n : n * lda + d;
            oracle_widen(base + idx * size_of[dtype], dtype, 1, &row[d]);
        }
        for (int32_t c = 0; c < C; ++c)
            codes[n * C + c] = (uint8_t)(oracle_hash_row(row, split_dims + 4 * c, thresholds + 16 * c) - 1);
    }
    return 0;
}

/* Two 4-bit codes per byte (C log2 K bits per row, Section 3): byte b of a row
 * holds codebook 2b in its low nibble and codebook 2b+1 in its high nibble; an
 * odd C leaves the last high nibble zero. */
void oracle_pack(const uint8_t *codes /*[N][C]*/, int64_t N, int32_t C,
                 uint8_t *packed /*[N][(C+1)/2]*/)
{
    int32_t Cb = (C + 1) / 2;
    for (int64_t n = 0; n < N; ++n)
        for (int32_t b = 0; b < Cb; ++b) {
            unsigned lo = codes[n * C + 2 * b];
            unsigned hi = (2 * b + 1 < C) ? codes[n * C + 2 * b + 1] : 0u;
            packed[n * Cb + b] = (uint8_t)(lo | (hi << 4));
        }
}

static unsigned code_of(const uint8_t *packed_row, int32_t c)
{
    unsigned byte = packed_row[c / 2];
    return (c & 1) ? (byte >> 4) : (byte & 15u);
}

/* h(B) before quantisation (Section 3, "Table Construction", with the dense
 * prototype matrix of Section 4.3): T[c][k][m] = sum_d P[c][k][d] * B[d][m],
 * summed in fp64 in index order. */
void oracle_build_luts_f64(const float *P /*[C][16][D]*/, const float *B /*[D][ldb]*/,
                           int32_t D, int32_t M, int64_t ldb, int32_t C,
                           double *T /*[C][16][M]*/)
{
    for (int32_t c = 0; c < C; ++c)
        for (int k = 0; k < ORACLE_K; ++k)
            for (int32_t m = 0; m < M; ++m) {
                double s = 0.0;
                const float *p = P + ((size_t)c * ORACLE_K + k) * D;
                for (int32_t d = 0; d < D; ++d)
                    s += (double)p[d] * (double)B[(size_t)d * ldb + m];
                T[((size_t)c * ORACLE_K + k) * M + m] = s;
            }
}

/* Largest integer l with r * 2^l <= 255 (Appendix A: alpha^-1 = 2^l with
 * l = floor(log2(255 / range))), found exactly: scaling by a power of two is
 * exact in binary floating point.  Kept inside fp32's normal exponent range so
 * that 2^-l is an fp32 number.  r must be finite and > 0. */
static int scale_exponent(double r)
{
    int l = (int)floor(log2(255.0 / r));
    while (ldexp(r, l + 1) <= 255.0) ++l;
    while (ldexp(r, l) > 255.0) --l;
    if (l > 126) l = 126;
    if (l < -126) l = -126;
    return l;
}

/* 8-bit quantisation of the tables (Section 3: subtract each table's minimum,
 * rescale so that the largest entry of any table is at most 255; Appendix A:
 * power-of-two scale shared by all codebooks, offsets delta_c, beta = sum_c
 * delta_c).  Done independently for every output column m:
 *   delta[c][m] = min_k T[c][k][m]
 *   r[m]        = max_{c,k} (T[c][k][m] - delta[c][m])
 *   l[m]        = largest integer with r 2^l <= 255   (0 if r is 0 or not finite)
 *   q           = clamp(round_half_even((T - delta) 2^l), 0, 255)
 *   scale[m]    = 2^-l,   offset[m] = (float) sum_c delta[c][m]
 * l_out and delta_out may be NULL. */
void oracle_quantize_luts(const double *T /*[C][16][M]*/, int32_t C, int32_t M,
                          uint8_t *luts /*[C][16][M]*/, float *scale /*[M]*/,
                          float *offset /*[M]*/, int32_t *l_out /*[M]*/,
                          double *delta_out /*[C][M]*/)
{
    for (int32_t m = 0; m < M; ++m) {
        double r = 0.0, beta = 0.0;
        for (int32_t c = 0; c < C; ++c) {
            const double *t = T + (size_t)c * ORACLE_K * M + m;
            double dmin = t[0];
            for (int k = 1; k < ORACLE_K; ++k)
                if (t[(size_t)k * M] < dmin) dmin = t[(size_t)k * M];
            for (int k = 0; k < ORACLE_K; ++k) {
                double e = t[(size_t)k * M] - dmin;
                if (e > r) r = e;
            }
            beta += dmin;
            if (delta_out) delta_out[(size_t)c * M + m] = dmin;
        }
        int l = (r > 0.0 && isfinite(r)) ? scale_exponent(r) : 0;
        for (int32_t c = 0; c < C; ++c) {
            const double *t = T + (size_t)c * ORACLE_K * M + m;
            double dmin = t[0];
            for (int k = 1; k < ORACLE_K; ++k)
                if (t[(size_t)k * M] < dmin) dmin = t[(size_t)k * M];
            for (int k = 0; k < ORACLE_K; ++k) {
                double q = nearbyint(ldexp(t[(size_t)k * M] - dmin, l)); /* ties to even */
                if (!(q >= 0.0)) q = 0.0;       /* also catches NaN */
                if (q > 255.0) q = 255.0;
                luts[((size_t)c * ORACLE_K + k) * M + m] = (uint8_t)q;
            }
        }
        scale[m] = ldexpf(1.0f, -l);
        offset[m] = (float)beta;
        if (l_out) l_out[m] = l;
    }
}

/* The quantisation of Appendix A as printed, pooled over the output columns:
 * one offset per codebook and one scale for everything,
 *   delta[c] = min_{m,k} T[c][k][m]
 *   r        = max_{c,m,k} (T[c][k][m] - delta[c])
 *   l        = largest integer with r 2^l <= 255   (0 if r is 0 or not finite)
 *   q        = clamp(round_half_even((T - delta[c]) 2^l), 0, 255)
 *   alpha = 2^-l, beta = sum_c delta[c]; written to scale[m], offset[m] for every
 *   m so that the scan consumes both variants in the same way.
 * (The printed l = max_c floor(log2(255 / range_c)) is read as "from the widest
 * table", as in oracle_quantize_luts.)  l_out: one int; delta_out: [C]. */
void oracle_quantize_luts_pooled(const double *T /*[C][16][M]*/, int32_t C, int32_t M,
                                 uint8_t *luts, float *scale, float *offset,
                                 int32_t *l_out, double *delta_out /*[C]*/)
{
    double r = 0.0, beta = 0.0;
    for (int32_t c = 0; c < C; ++c) {
        const double *t = T + (size_t)c * ORACLE_K * M;
        double dmin = t[0];
        for (size_t i = 1; i < (size_t)ORACLE_K * M; ++i)
            if (t[i] < dmin) dmin = t[i];
        for (size_t i = 0; i < (size_t)ORACLE_K * M; ++i) {
            double e = t[i] - dmin;
            if (e > r) r = e;
        }
        beta += dmin;
        if (delta_out) delta_out[c] = dmin;
    }
    int l = (r > 0.0 && isfinite(r)) ? scale_exponent(r) : 0;
    for (int32_t c = 0; c < C; ++c) {
        const double *t = T + (size_t)c * ORACLE_K * M;
        double dmin = t[0];
        for (size_t i = 1; i < (size_t)ORACLE_K * M; ++i)
            if (t[i] < dmin) dmin = t[i];
        for (size_t i = 0; i < (size_t)ORACLE_K * M; ++i) {
            double q = nearbyint(ldexp(t[i] - dmin, l));
            if (!(q >= 0.0)) q = 0.0;
            if (q > 255.0) q = 255.0;
            luts[(size_t)c * ORACLE_K * M + i] = (uint8_t)q;
        }
    }
    for (int32_t m = 0; m < M; ++m) {
        scale[m] = ldexpf(1.0f, -l);
        offset[m] = (float)beta;
    }
    if (l_out) *l_out = l;
}

/* f(g(A), h(B)) of Section 4.4 as an exact integer sum, then alpha f + beta
 * (the objective of Section 1.1):
 *   acc[n][m] = sum_c luts[c][code(n,c)][m]
 *   out[n][m] = fma((float)acc, scale[m], offset[m])
 * acc32 / acc16 / out may be NULL.  Returns the number of accumulators that do
 * not fit 16 bits (0 whenever 255 C <= 65535). */
int64_t oracle_scan(const uint8_t *packed /*[N][(C+1)/2]*/, int64_t N, int32_t C,
                    int32_t M, const uint8_t *luts /*[C][16][M]*/,
                    const float *scale, const float *offset,
                    float *out, int64_t ldo, uint32_t *acc32 /*[N][M]*/,
                    uint16_t *acc16 /*[N][M]*/)
{
    int32_t Cb = (C + 1) / 2;
    int64_t overflow = 0;
    for (int64_t n = 0; n < N; ++n)
        for (int32_t m = 0; m < M; ++m) {
            uint32_t acc = 0;
            for (int32_t c = 0; c < C; ++c) {
                unsigned k = code_of(packed + n * Cb, c);
                acc += luts[((size_t)c * ORACLE_K + k) * M + m];
            }
            if (acc > 65535u) ++overflow;
            if (acc32) acc32[n * M + m] = acc;
            if (acc16) acc16[n * M + m] = (uint16_t)acc;
            if (out) out[n * ldo + m] = fmaf((float)acc, scale[m], offset[m]);
        }
    return overflow;
}

/* Averaging Integer Sum Estimator (Appendix D, Definition D.1): the mean of a
 * block of values estimated by averaging pairs, then pairs of pairs, ...; every
 * average is floor((left + right + 1) / 2), left and right being the estimates of
 * the first and second half of the block. */
static unsigned aise_block(const uint8_t *x, int n)
{
    if (n == 1) return x[0];
    return (aise_block(x, n / 2) + aise_block(x + n / 2, n / 2) + 1u) / 2u;
}

/* f by pairwise averages (Section 4.4, second half; Appendix D) instead of the
 * exact sum: the C looked-up entries of an output are taken in blocks of U
 * consecutive codebooks (U a power of two dividing C), each block is reduced to
 * its AISE average, the averages are summed exactly and multiplied by U; the
 * expected excess C log2(U) / 4 of that estimate (Theorem D.1; every averaging
 * step rounds up) is subtracted, and alpha, beta are applied:
 *   est[n][m] = U sum_blocks aise(block) - C log2(U) / 4
 *   out[n][m] = fma(est, scale[m], offset[m])
 * usum (may be NULL) receives U sum_blocks aise(block).  Returns -1 if U does not
 * divide C or is not a power of two. */
int oracle_scan_averaged(const uint8_t *packed, int64_t N, int32_t C, int32_t M,
                         const uint8_t *luts, const float *scale, const float *offset,
                         int32_t U, float *out, int64_t ldo, uint16_t *usum /*[N][M]*/)
{
    int p = 0;
    while ((1 << p) < U) ++p;
    if (U < 1 || (1 << p) != U || C % U != 0 || U > 256) return -1;
    int32_t Cb = (C + 1) / 2;
    float debias = (float)(C * p) / 4.0f;       /* a multiple of 0.25: exact */
    uint8_t x[256];
    for (int64_t n = 0; n < N; ++n)
        for (int32_t m = 0; m < M; ++m) {
            uint32_t s = 0;
            for (int32_t c0 = 0; c0 < C; c0 += U) {
                for (int32_t u = 0; u < U; ++u) {
                    unsigned k = code_of(packed + n * Cb, c0 + u);
                    x[u] = luts[((size_t)(c0 + u) * ORACLE_K + k) * M + m];
                }
                s += aise_block(x, U);
            }
            s *= (uint32_t)U;
            if (usum) usum[n * M + m] = (uint16_t)s;
            if (out) out[n * ldo + m] = fmaf((float)s - debias, scale[m], offset[m]);
        }
    return 0;
}

/* Same sum with unquantised tables, in fp64: sum_c T[c][code(n,c)][m].  With
 * exact tables this equals (row of G) P B, the product of the reconstructed
 * row with B (proof of Lemma F.5). */
void oracle_scan_f64(const uint8_t *packed, int64_t N, int32_t C, int32_t M,
                     const double *T /*[C][16][M]*/, double *out /*[N][M]*/)
{
    int32_t Cb = (C + 1) / 2;
    for (int64_t n = 0; n < N; ++n)
        for (int32_t m = 0; m < M; ++m) {
            double s = 0.0;
            for (int32_t c = 0; c < C; ++c) {
                unsigned k = code_of(packed + n * Cb, c);
                s += T[((size_t)c * ORACLE_K + k) * M + m];
            }
            out[n * M + m] = s;
        }
}

/* The whole inference path on one batch of rows: g, then f, then alpha f + beta.
 * codes_scratch holds N*C bytes, packed holds N*((C+1)/2) bytes (both written). */
int64_t oracle_encode_scan(const float *A, int64_t N, int64_t lda, int32_t C,
                           const int32_t *split_dims, const float *thresholds,
                           int32_t M, const uint8_t *luts, const float *scale,
                           const float *offset, float *out, int64_t ldo,
                           uint16_t *acc16, uint8_t *codes_scratch, uint8_t *packed)
{
    oracle_encode(A, N, lda, C, split_dims, thresholds, codes_scratch);
    oracle_pack(codes_scratch, N, C, packed);
    return oracle_scan(packed, N, C, M, luts, scale, offset, out, ldo, NULL, acc16);
}

/* Exact product in fp64 and the error measure of Section 5.5:
 * NMSE = ||Yhat - Y||_F^2 / ||Y||_F^2. */
void oracle_matmul_f64(const float *A, int64_t N, int64_t lda, const float *B,
                       int32_t D, int32_t M, int64_t ldb, double *Y /*[N][M]*/)
{
    for (int64_t n = 0; n < N; ++n)
        for (int32_t m = 0; m < M; ++m) {
            double s = 0.0;
            for (int32_t d = 0; d < D; ++d)
                s += (double)A[n * lda + d] * (double)B[(size_t)d * ldb + m];
            Y[n * M + m] = s;
        }
}

double oracle_nmse(const float *Yhat, int64_t ldo, const double *Y, int64_t N, int32_t M)
{
    double num = 0.0, den = 0.0;
    for (int64_t n = 0; n < N; ++n)
        for (int32_t m = 0; m < M; ++m) {
            double e = (double)Yhat[n * ldo + m] - Y[n * M + m];
            num += e * e;
            den += Y[n * M + m] * Y[n * M + m];
        }
    return num / den;
}
