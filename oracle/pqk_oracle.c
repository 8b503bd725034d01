/*
 * pqk_oracle.c -- plain, slow, obviously-correct CPU definition of one
 * PQk-means iteration.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the checker, not the product.  Only the test-suite, the smoke
 * test and the benchmark's CPU-baseline leg may load it.  It shares no code,
 * header, table or helper with the HIP library and must never be called from
 * the product path.
 *
 * Every function is the paper's definition written out, with the
 * floating-point evaluation order fixed so that a second implementation can be
 * compared bit for bit:
 *   - tables:  Sec. 2.2 ("distance matrix among codewords", A^m_{i,j} is the
 *              squared distance between codewords i and j of subspace m)
 *   - SDC:     Eq. 3   (sum over m of A^m[x^m, y^m])
 *   - assign:  Eq. 5   (argmin over the K centers of the squared SD)
 *   - naive:   Eq. 6   (argmin over l of the summed table entries of members)
 *   - hist:    Eq. 7   (L-bin frequency histogram of a cluster's subcodes)
 *   - vote:    Eq. 8   (argmin over l of v = A^m h, zero bins skipped)
 *   - fit:     Alg. 1  (linear-scan branch: repeat { assign ; update })
 *   - encode:  Sec. 2.2 (per subvector, the index of the closest codeword)
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   indices are 0..255 instead of 1..L; ties in either argmin go to the
 *   lowest index; an empty cluster keeps its previous code; squared SD is
 *   used everywhere on the path; table entries are fp32, the SDC running sum
 *   is fp32 added in ascending m with no fused operation; the vote
 *   accumulates v in fp32 with one explicit fused multiply-add per non-zero
 *   bin in ascending bin order.  The encoder measures "closest" by the
 *   squared distance accumulated in fp32 over ascending dimension, one fp32
 *   subtraction and one fused multiply-add per dimension, and takes the
 *   lowest index on ties.
 *
 * Build: gcc -O2 -std=c99 -ffp-contract=off -fopenmp -shared -fPIC
 *        (no -ffast-math, no -march flags: arithmetic must be plain IEEE).
 * OpenMP is used only across independent outputs (codes n, centers k); it
 * never changes the order of any floating-point operation.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define PQKO_L 256 /* codewords per subspace; the paper fixes L = 256 (Sec. 2.2) */

/* Number of threads the parallel loops will use (1 without OpenMP). */
int pqko_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void pqko_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * Sec. 2.2: A^m[i][j] = || c^m_i - c^m_j ||^2.
 * codewords: [M][256][Ds] fp32; tables: [M][256][256] fp32.
 * Direct difference form, fp64 accumulation in ascending dimension, one
 * rounding to fp32.  This makes the diagonal exactly 0 and A bitwise
 * symmetric.
 */
void pqko_build_tables(const float *codewords, int M, int Ds, float *tables)
{
    for (int m = 0; m < M; ++m) {
        const float *cw = codewords + (size_t)m * PQKO_L * Ds;
        float *A = tables + (size_t)m * PQKO_L * PQKO_L;
        for (int i = 0; i < PQKO_L; ++i) {
            for (int j = 0; j < PQKO_L; ++j) {
                double acc = 0.0;
                for (int d = 0; d < Ds; ++d) {
                    double diff = (double)cw[(size_t)i * Ds + d] - (double)cw[(size_t)j * Ds + d];
                    double sq = diff * diff;
                    acc = acc + sq;
                }
                A[(size_t)i * PQKO_L + j] = (float)acc;
            }
        }
    }
}

/*
 * Sec. 2.2 (reconstructability): a PQ code decodes to the concatenation of
 * its codewords.  out: [N][M*Ds] fp64.  Used by the pins only.
 */
void pqko_decode(const float *codewords, int M, int Ds, const uint8_t *codes, int64_t N, double *out)
{
    for (int64_t n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            const float *c = codewords + ((size_t)m * PQKO_L + codes[n * M + m]) * Ds;
            for (int d = 0; d < Ds; ++d) out[((size_t)n * M + m) * Ds + d] = (double)c[d];
        }
}

/*
 * Sec. 2.2 (encoding): each of the M subvectors of a vector is replaced by the
 * index of its closest codeword.  vectors: [N][M*Ds] fp32, codes: [N][M] u8.
 * dist2 (may be NULL): [N][M] fp32, the squared distance to the chosen codeword.
 */
void pqko_encode(const float *vectors, int64_t N, int M, int Ds, const float *codewords, uint8_t *codes,
                 float *dist2)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            const float *x = vectors + ((size_t)n * M + m) * Ds;
            float best = INFINITY;
            int bl = 0;
            for (int l = 0; l < PQKO_L; ++l) {
                const float *c = codewords + ((size_t)m * PQKO_L + l) * Ds;
                float acc = 0.0f;
                for (int d = 0; d < Ds; ++d) {
                    float t = x[d] - c[d];
                    acc = fmaf(t, t, acc);
                }
                if (acc < best) {
                    best = acc;
                    bl = l;
                }
            }
            codes[n * M + m] = (uint8_t)bl;
            if (dist2) dist2[n * M + m] = best;
        }
}

/* Sec. 2.2 (reconstructability) in the codewords' own precision: out [N][M*Ds] fp32. */
void pqko_decode_f32(const float *codewords, int M, int Ds, const uint8_t *codes, int64_t N, float *out)
{
    for (int64_t n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            const float *c = codewords + ((size_t)m * PQKO_L + codes[n * M + m]) * Ds;
            for (int d = 0; d < Ds; ++d) out[((size_t)n * M + m) * Ds + d] = c[d];
        }
}

/* Eq. 3: squared symmetric distance of two codes, fp32, ascending m. */
static float sdc(const uint8_t *x, const uint8_t *y, int M, const float *tables)
{
    float s = tables[((size_t)0 * PQKO_L + x[0]) * PQKO_L + y[0]];
    for (int m = 1; m < M; ++m) {
        float a = tables[((size_t)m * PQKO_L + x[m]) * PQKO_L + y[m]];
        s = s + a;
    }
    return s;
}

/* Eq. 3 for a batch of code pairs (pins). */
void pqko_sdc_pairs(const uint8_t *x, const uint8_t *y, int64_t P, int M, const float *tables, float *out)
{
    for (int64_t p = 0; p < P; ++p) out[p] = sdc(x + p * M, y + p * M, M, tables);
}

/*
 * Eq. 5: a(n) = argmin_k d_SD(x_n, mu_k)^2 by linear scan, lowest k on ties.
 * tables are indexed [m][code subcode][center subcode].
 * dist may be NULL.
 */
void pqko_assign(const uint8_t *codes, int64_t N, int M, const uint8_t *centers, int K,
                 const float *tables, int32_t *assign, float *dist)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const uint8_t *x = codes + n * M;
        float best = INFINITY;
        int32_t bk = 0;
        for (int k = 0; k < K; ++k) {
            float s = sdc(x, centers + (size_t)k * M, M, tables);
            if (s < best) {
                best = s;
                bk = k;
            }
        }
        assign[n] = bk;
        if (dist) dist[n] = best;
    }
}

/*
 * Eq. 7: hist[k][m][j] = #{ n : a(n) = k and x_n^m = j }, counts[k] = N_k.
 * Serial on purpose (integer counts: any order gives the same result).
 */
void pqko_histogram(const uint8_t *codes, int64_t N, int M, const int32_t *assign, int K,
                    uint32_t *hist, uint32_t *counts)
{
    memset(hist, 0, (size_t)K * M * PQKO_L * sizeof(uint32_t));
    memset(counts, 0, (size_t)K * sizeof(uint32_t));
    for (int64_t n = 0; n < N; ++n) {
        int32_t k = assign[n];
        counts[k] += 1;
        for (int m = 0; m < M; ++m) hist[((size_t)k * M + m) * PQKO_L + codes[n * M + m]] += 1;
    }
}

/*
 * Eq. 8: mu_k^m <- argmin_l v_l with v = A^m h, where only the non-zero bins
 * of h are visited ("sparse voting").  v_l accumulates in fp32, one fused
 * multiply-add per non-zero bin j in ascending j; the lowest l wins ties.
 * A^m is read as [member subcode j][candidate l].
 * Clusters with counts[k] == 0 keep their code.
 */
void pqko_vote(const uint32_t *hist, const uint32_t *counts, int K, int M, const float *tables,
               uint8_t *centers)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int k = 0; k < K; ++k) {
        if (counts[k] == 0) continue;
        for (int m = 0; m < M; ++m) {
            const uint32_t *h = hist + ((size_t)k * M + m) * PQKO_L;
            const float *A = tables + (size_t)m * PQKO_L * PQKO_L;
            float vbest = INFINITY;
            int lbest = 0;
            for (int l = 0; l < PQKO_L; ++l) {
                float v = 0.0f;
                for (int j = 0; j < PQKO_L; ++j) {
                    if (h[j] != 0) v = fmaf((float)h[j], A[(size_t)j * PQKO_L + l], v);
                }
                if (v < vbest) {
                    vbest = v;
                    lbest = l;
                }
            }
            centers[(size_t)k * M + m] = (uint8_t)lbest;
        }
    }
}

/* Sparse-voting update: Eq. 7 then Eq. 8.  hist [K][M][256], counts [K] are outputs. */
void pqko_update(const uint8_t *codes, int64_t N, int M, const int32_t *assign, int K,
                 const float *tables, uint8_t *centers, uint32_t *hist, uint32_t *counts)
{
    pqko_histogram(codes, N, M, assign, K, hist, counts);
    pqko_vote(hist, counts, K, M, tables, centers);
}

/*
 * Eq. 6, the naive update: for every cluster and subspace test all L
 * candidates against all members.  Sums in fp64 (this is the mathematical
 * reference for the vote, not a bit-level one); lowest l on ties; empty
 * clusters keep their code.  cost_out (may be NULL): [K][M][256] fp64 sums.
 */
void pqko_update_naive(const uint8_t *codes, int64_t N, int M, const int32_t *assign, int K,
                       const float *tables, uint8_t *centers, double *cost_out)
{
    double *cost = (double *)calloc((size_t)K * M * PQKO_L, sizeof(double));
    uint32_t *cnt = (uint32_t *)calloc((size_t)K, sizeof(uint32_t));
    for (int64_t n = 0; n < N; ++n) {
        int32_t k = assign[n];
        cnt[k] += 1;
        for (int m = 0; m < M; ++m) {
            const float *row = tables + ((size_t)m * PQKO_L + codes[n * M + m]) * PQKO_L;
            double *c = cost + ((size_t)k * M + m) * PQKO_L;
            for (int l = 0; l < PQKO_L; ++l) c[l] += (double)row[l];
        }
    }
    for (int k = 0; k < K; ++k) {
        if (cnt[k] == 0) continue;
        for (int m = 0; m < M; ++m) {
            const double *c = cost + ((size_t)k * M + m) * PQKO_L;
            int lbest = 0;
            for (int l = 1; l < PQKO_L; ++l)
                if (c[l] < c[lbest]) lbest = l;
            centers[(size_t)k * M + m] = (uint8_t)lbest;
        }
    }
    if (cost_out) memcpy(cost_out, cost, (size_t)K * M * PQKO_L * sizeof(double));
    free(cost);
    free(cnt);
}

/* Sum over n of the squared SD to the assigned center, fp64 (Eq. 4 with squared SD). */
double pqko_objective(const uint8_t *codes, int64_t N, int M, const uint8_t *centers,
                      const int32_t *assign, const float *tables)
{
    double e = 0.0;
    for (int64_t n = 0; n < N; ++n)
        e += (double)sdc(codes + n * M, centers + (size_t)assign[n] * M, M, tables);
    return e;
}

/*
 * Alg. 1, linear-scan branch, fixed iteration count.
 * centers: in = initial centers (Init() is the caller's), out = centers after
 * the last update.  assign: result of the last assignment step (taken against
 * the centers before the last update).  hist/counts: those of the last update.
 */
void pqko_fit(const uint8_t *codes, int64_t N, int M, const float *tables, int K, uint8_t *centers,
              int iters, int32_t *assign, uint32_t *hist, uint32_t *counts)
{
    for (int it = 0; it < iters; ++it) {
        pqko_assign(codes, N, M, centers, K, tables, assign, NULL);
        pqko_update(codes, N, M, assign, K, tables, centers, hist, counts);
    }
}

/*
 * Alg. 1 with a stop condition ("any condition can be adopted", Sec. 3.3): stop after the iteration in
 * which the assignment step changed no assignment (the fixed point of the loop), or after max_iters.
 * Per iteration it, four statistics are recorded (layout [max_iters][4] doubles):
 *   0: objective  = sum over n of the squared SD of the assignment step (fp64 sum of the fp32 minima,
 *                   ascending n) -- Eq. 4 with the squared distance
 *   1: changed    = #{ n : a_it(n) != a_{it-1}(n) }, with a_{-1}(n) = -1 (so iteration 0 reports N)
 *   2: nonzero    = number of non-zero histogram bins over all (k, m) (the ||h||_0 of Tab. 3, summed)
 *   3: nonempty   = number of clusters with at least one member
 * Returns the number of iterations done.  centers / assign / hist / counts as in pqko_fit.
 */
int pqko_fit_until(const uint8_t *codes, int64_t N, int M, const float *tables, int K, uint8_t *centers,
                   int max_iters, int32_t *assign, uint32_t *hist, uint32_t *counts, double *stats)
{
    int32_t *prev = (int32_t *)malloc((size_t)(N > 0 ? N : 1) * sizeof(int32_t));
    float *dist = (float *)malloc((size_t)(N > 0 ? N : 1) * sizeof(float));
    for (int64_t n = 0; n < N; ++n) prev[n] = -1;
    int it = 0;
    while (it < max_iters) {
        pqko_assign(codes, N, M, centers, K, tables, assign, dist);
        double obj = 0.0;
        int64_t changed = 0;
        for (int64_t n = 0; n < N; ++n) {
            obj += (double)dist[n];
            if (assign[n] != prev[n]) changed += 1;
            prev[n] = assign[n];
        }
        pqko_update(codes, N, M, assign, K, tables, centers, hist, counts);
        int64_t nz = 0, ne = 0;
        for (size_t i = 0; i < (size_t)K * M * PQKO_L; ++i) nz += hist[i] != 0;
        for (int k = 0; k < K; ++k) ne += counts[k] != 0;
        stats[4 * it + 0] = obj;
        stats[4 * it + 1] = (double)changed;
        stats[4 * it + 2] = (double)nz;
        stats[4 * it + 3] = (double)ne;
        ++it;
        if (changed == 0) break;
    }
    free(prev);
    free(dist);
    return it;
}
