/*
 * pqkm.h -- C ABI of the PQk-means iteration for AMD MI355X (gfx950).
 *
 * One PQk-means iteration (Alg. 1, linear-scan branch) is an assignment step
 * (Eq. 5: every PQ code takes the nearest of K PQ-coded centers by squared
 * symmetric distance, Eq. 3) followed by the sparse-voting update (Eq. 7-8:
 * per center and subspace, a 256-bin histogram of the members' subcodes and
 * the subcodeword minimising the count-weighted table sum).
 *
 * Conventions common to every entry point
 *   - Unless a parameter says "host", every pointer is a DEVICE pointer to
 *     memory owned by the caller (e.g. torch.Tensor.data_ptr()) on the device
 *     that is current when the call is made.  Arrays are dense, row-major,
 *     unpadded.  The library keeps no pointer after the work it enqueued ends.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on `stream` and return; they never synchronise
 *     and allocate or free nothing.  Results are valid once `stream` reaches
 *     the end of the enqueued work.  (pqkm_fit_until is the exception: it
 *     reads a few counters back per iteration and waits for them.)  The
 *     enqueued work is kernels only -- no memset or copy nodes -- so a caller
 *     may capture pqkm_build_tables, pqkm_encode, pqkm_decode, pqkm_assign,
 *     pqkm_update, pqkm_update_naive and pqkm_fit in a HIP graph (with the
 *     "profile" option of pqkm_tuning.h off) and replay it; the workspace need not keep its
 *     contents between replays.
 *   - `workspace` is device scratch of at least
 *     pqkm_workspace_bytes(N, M, K) bytes, 256-byte aligned, used only during
 *     the call's enqueued work (tile images of the centers, for M = 4 a
 *     regrouped copy of the codes of one scan launch, histograms).  Two calls that overlap in time on different
 *     streams need different workspaces.
 *   - Subcode/center indices are 0..255 (the paper's 1..L with L = 256,
 *     Sec. 2.2).  `codes` must be 4-byte aligned when M is a multiple of 4.
 *   - Arguments are validated on the host before anything is launched; on an
 *     error nothing has been enqueued and outputs are untouched.
 *   - Floating point: table entries are fp32; the symmetric distance is an
 *     fp32 running sum over m = 0..M-1 in ascending order, one IEEE add each;
 *     the vote accumulates in fp32 with one fused multiply-add per non-zero
 *     bin in ascending bin order.  Ties in either argmin go to the lowest
 *     index.  With these rules the result is unique, so a second
 *     implementation can be compared bit for bit.
 */
#ifndef PQKM_H
#define PQKM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PQKM_OK = 0,
    PQKM_ERR_NULL = 1,      /* a required pointer is NULL                                  */
    PQKM_ERR_SHAPE = 2,     /* N < 0, K < 1, M < 1 or M > 64, Ds < 1, iters < 0, bad align */
    PQKM_ERR_WORKSPACE = 3, /* workspace NULL / misaligned / smaller than required         */
    PQKM_ERR_DEVICE = 4,    /* not a gfx950 device, or a HIP call failed                   */
    PQKM_ERR_TOO_LARGE = 5  /* pqkm_assign_noalloc: the problem exceeds its static scratch */
} pqkm_status;

/* Static, NUL-terminated description of a status code. */
const char *pqkm_status_string(pqkm_status status);

/*
 * Bytes of device scratch that pqkm_assign / pqkm_update / pqkm_fit need for
 * a problem of N codes, M subspaces, K centers.  Pure host arithmetic (no HIP
 * call).  Returns 0 for invalid shapes.
 */
size_t pqkm_workspace_bytes(int64_t N, int32_t M, int32_t K);

/*
 * Distance matrices among codewords (Sec. 2.2):
 *   tables[m][i][j] = || codewords[m][i][:] - codewords[m][j][:] ||^2
 * accumulated in fp64 over ascending dimension in the direct-difference form
 * and rounded once to fp32, so the diagonal is exactly 0 and each matrix is
 * bitwise symmetric.
 *   codewords  [M][256][Ds] fp32, in
 *   tables     [M][256][256] fp32, out
 */
pqkm_status pqkm_build_tables(const float *codewords, int32_t M, int32_t Ds, float *tables,
                              void *stream);

/*
 * Product-quantisation encoding (Sec. 2.2): every one of the M subvectors (Ds consecutive
 * components) of a vector is replaced by the index of its closest codeword,
 *   codes[n][m] = argmin_l  sum_{d} (vectors[n][m*Ds + d] - codewords[m][l][d])^2,
 * lowest l on ties.  The sum is accumulated in fp32 over ascending d with one fp32 subtraction
 * and one fused multiply-add per component, which makes the result unique.
 *   vectors    [N][M*Ds] fp32, in       codewords [M][256][Ds] fp32, in
 *   codes      [N][M] u8, out
 * This is the preprocessing step in front of the clustering; N = 0 is legal.
 *
 * pqkm_decode is the reconstruction of Sec. 2.2: vectors[n][m*Ds + d] = codewords[m][codes[n][m]][d].
 *   codes      [N][M] u8, in            vectors   [N][M*Ds] fp32, out
 */
pqkm_status pqkm_encode(const float *vectors, int64_t N, int32_t M, int32_t Ds, const float *codewords,
                        uint8_t *codes, void *stream);
pqkm_status pqkm_decode(const uint8_t *codes, int64_t N, int32_t M, int32_t Ds, const float *codewords,
                        float *vectors, void *stream);

/*
 * Assignment step (Eq. 5 with the squared symmetric distance of Eq. 3):
 *   assign[n] = argmin_k  sum_{m} tables[m][codes[n][m]][centers[k][m]]
 * lowest k on ties.
 *   codes    [N][M] u8, in          centers [K][M] u8, in
 *   tables   [M][256][256] fp32, in (row = the code's subcode, column = the center's)
 *   assign   [N] i32, out           dist    [N] fp32, out, may be NULL (the minimum itself)
 * N = 0 is legal and does nothing.
 */
pqkm_status pqkm_assign(const uint8_t *codes, int64_t N, int32_t M, const uint8_t *centers,
                        int32_t K, const float *tables, int32_t *assign, float *dist,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * pqkm_assign for callers that can neither allocate device memory nor hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same
 * results as pqkm_assign, but the scratch is a static device array inside the library
 * (PQKM_NOALLOC_SCRATCH_BYTES per GPU, held from library load until the process ends), so the call allocates
 * and frees nothing and takes no workspace argument.
 *   - Limit: pqkm_workspace_bytes(N, M, K) <= PQKM_NOALLOC_SCRATCH_BYTES, else PQKM_ERR_TOO_LARGE and
 *     nothing is launched (64 MiB cover e.g. N = 1e6 four-byte codes against K = 1000 centers).
 *   - Every call on a GPU shares that GPU's array: two calls that overlap in time on one GPU (different
 *     streams, or threads) race and give undefined results.  Calls in stream order are fine; nothing needs
 *     clearing between them (the kernels initialise what they read).
 *   - The "profile" option of pqkm_tuning.h is ignored here (its events are created on demand).
 */
#define PQKM_NOALLOC_SCRATCH_BYTES (64u * 1024u * 1024u)
pqkm_status pqkm_assign_noalloc(const uint8_t *codes, int64_t N, int32_t M, const uint8_t *centers,
                                int32_t K, const float *tables, int32_t *assign, float *dist,
                                void *stream);

/*
 * Assignment step through an exact index over the centers (Sec. 3.1: Alg. 1's BuildTable + FindNN with
 * the table, the branch the paper takes for very many centers).  Same definition and same result as
 * pqkm_assign, bit for bit, ties included: the centers are filed in 65536 buckets by their first two
 * subcodes, and every code walks the buckets in ascending partial distance, stopping a walk once a lower
 * bound of all that is left (the partial sum continued with the row minima of the remaining subspaces, in
 * the order of Eq. 3) exceeds the best distance found.  The bounds are exact in fp32 for any table entries
 * (fp32 addition is monotone); NaN entries only make the walk longer.  How much is pruned depends on the
 * data: on codes whose nearest center is close the walk is short, on codes far from every center it visits
 * most buckets and is far slower than the scan.  pqkm_check measures which of the two is faster.
 *   workspace: at least pqkm_index_workspace_bytes(M, K) bytes; M >= 2.
 */
size_t pqkm_index_workspace_bytes(int32_t M, int32_t K);
pqkm_status pqkm_assign_indexed(const uint8_t *codes, int64_t N, int32_t M, const uint8_t *centers,
                                int32_t K, const float *tables, int32_t *assign, float *dist,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * Check() of Alg. 1 (Sec. 3.1): runs the linear scan and the indexed search on a sample of the codes,
 * `trials` times each after one warm-up run, and reports the faster (the paper uses 10 trials).
 *   sample_codes [n_sample][M] u8, in: the sampled codes (the caller draws the sample)
 *   use_index    host, out: 1 if the indexed search was faster, else 0
 *   scan_ms, index_ms   host, out, may be NULL: the best time of each, in milliseconds
 * BLOCKS: it times with HIP events it creates and destroys, and waits for them.
 *   workspace: at least pqkm_check_workspace_bytes(n_sample, M, K) bytes; M >= 2.
 */
size_t pqkm_check_workspace_bytes(int64_t n_sample, int32_t M, int32_t K);
pqkm_status pqkm_check(const uint8_t *sample_codes, int64_t n_sample, int32_t M, const uint8_t *centers,
                       int32_t K, const float *tables, int32_t trials, void *workspace,
                       size_t workspace_bytes, void *stream, int32_t *use_index, float *scan_ms,
                       float *index_ms);

/*
 * Update step by sparse voting (Eq. 7 then Eq. 8):
 *   hist[k][m][j] = #{ n : assign[n] = k and codes[n][m] = j },  counts[k] = #{ n : assign[n] = k }
 *   centers[k][m] <- argmin_l  sum_{j : hist[k][m][j] > 0} hist[k][m][j] * tables[m][j][l]
 * lowest l on ties; a center with counts[k] = 0 keeps its code.
 *   assign   [N] i32, in; every value must lie in [0, K) (not checked on the device:
 *            out-of-range values are ignored by the histogram, making counts inconsistent)
 *   centers  [K][M] u8, in/out
 *   hist     [K][M][256] u32, out, may be NULL (then it lives in the workspace)
 *   counts   [K] u32, out, may be NULL
 */
pqkm_status pqkm_update(const uint8_t *codes, int64_t N, int32_t M, const int32_t *assign,
                        int32_t K, const float *tables, uint8_t *centers, uint32_t *hist,
                        uint32_t *counts, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The naive update (Eq. 6), the method sparse voting is measured against (Sec. 3.2, Tab. 3):
 *   cost[k][m][l] = sum over the members n of cluster k of tables[m][codes[n][m]][l]
 *   centers[k][m] <- argmin_l cost[k][m][l], lowest l on ties; empty clusters keep their code.
 * O(256 M N) table entries instead of the vote's O(M (N + K 256 ||h||_0)).  The sums are fp64, taken in
 * the order a counting sort leaves the members in, which is not fixed: they are reproducible up to
 * fp64 rounding, and exactly when the table entries are integers.  With exact sums the result is
 * that of pqkm_update.
 *   cost   [K][M][256] fp64, out, may be NULL
 * N must be below 2^32.  Arguments otherwise as for pqkm_update.
 */
pqkm_status pqkm_update_naive(const uint8_t *codes, int64_t N, int32_t M, const int32_t *assign,
                              int32_t K, const float *tables, uint8_t *centers, double *cost,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * Alg. 1 with the linear scan and a fixed iteration count:
 *   repeat iters times { pqkm_assign ; pqkm_update }.
 * Init() is the caller's: `centers` holds the initial centers on entry and the
 * centers after the last update on return.  `assign` receives the result of
 * the LAST assignment step, i.e. taken against the centers as they were before
 * the last update (the order of Alg. 1).  `hist` / `counts` (may be NULL) are
 * those of the last update.  iters = 0 leaves everything untouched.
 */
pqkm_status pqkm_fit(const uint8_t *codes, int64_t N, int32_t M, const float *tables, int32_t K,
                     uint8_t *centers, int32_t iters, int32_t *assign, uint32_t *hist,
                     uint32_t *counts, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Alg. 1 with a stop condition (Sec. 3.3 leaves the stop rule of the loop open): iterate
 * { pqkm_assign ; pqkm_update } until an assignment step changes no assignment, or max_iters.
 * Per iteration the library reports, to HOST memory:
 *   objective     sum over n of the squared symmetric distance found by the assignment step
 *                 (Eq. 4 with the squared distance), accumulated in fp64 in a fixed tree order
 *   changed       number of codes whose assignment differs from the previous iteration's
 *                 (the first iteration reports N)
 *   nonzero_bins  non-zero histogram bins over all centers and subspaces (the ||h||_0 of Tab. 3, summed)
 *   nonempty      centers with at least one member
 * This is the one method entry point that BLOCKS: it synchronises `stream` once per iteration to
 * read those four numbers back.  centers / assign / hist / counts as in pqkm_fit.
 *   stats       host, [max_iters], out, may be NULL
 *   iters_done  host, out, may be NULL
 * Needs pqkm_fit_until_workspace_bytes(N, M, K) of workspace (the pqkm_fit workspace plus 8 bytes per
 * code for the previous assignment and the distances).
 */
typedef struct {
    double objective;
    int64_t changed;
    int64_t nonzero_bins;
    int64_t nonempty;
} pqkm_iter_stats;

size_t pqkm_fit_until_workspace_bytes(int64_t N, int32_t M, int32_t K);
pqkm_status pqkm_fit_until(const uint8_t *codes, int64_t N, int32_t M, const float *tables, int32_t K,
                           uint8_t *centers, int32_t max_iters, int32_t *assign, uint32_t *hist,
                           uint32_t *counts, pqkm_iter_stats *stats, int32_t *iters_done,
                           void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PQKM_H */
