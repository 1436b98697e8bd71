/*
 * qc_tap.h - C ABI of the calibration-set clustering (temporal-aware parallel
 * clustering, TAP) of "Q&C: When Quantization Meets Cache in Efficient Image
 * Generation" (arXiv 2503.02508), section "Temporal-Aware Parallel Clustering
 * for Calibration" and its algorithm, for MI355X (gfx950).
 *
 * A pool of N intermediate samples (feature vectors X[N, F], timestamps t[N])
 * is clustered into k groups.  For each of m subsamples S (n pool indices):
 *   A[r, h] = alpha cos(x_r, x_S[h]) + (1 - alpha) exp(-|t_r - t_S[h]|)   [N, n]
 *   L = D_r^(-1/2) A D_c^(-1/2),  d_r / d_c the row / column sums of A
 *   U = the k leading left singular vectors of L                          [N, k]
 *   labels = k-means on the rows of U
 * and the m label vectors are merged.  The readings taken where the paper
 * leaves a choice (N x n shape, exponent -1/2, singular vectors for the
 * "eigenvectors" of a rectangular matrix, Lloyd's iteration from given rows,
 * renaming by greedy overlap and majority vote) are stated at each call.
 *
 * Conventions are those of qc.h: return QC_OK or a negative qc_status with a
 * text in qc_last_error(); "dev" pointers are device memory owned by the
 * caller, 16-byte aligned, tensors row-major and dense; `stream` is a
 * hipStream_t as void*.  The library allocates nothing: every call takes a
 * device workspace `work` of at least the size qc_tap_workspace_bytes gives
 * for its dimensions (one size covers every call).  Argument checks run before
 * any device call.  Calls that report a data-dependent error (an index out of
 * range, a non-positive degree, a rank-deficient start block) or a count wait
 * for the stream before they return; this is said at each call.
 *
 * Limits: 1 <= k <= kb <= 128, kb a multiple of 8, kb <= n <= N, m <= 8,
 * N * max(n, F) < 2^31.
 */
#ifndef QC_TAP_H_
#define QC_TAP_H_

#include <stddef.h>
#include "qc.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Workspace bytes that cover every call below at these dimensions (kb = size of
 * the iteration block of qc_tap_embed; pass kb = k rounded up to a multiple of
 * 8 plus the guard vectors wanted).  Host call. */
int qc_tap_workspace_bytes(int N, int F, int n, int k, int kb, size_t *bytes_out);

/* Weighted similarity of every pool sample with every sample of one subsample
 * (the spatial cosine matrix, the temporal matrix exp(-|dt|) and their
 * alpha-weighted sum), and its degrees:
 *   A[r, h] = alpha x_r.x_s / (|x_r| |x_s|) + (1 - alpha) exp(-|t_r - t_s|), s = idx[h]
 *   d_r[r] = sum_h A[r, h],  d_c[h] = sum_r A[r, h]
 * X dev [N, F] fp32, t dev [N] fp32 (in the unit the caller chooses), idx dev
 * [n] int32 pool indices (need not be sorted), A dev [N, n], d_r dev [N], d_c
 * dev [n] fp32 out.  The contraction runs on the fp32 matrix cores with fp32
 * accumulation; norms and degree sums accumulate in fp64.  A zero feature
 * vector has cosine 0 with everything.  Waits for the stream; QC_ERR_RANGE if
 * an index lies outside [0, N) (A, d_r, d_c are then unspecified). */
int qc_tap_similarity(const float *X, const float *t, int N, int F, const int *idx, int n, float alpha,
                      float *A, float *d_r, float *d_c, void *work, size_t work_bytes, void *stream);

/* Degree normalisation in place: A[r, h] <- A[r, h] / sqrt(d_r[r] d_c[h]) (the
 * "normalised Laplacian" equation with the exponent read as -1/2: the matrix
 * whose largest singular value is 1).  Waits for the stream; QC_ERR_RANGE if a
 * degree is not positive and finite (A is then left as it was). */
int qc_tap_normalise(float *A, const float *d_r, const float *d_c, int N, int n, void *work, size_t work_bytes,
                     void *stream);

/* The k leading left singular vectors of L[N, n] ("top k eigenvectors") and the
 * singular values: block power iteration on L^T L with kb >= k vectors started
 * from q0 (dev [kb, n] fp32, caller-drawn random numbers), `iters` rounds of
 * multiply + shifted Cholesky QR in fp64 (one pass between two multiplications,
 * three passes for the final basis), then a Rayleigh-Ritz step on the kb-dimensional subspace (Jacobi rotations) that
 * keeps the k largest.  U dev [N, k] out: orthonormal columns, column j
 * belonging to sigma[j] (dev [k] out, descending); each column's sign is
 * arbitrary.  The error of the subspace falls as (sigma_kb+1 / sigma_k)^(2 iters).
 * Directions of the block that the multiplication sends into rounding noise are
 * replaced by arbitrary orthonormal ones.  Waits for the stream; QC_ERR_RANGE if
 * the block still has no full rank after orthonormalisation (a zero start
 * vector). */
int qc_tap_embed(const float *L, int N, int n, int k, int kb, int iters, const float *q0, float *U, float *sigma,
                 void *work, size_t work_bytes, void *stream);

/* k-means on the rows of U[N, d] (Lloyd's iteration): the initial centres are
 * the rows init_idx[k] (dev int32, caller-drawn), a row goes to the nearest
 * centre in squared Euclidean distance (fp32, ties to the lowest centre), a
 * centre becomes the mean of its rows (fp64 sums in a fixed order; an empty
 * cluster keeps its centre); stops when a pass changes no label or after
 * max_iter assignment passes.  labels dev [N] int32 out, centres dev [k, d]
 * fp32 out, *passes_out host (may be NULL) = assignment passes run.  d <= 128.
 * The passes decide on the device whether they still have work; the host waits
 * for the stream after every eighth pass (and at the end).  QC_ERR_RANGE for an
 * index outside [0, N). */
int qc_tap_kmeans(const float *U, int N, int d, int k, const int *init_idx, int max_iter, int *labels,
                  float *centres, int *passes_out, void *work, size_t work_bytes, void *stream);

/* Merges m label vectors (labels dev [m, N] int32, values in [0, k)) into one
 * (out dev [N] int32): the clusters of vector i > 0 are renamed to those of
 * vector 0 by greedy maximum overlap on the k x k contingency table (largest
 * count first, ties to the lowest (row, column), each name used once), then
 * each sample takes the name most vectors give it (ties to the name given by
 * the earliest vector among the most frequent).  perm_out dev [m, k] int32 out
 * (may be NULL): perm_out[i, q] = the name in vector 0's terms of cluster q of
 * vector i.  Only enqueues work.  A label outside [0, k) is counted as k - 1 or
 * 0, whichever is nearer. */
int qc_tap_aggregate(const int *labels, int m, int N, int k, int *out, int *perm_out, void *work, size_t work_bytes,
                     void *stream);

/* The whole algorithm: for each of the m subsamples (subsamples dev [m, n]
 * int32) similarity, normalisation, embedding (start block q0 dev [kb, n],
 * shared by the subsamples) and k-means (init_idx dev [m, k]); then the merge.
 * labels_out dev [N] int32, per_labels dev [m, N] int32 out.  With a workspace
 * of s times the size qc_tap_workspace_bytes gives (s = 2 or 3) the call
 * works on s subsamples at a time: the first on `stream`, the others on
 * internal streams of the library that start after the work already enqueued
 * on `stream` and have drained when the call returns (the results do not
 * depend on s).  Waits for the stream; errors as in the calls above, reported
 * after the k-means of the subsample concerned (the outputs are then
 * unspecified).  Process-wide internal streams: calls must not overlap. */
int qc_tap_cluster(const float *X, const float *t, int N, int F, const int *subsamples, int m, int n, float alpha,
                   int k, int kb, int iters, const float *q0, const int *init_idx, int max_iter, int *labels_out,
                   int *per_labels, void *work, size_t work_bytes, void *stream);

/* Measurement aid: between qc_tap_profile_begin and qc_tap_profile_end every
 * launch of the similarity contraction (the dominant kernel of the algorithm)
 * is bracketed by events on the stream it is launched on.  _end waits for
 * them and returns the summed duration in milliseconds and the number of
 * launches (host pointers); QC_ERR_STATE without a _begin.  Process-wide, not
 * thread-safe. */
int qc_tap_profile_begin(void);
int qc_tap_profile_end(float *sim_ms_out, int *launches_out);

#ifdef __cplusplus
}
#endif
#endif
