"""Oracle: temporal-aware parallel clustering, TAP ("Temporal-Aware Parallel
Clustering for Calibration" section: the similarity matrices, their weighted
sum, the degree-normalised matrix, its leading eigenvectors, k-means on the
rows, aggregation over the subsamples; Algorithm TAP).  Test infrastructure.
float64.

A pool of N intermediate samples x_r (feature vectors, [N, F]) with timestamps
t_r is clustered into k groups.  For each of m subsamples S_i (n pool indices):

    A_spatial[r, h]  = x_r . x_s / (|x_r| |x_s|),   s = S_i[h]      (cosine)
    A_temporal[r, h] = exp(-|t_r - t_s|)
    A = alpha A_spatial + (1 - alpha) A_temporal                [N, n]
    d_r = row sums of A, d_c = column sums of A
    L = D_r^(-1/2) A D_c^(-1/2)                                 [N, n]
    U = the k leading left singular vectors of L               [N, k]
    labels_i = k-means on the rows of U

and the m label vectors are merged into one.

Readings taken where the paper is silent, garbled or at odds with itself:
  * shape of the similarity matrix.  The normalised matrix is stated to be
    N x n while the pair loops of the algorithm run inside the subsample.  The
    N x n shape is taken (pool rows against subsample columns): it is the only
    one that gives every pool sample a cluster, which the calibration-set
    construction of the Experimental Settings needs, and it is what makes the
    cost linear in N.  With S_i = the whole pool it is the n x n matrix.
  * exponent of the degree matrices: printed +1/2.  -1/2 is taken, the
    normalisation under which the matrix has largest singular value 1 with
    singular vectors D^(1/2) 1 (pinned), i.e. the spectral-clustering
    normalisation the text names.
  * "top k eigenvectors" of a rectangular matrix: the left singular vectors of
    the k largest singular values (= eigenvectors of L L^T).  Rows are not
    re-normalised before k-means (the text does not say so).
  * timestamps enter in the unit the caller supplies (the generators give
    step / number of steps, in [0, 1)).
  * a subsample is n distinct pool indices (each pool sample equally likely);
    the draw is an input.
  * k-means: Lloyd's iteration from initial centres that are rows of U at
    caller-supplied pool indices (the draw is an input), squared Euclidean
    distance, ties to the lowest centre index, an empty cluster keeps its
    centre, stop when no label changes or after max_iter assignment passes.
  * aggregation (not specified): the clusters of subsample i > 0 are renamed to
    those of subsample 0 by greedy maximum overlap on the k x k contingency
    table (largest count first, ties to the lowest (row, column)), then every
    sample takes the label most subsamples give it (ties to the label of the
    earliest subsample that is among the most frequent).
  * a non-positive degree (possible only when negative cosines outweigh the
    temporal term along a whole row or column) is an error.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def spatial_similarity(X, idx):
    """Cosine similarity of every pool row with every subsample row: [N, n]."""
    X = np.asarray(X, dtype=F64)
    S = X[np.asarray(idx)]
    nx = np.sqrt((X * X).sum(axis=1))
    ns = np.sqrt((S * S).sum(axis=1))
    return (X @ S.T) / (nx[:, None] * ns[None, :])


def temporal_similarity(t, idx):
    t = np.asarray(t, dtype=F64)
    ts = t[np.asarray(idx)]
    return np.exp(-np.abs(t[:, None] - ts[None, :]))


def similarity(X, t, idx, alpha: float):
    """The weighted similarity matrix of one subsample, [N, n]."""
    return alpha * spatial_similarity(X, idx) + (1.0 - alpha) * temporal_similarity(t, idx)


def degrees(A):
    A = np.asarray(A, dtype=F64)
    return A.sum(axis=1), A.sum(axis=0)


def normalised(A):
    """D_r^(-1/2) A D_c^(-1/2)."""
    A = np.asarray(A, dtype=F64)
    dr, dc = degrees(A)
    if dr.min() <= 0 or dc.min() <= 0:
        raise ValueError("non-positive degree")
    return A / np.sqrt(dr)[:, None] / np.sqrt(dc)[None, :]


def embed(L, k: int):
    """(U [N, k], sigma [k]): leading left singular vectors and values of L."""
    U, s, _ = np.linalg.svd(np.asarray(L, dtype=F64), full_matrices=False)
    return U[:, :k], s[:k]


def kmeans(U, init_idx, max_iter: int):
    """Lloyd's iteration.  Returns (labels [N] int, centres [k, d], passes)."""
    U = np.asarray(U, dtype=F64)
    centres = U[np.asarray(init_idx)].copy()
    k = centres.shape[0]
    labels = None
    passes = 0
    for _ in range(max_iter):
        d2 = ((U[:, None, :] - centres[None, :, :]) ** 2).sum(axis=2)
        new = np.argmin(d2, axis=1)                 # first minimum = lowest index on ties
        passes += 1
        if labels is not None and np.array_equal(new, labels):
            break
        labels = new
        for c in range(k):
            members = U[labels == c]
            if len(members):
                centres[c] = members.mean(axis=0)
    return labels, centres, passes


def contingency(a, b, k: int):
    """T[p, q] = number of samples with label p in a and q in b."""
    T = np.zeros((k, k), dtype=np.int64)
    for p, q in zip(np.asarray(a), np.asarray(b)):
        T[p, q] += 1
    return T


def greedy_match(T):
    """Renaming perm[q] = p of the columns of the contingency table T to its rows: the largest remaining count
    first, ties to the lowest (row, column), each row and column used once."""
    T = np.array(T, dtype=np.int64)
    k = T.shape[0]
    perm = np.full(k, -1, dtype=np.int64)
    for _ in range(k):
        flat = int(np.argmax(T))                   # first maximum in row-major order
        p, q = divmod(flat, k)
        perm[q] = p
        T[p, :] = -1
        T[:, q] = -1
    return perm


def aggregate(labels, k: int):
    """labels [m, N] -> [N]."""
    labels = np.asarray(labels)
    m, N = labels.shape
    renamed = [labels[0]]
    for i in range(1, m):
        perm = greedy_match(contingency(labels[0], labels[i], k))
        renamed.append(perm[labels[i]])
    renamed = np.stack(renamed)
    out = np.empty(N, dtype=np.int64)
    for r in range(N):
        votes = np.bincount(renamed[:, r], minlength=k)
        best = votes.max()
        for i in range(m):                          # earliest subsample whose label is among the most frequent
            if votes[renamed[i, r]] == best:
                out[r] = renamed[i, r]
                break
    return out


def tap(X, t, subsamples, alpha: float, k: int, init_idx, max_iter: int):
    """The whole algorithm.  subsamples [m, n] pool indices, init_idx [m, k] pool indices of the initial centres.
    Returns (final labels [N], per-subsample labels [m, N])."""
    per = []
    for S, init in zip(subsamples, init_idx):
        U, _ = embed(normalised(similarity(X, t, S, alpha)), k)
        per.append(kmeans(U, init, max_iter)[0])
    per = np.stack(per)
    return aggregate(per, k), per
