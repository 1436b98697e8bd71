"""Pins for the clustering oracle (similarity matrices, degree normalisation, leading singular vectors, k-means,
aggregation over subsamples; the calibration-set clustering section of the paper and its algorithm).  CPU only.  Each
test checks the oracle against something other than itself: hand values, theorems about the normalised matrix,
library routines it does not call, brute force."""
import itertools
import math

import numpy as np
import pytest

from oracle import tap
from synthetic import tap_inputs as TI


# ------------------------------------------------------------------ similarity
def test_similarity_hand_values():
    # unit vectors at 0, 60 and 90 degrees and an opposite one; lengths must not matter
    X = np.array([[2.0, 0.0], [0.5, 0.5 * math.sqrt(3)], [0.0, 3.0], [-1.0, 0.0]])
    t = np.array([0.0, 1.0, 0.25, 0.0])
    idx = [0, 2]
    S = tap.spatial_similarity(X, idx)
    assert np.allclose(S, [[1, 0], [0.5, math.sqrt(3) / 2], [0, 1], [-1, 0]], atol=1e-15)
    T = tap.temporal_similarity(t, idx)
    assert np.allclose(T, [[1, math.exp(-0.25)], [math.exp(-1), math.exp(-0.75)], [math.exp(-0.25), 1], [1, math.exp(-0.25)]])
    A = tap.similarity(X, t, idx, 0.3)
    assert np.allclose(A, 0.3 * S + 0.7 * T)
    assert np.allclose(tap.similarity(X, t, idx, 1.0), S) and np.allclose(tap.similarity(X, t, idx, 0.0), T)


def test_spatial_similarity_against_library_distance():
    from scipy.spatial.distance import cdist
    rng = np.random.default_rng(0)
    X = rng.standard_normal((40, 17)) * rng.uniform(0.1, 10, size=(40, 1))
    idx = np.sort(rng.choice(40, 9, replace=False))
    want = 1.0 - cdist(X, X[idx], metric="cosine")
    assert np.allclose(tap.spatial_similarity(X, idx), want, atol=1e-13)
    # whole pool as the subsample: symmetric, unit diagonal
    S = tap.spatial_similarity(X, np.arange(40))
    assert np.allclose(S, S.T) and np.allclose(np.diag(S), 1.0)


# ------------------------------------------------------------- normalisation
def test_normalised_matrix_has_unit_top_singular_value_with_root_degree_vectors():
    """For a non-negative matrix, D_r^-1/2 A D_c^-1/2 has largest singular value exactly 1, with left and right
    singular vectors sqrt(d_r) and sqrt(d_c) (normalised).  Fails for +1/2 exponents and for swapped degrees."""
    rng = np.random.default_rng(1)
    A = rng.uniform(0.1, 1.0, size=(30, 7))
    L = tap.normalised(A)
    dr, dc = A.sum(axis=1), A.sum(axis=0)
    u, v = np.sqrt(dr / dr.sum()), np.sqrt(dc / dc.sum())
    assert np.allclose(L @ v, u, atol=1e-14) and np.allclose(L.T @ u, v, atol=1e-14)
    s = np.linalg.svd(L, compute_uv=False)
    assert abs(s[0] - 1.0) < 1e-13 and s[1] < 1.0
    U, sig = tap.embed(L, 3)
    assert abs(abs(U[:, 0] @ u) - 1.0) < 1e-12 and np.allclose(sig, s[:3])
    # all-ones matrix: every entry 1 / sqrt(N n)
    assert np.allclose(tap.normalised(np.ones((6, 4))), 1.0 / math.sqrt(24))
    with pytest.raises(ValueError):
        tap.normalised(np.array([[1.0, -2.0], [0.5, 0.5]]))


def test_disconnected_groups_give_unit_singular_values_and_piecewise_embedding():
    """Block structure (no similarity across groups): one singular value 1 per group; within a group the rows of
    the embedding are parallel (they differ only by the root-degree scale)."""
    rng = np.random.default_rng(2)
    sizes_r, sizes_c = [5, 9, 4], [3, 2, 4]
    A = np.zeros((18, 9))
    r0 = c0 = 0
    groups = []
    for g, (a, b) in enumerate(zip(sizes_r, sizes_c)):
        A[r0:r0 + a, c0:c0 + b] = rng.uniform(0.2, 1.0, size=(a, b))
        groups += [g] * a
        r0 += a; c0 += b
    L = tap.normalised(A)
    U, s = tap.embed(L, 3)
    assert np.allclose(s, 1.0, atol=1e-12)
    assert np.linalg.svd(L, compute_uv=False)[3] < 1 - 1e-3
    groups = np.array(groups)
    for g in range(3):
        rows = U[groups == g]
        unit = rows / np.linalg.norm(rows, axis=1, keepdims=True)
        assert np.allclose(np.abs(unit @ unit[0]), 1.0, atol=1e-10)
    for g, h in itertools.combinations(range(3), 2):       # rows of different groups are orthogonal
        assert np.allclose(U[groups == g] @ U[groups == h].T, 0.0, atol=1e-10)


def test_embedding_against_symmetric_eigensolver():
    rng = np.random.default_rng(3)
    L = tap.normalised(rng.uniform(0.0, 1.0, size=(50, 12)) ** 3)
    U, s = tap.embed(L, 4)
    w, V = np.linalg.eigh(L @ L.T)                            # a different routine: eigenvectors of L L^T
    order = np.argsort(w)[::-1][:4]
    assert np.allclose(np.sqrt(w[order]), s, atol=1e-12)
    P_svd, P_eig = U @ U.T, V[:, order] @ V[:, order].T       # projectors do not depend on signs
    assert np.allclose(P_svd, P_eig, atol=1e-10)
    assert np.allclose(U.T @ U, np.eye(4), atol=1e-13)


# -------------------------------------------------------------------- k-means
def test_kmeans_against_library_lloyd():
    from sklearn.cluster import KMeans
    rng = np.random.default_rng(4)
    centres = rng.standard_normal((5, 6)) * 3
    U = centres[rng.integers(0, 5, size=400)] + 0.7 * rng.standard_normal((400, 6))
    init = rng.choice(400, 5, replace=False)
    labels, c, passes = tap.kmeans(U, init, 100)
    km = KMeans(n_clusters=5, init=U[init], n_init=1, algorithm="lloyd", max_iter=300, tol=0.0).fit(U)
    assert np.array_equal(labels, km.labels_)
    assert np.allclose(c, km.cluster_centers_, atol=1e-12)
    assert 2 <= passes < 100


def test_kmeans_fixed_point_ties_and_empty_cluster():
    # 1-D points traced by hand; initial centres on points 0 and 1, point 2 starts equidistant
    U = np.array([[0.0], [2.0], [1.0], [10.0]])
    labels, c, passes = tap.kmeans(U, [0, 1], 10)
    # pass 1: centres 0, 2 -> point 1.0 ties -> lowest index (0); point 10 -> 1. centres 0.5, 6
    # pass 2: 0 -> 0, 2 -> 0, 1 -> 0, 10 -> 1: centres 1, 10;  pass 3 unchanged
    assert labels.tolist() == [0, 0, 0, 1] and np.allclose(c[:, 0], [1.0, 10.0]) and passes == 3
    # an empty cluster keeps its centre: two identical initial centres, the second loses every tie of the first
    # pass and is left where it was; in the second pass it wins back the two points it sits on
    U = np.array([[1.0], [1.0], [3.0]])
    labels, c, _ = tap.kmeans(U, [0, 1], 1)
    assert labels.tolist() == [0, 0, 0] and c[1, 0] == 1.0 and c[0, 0] == pytest.approx(5.0 / 3)
    labels, c, passes = tap.kmeans(U, [0, 1], 10)
    assert labels.tolist() == [1, 1, 0] and c[:, 0].tolist() == [3.0, 1.0] and passes == 3
    # labels are the nearest centre, the centres the member means (fixed point), the objective never below brute force
    rng = np.random.default_rng(5)
    U = rng.standard_normal((9, 2))
    labels, c, _ = tap.kmeans(U, [0, 1, 2], 50)
    d2 = ((U[:, None] - c[None]) ** 2).sum(-1)
    assert np.array_equal(labels, d2.argmin(1))
    obj = d2[np.arange(9), labels].sum()
    best = min(sum(((U[np.array(a) == g] - U[np.array(a) == g].mean(0)) ** 2).sum() for g in set(a))
               for a in itertools.product(range(3), repeat=9))
    assert obj >= best - 1e-12


# ---------------------------------------------------------------- aggregation
def test_contingency_and_greedy_match():
    a = np.array([0, 0, 1, 1, 2, 2, 2])
    b = np.array([2, 2, 0, 0, 1, 1, 0])
    T = tap.contingency(a, b, 3)
    assert T.tolist() == [[0, 0, 2], [2, 0, 0], [1, 2, 0]] and T.sum() == 7
    perm = tap.greedy_match(T)
    assert perm.tolist() == [1, 2, 0]                        # b's 0 -> a's 1, 1 -> 2, 2 -> 0
    # ties go to the lowest (row, column) and every label is used once
    assert sorted(tap.greedy_match(np.ones((4, 4), dtype=int)).tolist()) == [0, 1, 2, 3]
    assert tap.greedy_match(np.ones((3, 3), dtype=int)).tolist() == [0, 1, 2]


def test_aggregate_is_invariant_to_renaming_and_votes_by_majority():
    rng = np.random.default_rng(6)
    base = rng.integers(0, 5, size=200)
    perms = [rng.permutation(5) for _ in range(3)]
    labels = np.stack([base, perms[1][base], perms[2][base]])
    assert np.array_equal(tap.aggregate(labels, 5), base)
    # one subsample disagrees on some samples: the other two outvote it
    noisy = labels.copy()
    flip = rng.choice(200, 20, replace=False)
    noisy[2, flip] = (noisy[2, flip] + 1) % 5
    assert np.array_equal(tap.aggregate(noisy, 5), base)
    # greedy matching agrees with the best of all renamings when the overlap is clear (brute force, k = 4)
    a = rng.integers(0, 4, size=300)
    b = rng.permutation(4)[a]
    b[rng.choice(300, 30, replace=False)] = rng.integers(0, 4, size=30)
    perm = tap.greedy_match(tap.contingency(a, b, 4))
    best = max(itertools.permutations(range(4)), key=lambda p: np.sum(np.array(p)[b] == a))
    assert perm.tolist() == list(best)
    # three-way disagreement: the earliest subsample's label wins
    three = np.array([[0, 1], [1, 1], [2, 0]])
    out = tap.aggregate(np.stack([np.r_[three[:, 0], np.arange(3)], np.r_[three[:, 1], np.arange(3)]]), 3)
    assert out[:3].tolist() == [0, 1, 2]


# ------------------------------------------------------------------ whole algorithm
def test_planted_groups_are_recovered():
    k, N = 6, 360
    X, t, truth = TI.make_planted(N, 48, k, seed=7)
    subs = TI.make_subsamples(N, 60, 3, seed=8)
    init = np.stack([[int(np.flatnonzero(truth == g)[i]) for g in range(k)] for i in range(3)])
    final, per = tap.tap(X, t, subs, 0.5, k, init, 50)
    for lab in list(per) + [final]:
        T = tap.contingency(truth, lab, k)
        assert (T > 0).sum() == k                            # a one-to-one renaming of the planted groups
    assert np.array_equal(tap.greedy_match(tap.contingency(truth, final, k))[final], truth)


def test_generators_are_seeded_and_shaped():
    wl = TI.TAP_WORKLOADS["tap0"]
    X, t, cls, step = TI.make_pool(wl.N, wl.F, wl.steps, wl.classes, wl.seed)
    X2, _, _, _ = TI.make_pool(wl.N, wl.F, wl.steps, wl.classes, wl.seed)
    assert X.shape == (wl.N, wl.F) and X.dtype == np.float32 and np.array_equal(X, X2)
    assert t.min() >= 0 and t.max() < 1
    s = TI.make_subsamples(wl.N, wl.n, wl.m, 1)
    assert s.shape == (wl.m, wl.n) and all(len(set(r)) == wl.n and np.all(np.diff(r) > 0) for r in s)
    assert TI.make_init(wl.N, wl.k, wl.m, 2).shape == (wl.m, wl.k)
