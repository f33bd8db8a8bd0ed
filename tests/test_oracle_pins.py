"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- library routines (torch SDPA, scipy softmax / kmeans2,
scikit-learn Lloyd, numpy stable argsort), closed forms, invariants the paper
proves (Section 4.1 permutation equivalence), brute force on tiny inputs and
the one worked number the paper prints (Section 4.3 padding example)."""
import os

import numpy as np
import pytest
import scipy.special
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _sdpa(Q, K, V, scale=None):
    """Library dense attention in float64."""
    q, k, v = (torch.from_numpy(np.asarray(a, dtype=np.float64))[None, None] for a in (Q, K, V))
    o = torch.nn.functional.scaled_dot_product_attention(q, k, v, scale=scale)
    return o[0, 0].numpy()


# ------------------------------------------------------------------ dense attention (Section 3.1)

def test_dense_matches_library_sdpa(oracle):
    r = _rng(0)
    Q, K, V = r.standard_normal((37, 24)), r.standard_normal((53, 24)), r.standard_normal((53, 24))
    O, lse = oracle.dense_attention(Q, K, V)
    np.testing.assert_allclose(O, _sdpa(Q.astype(np.float32), K.astype(np.float32), V.astype(np.float32)),
                               rtol=1e-10, atol=1e-12)
    S = (Q.astype(np.float32).astype(np.float64) @ K.astype(np.float32).astype(np.float64).T) / np.sqrt(24)
    np.testing.assert_allclose(lse, scipy.special.logsumexp(S, axis=1), rtol=1e-12)


def test_dense_closed_forms(oracle):
    r = _rng(1)
    Q, K = r.standard_normal((9, 8)), r.standard_normal((11, 8))
    # constant V -> constant output
    V = np.tile(r.standard_normal((1, 8)), (11, 1))
    O, _ = oracle.dense_attention(Q, K, V)
    np.testing.assert_allclose(O, np.tile(V[:1].astype(np.float32), (9, 1)), rtol=1e-12)
    # a single key -> its value row, lse = the score
    V1 = r.standard_normal((1, 8))
    O, lse = oracle.dense_attention(Q, K[:1], V1)
    np.testing.assert_allclose(O, np.tile(V1.astype(np.float32), (9, 1)), rtol=1e-12)
    s = (Q.astype(np.float32).astype(np.float64) @ K[:1].astype(np.float32).astype(np.float64).T)[:, 0] / np.sqrt(8)
    np.testing.assert_allclose(lse, s, rtol=1e-12)
    # zero queries -> uniform weights: O = mean(V), lse = log Nk
    V = r.standard_normal((11, 8))
    O, lse = oracle.dense_attention(np.zeros((3, 8)), K, V)
    np.testing.assert_allclose(O, np.tile(V.astype(np.float32).astype(np.float64).mean(0), (3, 1)), rtol=1e-12)
    np.testing.assert_allclose(lse, np.log(11.0), rtol=1e-12)
    # two keys -> logistic function of the score difference, scale applied once
    q = np.array([[2.0, 0.0]]); K2 = np.array([[1.0, 0.0], [-1.0, 0.0]]); V2 = np.array([[1.0, 0.0], [0.0, 1.0]])
    O, _ = oracle.dense_attention(q, K2, V2)
    w = 1.0 / (1.0 + np.exp(-(4.0 / np.sqrt(2.0))))
    np.testing.assert_allclose(O, [[w, 1.0 - w]], rtol=1e-12)


def test_dense_rectangular_uses_value_of_matching_key(oracle):
    # catches a transposed operand: one-hot-like scores pick distinct value rows
    K = np.eye(4) * 50.0
    Q = np.eye(4)[[2, 0, 3]] * 50.0
    V = np.arange(16, dtype=np.float64).reshape(4, 4)
    O, _ = oracle.dense_attention(Q, K, V)
    np.testing.assert_allclose(O, V[[2, 0, 3]], atol=1e-9)


# ------------------------------------------------------------------ k-means (Section 4.1)

def _mixture(r, N, d, M, sep):
    mu = sep * r.standard_normal((M, d))
    comp = r.integers(0, M, size=N)
    X = (mu[comp] + r.standard_normal((N, d))).astype(np.float32)
    return X, mu, comp


def test_kmeans_matches_scipy_kmeans2(oracle):
    from scipy.cluster.vq import kmeans2
    r = _rng(2)
    X, _, _ = _mixture(r, 600, 8, 5, 1.0)
    init = X[r.choice(600, 12, replace=False)].astype(np.float64)
    for T in (1, 2, 5):
        res = oracle.kmeans(X, init, T, round_bf16=False)
        cb, lab = kmeans2(X.astype(np.float64), init.copy(), iter=T, minit="matrix", missing="warn")
        np.testing.assert_array_equal(res.labels, lab)
        np.testing.assert_allclose(res.centroids, cb, rtol=1e-10, atol=1e-12)
        np.testing.assert_array_equal(res.counts, np.bincount(lab, minlength=12))


def test_kmeans_matches_sklearn_lloyd(oracle):
    from sklearn.cluster import KMeans
    r = _rng(3)
    X, _, _ = _mixture(r, 500, 6, 4, 2.0)
    init = X[r.choice(500, 7, replace=False)].astype(np.float64)
    T = 3
    res = oracle.kmeans(X, init, T, round_bf16=False)
    assert res.counts.min() > 0          # scikit-learn relocates empty clusters; none here
    km = KMeans(n_clusters=7, init=init, n_init=1, max_iter=T, tol=0.0, algorithm="lloyd").fit(X.astype(np.float64))
    np.testing.assert_allclose(res.centroids, km.cluster_centers_, rtol=1e-6, atol=1e-8)


def test_kmeans_objective_never_increases(oracle):
    r = _rng(4)
    X, _, _ = _mixture(r, 800, 16, 6, 0.7)
    init = X[r.choice(800, 20, replace=False)]
    res = oracle.kmeans(X, init, 8, round_bf16=False)
    J = res.objective
    assert np.all(np.diff(J) <= 1e-9 * J[0]), J
    # the value itself: brute force against the returned means
    d2 = ((X.astype(np.float64) - res.centroids[res.labels]) ** 2).sum()
    np.testing.assert_allclose(J[-1], d2, rtol=1e-12)
    # with centroids rounded for the assign step each half step still cannot increase
    res = oracle.kmeans(X, init, 6, round_bf16=True)
    J = res.objective
    assert np.all(J[1::2] <= J[0::2] * (1 + 1e-12))     # update <= the assign before it


def test_kmeans_special_cases(oracle):
    r = _rng(5)
    X = r.standard_normal((300, 5)).astype(np.float32)
    # C = 1: the centroid is the global mean after one iteration
    res = oracle.kmeans(X, np.zeros((1, 5)), 1, False)
    np.testing.assert_allclose(res.centroids[0], X.astype(np.float64).mean(0), rtol=1e-12)
    assert res.counts[0] == 300 and not res.labels.any()
    # C = N with the points as centroids: identity labels, zero objective
    res = oracle.kmeans(X[:40], X[:40], 2, False)
    np.testing.assert_array_equal(res.labels, np.arange(40))
    np.testing.assert_allclose(res.objective, 0.0, atol=1e-9)
    # counts sum to N, centroid * count = sum of members
    init = X[:9]
    res = oracle.kmeans(X, init, 3, False)
    assert res.counts.sum() == 300
    for j in range(9):
        np.testing.assert_allclose(res.centroids[j] * res.counts[j],
                                   X[res.labels == j].astype(np.float64).sum(0), rtol=1e-10, atol=1e-10)


def test_kmeans_recovers_separated_mixture_and_is_stable_under_warm_start(oracle):
    r = _rng(6)
    X, mu, comp = _mixture(r, 1000, 12, 6, 8.0)
    res = oracle.kmeans(X, mu, 3, False)
    np.testing.assert_array_equal(res.labels, comp)
    again = oracle.kmeans(X, res.centroids, 2, False)
    np.testing.assert_array_equal(again.labels, res.labels)
    np.testing.assert_allclose(again.centroids, res.centroids, rtol=1e-12)


def test_kmeans_tie_goes_to_lowest_index_and_empty_cluster_keeps_centroid(oracle):
    X = np.array([[0.0, 0.0], [1.0, 0.0], [0.0, 1.0], [1.0, 1.0]], dtype=np.float32)
    far = np.array([100.0, 100.0])
    init = np.array([[0.5, 0.5], [0.5, 0.5], far])          # clusters 0 and 1 tie everywhere
    res = oracle.kmeans(X, init, 2, False)
    np.testing.assert_array_equal(res.labels, [0, 0, 0, 0])
    np.testing.assert_array_equal(res.counts, [4, 0, 0])
    np.testing.assert_allclose(res.centroids[1], [0.5, 0.5])
    np.testing.assert_allclose(res.centroids[2], far)
    # the sign of the cross term matters: the nearest centroid is NOT the one with the smallest norm
    X = np.array([[10.0, 0.0]], dtype=np.float32)
    res = oracle.kmeans(X, np.array([[0.0, 0.0], [9.0, 0.0]]), 1, False)
    assert res.labels[0] == 1


def test_kmeans_labels_on_near_ties_and_exact_ties_follow_exact_arithmetic(oracle):
    """The input of the GPU's near-tie test (tokens next to, and exactly on, the hyperplane between two centroids):
    the oracle's labels are the argmin of the squared distances in EXACT arithmetic -- Python integers on the bf16
    values scaled to integers -- with the lower index on a tie.  A float64 shortcut in the oracle that lost the
    last bits of a near-tie, or a tie rule that went the other way, fails here."""
    from _util import bisector_case
    X, cent, n_tie = bisector_case(64, 24, N=1500, n_tie=300)
    assert n_tie == 300
    res = oracle.kmeans(X, cent, 1, True)
    # bf16 values are integers times 2^-133 at the finest; these inputs are O(1..10) with 8-bit mantissas, so 2^40
    # scales every value to an exact integer that Python's integers then square and sum without rounding
    Xi = [[int(v) for v in row] for row in np.round(X.astype(np.float64) * 2.0 ** 40)]
    Ci = [[int(v) for v in row] for row in np.round(cent.astype(np.float64) * 2.0 ** 40)]
    assert np.array_equal(np.array(Xi, dtype=np.float64) * 2.0 ** -40, X.astype(np.float64))
    assert np.array_equal(np.array(Ci, dtype=np.float64) * 2.0 ** -40, cent.astype(np.float64))
    ties = 0
    for n, x in enumerate(Xi):
        dist = [sum((a - b) * (a - b) for a, b in zip(x, c)) for c in Ci]
        best = min(dist)
        ties += dist.count(best) > 1
        assert res.labels[n] == dist.index(best), (n, res.labels[n], dist.index(best))
    assert ties >= 250


def test_kmeans_assign_sees_bf16_rounded_centroids(oracle):
    r = _rng(7)
    X = r.standard_normal((400, 16)).astype(np.float32)
    X = torch.from_numpy(X).to(torch.bfloat16).to(torch.float32).numpy()
    init = (X[:10] + 0.37 * r.standard_normal((10, 16))).astype(np.float32)
    res = oracle.kmeans(X, init, 1, round_bf16=True)
    cr = torch.from_numpy(init).to(torch.bfloat16).to(torch.float64).numpy()      # library rounding (RNE)
    dist = ((X.astype(np.float64)[:, None, :] - cr[None]) ** 2).sum(-1)
    np.testing.assert_array_equal(res.labels, dist.argmin(1))
    # the returned centroids are unrounded means
    for j in range(10):
        if res.counts[j]:
            np.testing.assert_allclose(res.centroids[j], X[res.labels == j].astype(np.float64).mean(0), rtol=1e-12)
    # and the top-2 gap helper agrees with a sort of the same distances
    gap = oracle.top2_gap(X, init, True)
    ds = np.sort(dist, axis=1)
    np.testing.assert_allclose(gap, (ds[:, 1] - ds[:, 0]) / ds[:, 1], rtol=1e-9, atol=1e-12)


# ------------------------------------------------------------------ permutation (Section 4.1)

def test_permute_is_a_stable_sort_by_label(oracle):
    r = _rng(8)
    labels = r.integers(0, 13, size=1000).astype(np.int32)
    labels[labels == 5] = 6                                  # leave one cluster empty
    res = oracle.permute(labels, 13)
    np.testing.assert_array_equal(res.perm, np.argsort(labels, kind="stable"))
    np.testing.assert_array_equal(res.counts, np.bincount(labels, minlength=13))
    np.testing.assert_array_equal(res.offsets, np.concatenate([[0], np.cumsum(res.counts)]))
    assert res.offsets[-1] == 1000 and res.counts[5] == 0
    np.testing.assert_array_equal(np.sort(res.perm), np.arange(1000))        # bijection
    np.testing.assert_array_equal(res.inv_perm[res.perm], np.arange(1000))   # inverse
    np.testing.assert_array_equal(res.perm[res.inv_perm], np.arange(1000))
    assert np.all(np.diff(labels[res.perm]) >= 0)
    X = r.standard_normal((1000, 4)).astype(np.float32)
    np.testing.assert_array_equal(oracle.gather_rows(X, res.perm), X[res.perm])


# ------------------------------------------------------------------ Eq. 1, Eq. 2, top-p (Section 4.2)

def test_select_hand_worked_example(oracle):
    # zero centroids -> S = 0 -> P' is the size share: 0.1, 0.2, 0.3, 0.4
    cq = np.zeros((2, 4)); ck = np.zeros((4, 4))
    counts_k = np.array([1, 2, 3, 4])
    res = oracle.select_topp(cq, ck, np.array([5, 7]), counts_k, 0.65)
    np.testing.assert_allclose(res.p_est, np.tile([0.1, 0.2, 0.3, 0.4], (2, 1)), rtol=1e-12)
    np.testing.assert_array_equal(res.row_ptr, [0, 2, 4])
    np.testing.assert_array_equal(res.col_idx, [2, 3, 2, 3])                 # 0.4 + 0.3 crosses 0.65
    np.testing.assert_allclose(res.density, 0.7, rtol=1e-12)                 # 7 of 10 keys for every query
    np.testing.assert_allclose(res.margin, [0.05, 0.05], rtol=1e-9)
    res = oracle.select_topp(cq, ck, None, counts_k, 0.75)
    np.testing.assert_array_equal(res.col_idx, [1, 2, 3, 1, 2, 3])
    res = oracle.select_topp(cq, ck, None, counts_k, 0.3)                    # first element alone suffices
    np.testing.assert_array_equal(res.col_idx, [3, 3])
    # a score that favours the small cluster: S = ln 8 for cluster 0 -> weights 8,2,3,4
    ckb = np.zeros((4, 4)); ckb[0, 0] = 2.0 * np.log(8.0)
    cqb = np.zeros((1, 4)); cqb[0, 0] = 1.0                                  # sqrt(d) = 2
    res = oracle.select_topp(cqb, ckb, None, counts_k, 0.5)
    np.testing.assert_allclose(res.p_est[0], np.array([8, 2, 3, 4]) / 17.0, rtol=1e-12)
    np.testing.assert_array_equal(res.col_idx, [0, 3])


def test_select_margin_is_set_by_the_gap_between_last_kept_and_first_dropped(oracle):
    # zero centroids -> P' is the size share 0.5, 0.25, 0.249, 0.001.  At p = 0.7 the kept clusters are {0, 1}:
    # mass before the last kept 0.5 (0.2 from p), mass including it 0.75 (0.05 from p), but the first dropped
    # cluster is within (0.25 - 0.249) / 0.25 = 0.004 of the last kept: the relative P' gap is what makes the
    # decision fragile, so it is the margin
    cq = np.zeros((1, 4)); ck = np.zeros((4, 4))
    counts_k = np.array([500, 250, 249, 1])
    res = oracle.select_topp(cq, ck, None, counts_k, 0.7)
    np.testing.assert_array_equal(res.col_idx, [0, 1])
    np.testing.assert_allclose(res.margin, [0.004], rtol=1e-9)
    # the same sizes at p = 0.755: {0, 1, 2} kept (0.75 < 0.755), the mass including the last kept is 0.999;
    # |0.75 - 0.755| = 0.005 binds, not the gap to the 0.001 cluster ((0.249 - 0.001) / 0.249 = 0.996)
    res = oracle.select_topp(cq, ck, None, counts_k, 0.755)
    np.testing.assert_array_equal(res.col_idx, [0, 1, 2])
    np.testing.assert_allclose(res.margin, [0.005], rtol=1e-9)
    # an empty cluster between them is never "the first dropped": sizes 500, 250, 0, 249, 1 give the same margin
    res = oracle.select_topp(cq, np.zeros((5, 4)), None, np.array([500, 250, 0, 249, 1]), 0.7)
    np.testing.assert_array_equal(res.col_idx, [0, 1])
    np.testing.assert_allclose(res.margin, [0.004], rtol=1e-9)
    # everything kept: nothing is dropped, so only the two mass terms count (p = 0.9995: |0.999 - p| = 0.0005)
    res = oracle.select_topp(cq, ck, None, counts_k, 0.9995)
    np.testing.assert_array_equal(res.col_idx, [0, 1, 2, 3])
    np.testing.assert_allclose(res.margin, [0.0005], rtol=1e-6)
    # an exact tie between last kept and first dropped (equal sizes): margin 0, the lower index is kept
    res = oracle.select_topp(cq, ck, None, np.array([400, 200, 200, 200]), 0.55)
    np.testing.assert_array_equal(res.col_idx, [0, 1])
    np.testing.assert_allclose(res.margin, [0.0], atol=1e-15)


def test_select_probabilities(oracle):
    r = _rng(9)
    cq, ck = r.standard_normal((7, 16)), r.standard_normal((19, 16))
    counts = r.integers(1, 50, size=19)
    res = oracle.select_topp(cq, ck, None, counts, 0.9)
    np.testing.assert_allclose(res.p_est.sum(1), 1.0, rtol=1e-12)
    S = cq @ ck.T / 4.0
    # equal sizes -> plain softmax of S (library)
    eq = oracle.select_topp(cq, ck, None, np.full(19, 3), 0.9)
    np.testing.assert_allclose(eq.p_est, scipy.special.softmax(S, axis=1), rtol=1e-11)
    # general sizes -> softmax of S + ln|K_j|
    np.testing.assert_allclose(res.p_est, scipy.special.softmax(S + np.log(counts)[None], axis=1), rtol=1e-11)
    # a cluster of size |K_j| weighs like |K_j| singleton clusters at the same centroid
    rep = np.repeat(np.arange(19), counts)
    single = oracle.select_topp(cq, ck[rep], None, np.ones(rep.size, dtype=np.int32), 0.9)
    merged = np.zeros_like(res.p_est)
    np.add.at(merged.T, rep, single.p_est.T)
    np.testing.assert_allclose(res.p_est, merged, rtol=1e-10)
    # huge logits do not overflow
    big = oracle.select_topp(cq * 100, ck * 100, None, counts, 0.9)
    assert np.isfinite(big.p_est).all()
    np.testing.assert_allclose(big.p_est.sum(1), 1.0, rtol=1e-12)


def test_select_singletons_reproduce_exact_attention_and_oracle_policy(oracle):
    # every token its own cluster: P' is the true attention matrix and the
    # selection is the oracle policy of Section 3.1 (rank keys by true score)
    r = _rng(10)
    Q, K = r.standard_normal((40, 8)), 1.5 * r.standard_normal((60, 8))
    res = oracle.select_topp(Q, K, np.ones(40, dtype=np.int32), np.ones(60, dtype=np.int32), 0.8)
    P = scipy.special.softmax(Q @ K.T / np.sqrt(8), axis=1)
    np.testing.assert_allclose(res.p_est, P, rtol=1e-11)
    for i in range(40):
        order = np.argsort(-P[i], kind="stable")
        cum = np.cumsum(P[i][order])
        n_keep = int(np.searchsorted(cum, 0.8, side="left")) + 1            # first prefix with mass >= p
        got = res.col_idx[res.row_ptr[i]:res.row_ptr[i + 1]]
        np.testing.assert_array_equal(got, np.sort(order[:n_keep]))


def test_select_minimal_prefix_monotone_and_p_one(oracle):
    r = _rng(11)
    cq, ck = 2 * r.standard_normal((12, 8)), 2 * r.standard_normal((30, 8))
    counts = r.integers(0, 9, size=30)
    counts[[3, 17]] = 0
    prev = None
    for p in (0.3, 0.5, 0.8, 0.9, 0.99, 1.0):
        res = oracle.select_topp(cq, ck, None, counts, p)
        rows = [set(res.col_idx[res.row_ptr[i]:res.row_ptr[i + 1]].tolist()) for i in range(12)]
        for i, s in enumerate(rows):
            assert len(s) >= 1 and 3 not in s and 17 not in s
            cols = np.array(sorted(s))
            np.testing.assert_array_equal(res.col_idx[res.row_ptr[i]:res.row_ptr[i + 1]], cols)   # ascending
            mass = res.p_est[i, cols]
            if p < 1.0:
                assert mass.sum() >= p - 1e-12                        # reaches the target ...
                assert mass.sum() - mass.min() < p                    # ... and no kept element is superfluous
                assert mass.min() >= np.delete(res.p_est[i], cols).max(initial=0.0)   # kept = the largest
            else:
                assert s == set(np.nonzero(counts)[0].tolist())
            if prev is not None:
                assert prev[i] <= s                                    # monotone in p
        prev = rows
    # a query cluster of size 0 gets an empty row
    cnt_q = np.ones(12, dtype=np.int32); cnt_q[4] = 0
    res = oracle.select_topp(cq, ck, cnt_q, counts, 0.9)
    assert res.row_ptr[5] == res.row_ptr[4]


def test_select_ties_go_to_lower_index(oracle):
    cq = np.zeros((1, 2)); ck = np.zeros((4, 2))
    res = oracle.select_topp(cq, ck, None, np.array([2, 2, 2, 2]), 0.5)      # four equal 0.25
    np.testing.assert_array_equal(res.col_idx, [0, 1])


def test_density_counts_selected_pairs(oracle):
    r = _rng(12)
    cq, ck = r.standard_normal((5, 4)), r.standard_normal((8, 4))
    cnt_q, cnt_k = r.integers(1, 20, size=5), r.integers(1, 20, size=8)
    res = oracle.select_topp(cq, ck, cnt_q, cnt_k, 0.6)
    mask = np.zeros((cnt_q.sum(), cnt_k.sum()), dtype=bool)                  # the token-level attention mask
    oq, ok = np.concatenate([[0], np.cumsum(cnt_q)]), np.concatenate([[0], np.cumsum(cnt_k)])
    for i in range(5):
        for j in res.col_idx[res.row_ptr[i]:res.row_ptr[i + 1]]:
            mask[oq[i]:oq[i + 1], ok[j]:ok[j + 1]] = True
    np.testing.assert_allclose(res.density, mask.mean(), rtol=1e-12)


# ------------------------------------------------------------------ sparse attention (Sections 4.1, 4.3)

def _random_partition(r, N, C):
    labels = r.integers(0, C, size=N).astype(np.int32)
    return labels


def test_sparse_attention_with_everything_selected_is_dense_for_any_permutation(oracle):
    # the equivalence proved in Section 4.1
    r = _rng(13)
    N, d, Cq, Ck = 150, 16, 7, 11
    Q, K, V = (r.standard_normal((N, d)).astype(np.float32) for _ in range(3))
    pq = oracle.permute(_random_partition(r, N, Cq), Cq)
    pk = oracle.permute(_random_partition(r, N, Ck), Ck)
    row_ptr = np.arange(Cq + 1, dtype=np.int32) * Ck
    col_idx = np.tile(np.arange(Ck, dtype=np.int32), Cq)
    O, lse = oracle.sparse_attention(Q[pq.perm], K[pk.perm], V[pk.perm], pq.offsets, pk.offsets,
                                     row_ptr, col_idx, perm_q=pq.perm)
    np.testing.assert_allclose(O, _sdpa(Q, K, V), rtol=1e-10, atol=1e-12)
    # without perm_q the rows stay in permuted order
    O2, _ = oracle.sparse_attention(Q[pq.perm], K[pk.perm], V[pk.perm], pq.offsets, pk.offsets, row_ptr, col_idx)
    np.testing.assert_allclose(O2, _sdpa(Q, K, V)[pq.perm], rtol=1e-10, atol=1e-12)


def test_sparse_attention_rows_equal_library_attention_over_selected_keys(oracle):
    r = _rng(14)
    N, d, Cq, Ck = 120, 8, 5, 9
    Q, K, V = (r.standard_normal((N, d)).astype(np.float32) for _ in range(3))
    lq, lk = _random_partition(r, N, Cq), _random_partition(r, N, Ck)
    pq, pk = oracle.permute(lq, Cq), oracle.permute(lk, Ck)
    sel = [np.sort(r.choice(Ck, size=r.integers(1, Ck), replace=False)) for _ in range(Cq)]
    row_ptr = np.concatenate([[0], np.cumsum([len(s) for s in sel])]).astype(np.int32)
    col_idx = np.concatenate(sel).astype(np.int32)
    O, lse = oracle.sparse_attention(Q[pq.perm], K[pk.perm], V[pk.perm], pq.offsets, pk.offsets,
                                     row_ptr, col_idx, perm_q=pq.perm)
    _, lse_dense = oracle.dense_attention(Q, K, V)
    for i in range(Cq):
        rows = np.nonzero(lq == i)[0]
        keys = np.nonzero(np.isin(lk, sel[i]))[0]
        if rows.size == 0:
            continue
        np.testing.assert_allclose(O[rows], _sdpa(Q[rows], K[keys], V[keys]), rtol=1e-10, atol=1e-12)
        assert np.all(lse[rows] <= lse_dense[rows] + 1e-12)
        if len(sel[i]) == Ck:
            np.testing.assert_allclose(lse[rows], lse_dense[rows], rtol=1e-12)
    # a sampled subset of rows gives the same numbers and leaves the rest untouched
    rows = np.array([3, 17, 64, 119], dtype=np.int32)
    Os, _ = oracle.sparse_attention(Q[pq.perm], K[pk.perm], V[pk.perm], pq.offsets, pk.offsets,
                                    row_ptr, col_idx, perm_q=pq.perm, rows=rows)
    np.testing.assert_array_equal(Os[pq.perm[rows]], O[pq.perm[rows]])
    assert np.isnan(np.delete(Os, pq.perm[rows], axis=0)).all()


def test_forward_with_top_p_one_is_dense_attention(oracle):
    r = _rng(15)
    N, d = 256, 16
    Q, K, V = (r.standard_normal((N, d)).astype(np.float32) for _ in range(3))
    res = oracle.forward(Q, K, V, Q[:6], K[:10], 3, 1.0, round_bf16=False)
    np.testing.assert_allclose(res.O, _sdpa(Q, K, V), rtol=1e-10, atol=1e-12)
    assert res.density == pytest.approx(1.0)
    # and with top-p < 1 each row is library attention over its cluster's selected keys
    res = oracle.forward(Q, K, V, Q[:6], K[:10], 3, 0.6, round_bf16=False)
    assert 0.0 < res.density < 1.0
    for i in range(6):
        rows = np.nonzero(res.kq.labels == i)[0]
        cols = res.sel.col_idx[res.sel.row_ptr[i]:res.sel.row_ptr[i + 1]]
        keys = np.nonzero(np.isin(res.kk.labels, cols))[0]
        if rows.size:
            np.testing.assert_allclose(res.O[rows], _sdpa(Q[rows], K[keys], V[keys]), rtol=1e-10, atol=1e-12)


# ------------------------------------------------------------------ accounting (Sections 4.2, 4.3, 5.1)

def test_padding_example_printed_in_the_paper(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "padding_example.txt")) if l.strip() and l[0] != "#"]
    for qr, kr, bm, bn, waste in rows:
        assert oracle.padding_waste(int(qr), int(kr), int(bm), int(bn)) == pytest.approx(float(waste))
    assert oracle.padding_waste(128, 128, 128, 128) == 0.0
    assert oracle.padding_waste(129, 128, 128, 128) == pytest.approx(1 - 129 / 256)


def test_identification_cost_bound_from_the_paper():
    # Eq. 1 costs 2*Cq*Ck*d flops against 4*N*N*d for attention
    for l in open(os.path.join(GOLDEN, "identification_cost.txt")):
        if l.strip() and l[0] != "#":
            N, Cq, Ck, bound = l.split()
            assert 2 * int(Cq) * int(Ck) / (4 * int(N) ** 2) < float(bound)


# ------------------------------------------------------------------ attention recall (Section 3.1)

def _recall_case(seed, N=96, d=16, Cq=5, Ck=7):
    r = _rng(seed)
    Q = r.standard_normal((N, d)).astype(np.float32)
    K = r.standard_normal((N, d)).astype(np.float32)
    lq = r.integers(0, Cq, N).astype(np.int32)
    lk = r.integers(0, Ck, N).astype(np.int32)
    sel = [np.sort(r.choice(Ck, size=int(r.integers(0, Ck + 1)), replace=False)) for _ in range(Cq)]
    row_ptr = np.concatenate([[0], np.cumsum([len(s) for s in sel])]).astype(np.int32)
    col = np.concatenate(sel).astype(np.int32) if row_ptr[-1] else np.zeros(0, np.int32)
    return Q, K, lq, lk, sel, row_ptr, col


def test_recall_matches_library_softmax_brute_force(oracle):
    Q, K, lq, lk, sel, row_ptr, col = _recall_case(50)
    got = oracle.attention_recall(Q, K, lq, lk, 5, 7, row_ptr, col)
    P = scipy.special.softmax((Q.astype(np.float64) @ K.astype(np.float64).T) / np.sqrt(Q.shape[1]), axis=1)
    want = np.array([P[n, np.isin(lk, sel[lq[n]])].sum() for n in range(Q.shape[0])])
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-15)


def test_recall_limits_and_complement(oracle):
    Q, K, lq, lk, sel, row_ptr, col = _recall_case(51)
    Cq, Ck = 5, 7
    full_ptr = (np.arange(Cq + 1) * Ck).astype(np.int32)
    full_col = np.tile(np.arange(Ck, dtype=np.int32), Cq)
    np.testing.assert_allclose(oracle.attention_recall(Q, K, lq, lk, Cq, Ck, full_ptr, full_col), 1.0, rtol=1e-12)
    none = oracle.attention_recall(Q, K, lq, lk, Cq, Ck, np.zeros(Cq + 1, np.int32), np.zeros(0, np.int32))
    assert np.all(none == 0.0)
    comp = [np.setdiff1d(np.arange(Ck), s) for s in sel]
    cptr = np.concatenate([[0], np.cumsum([len(s) for s in comp])]).astype(np.int32)
    ccol = np.concatenate(comp).astype(np.int32)
    a = oracle.attention_recall(Q, K, lq, lk, Cq, Ck, row_ptr, col)
    b = oracle.attention_recall(Q, K, lq, lk, Cq, Ck, cptr, ccol)
    np.testing.assert_allclose(a + b, 1.0, rtol=1e-12)
    assert np.all((a >= 0) & (a <= 1))


def test_recall_is_ratio_of_softmax_denominators(oracle):
    # sum over selected keys of softmax = exp(lse over the selected keys - lse over all keys): ties the recall to
    # the (separately pinned) sparse and dense attention of the oracle
    Q, K, lq, lk, sel, row_ptr, col = _recall_case(52)
    V = _rng(53).standard_normal(Q.shape).astype(np.float32)
    pq, pk = oracle.permute(lq, 5), oracle.permute(lk, 7)
    _, lse_s = oracle.sparse_attention(Q[pq.perm], K[pk.perm], V[pk.perm], pq.offsets, pk.offsets, row_ptr, col,
                                       perm_q=pq.perm)
    _, lse_d = oracle.dense_attention(Q, K, V)
    got = oracle.attention_recall(Q, K, lq, lk, 5, 7, row_ptr, col)
    np.testing.assert_allclose(got, np.exp(lse_s - lse_d), rtol=1e-10, atol=1e-300)


def test_recall_of_the_oracle_policy_reaches_p(oracle):
    # singleton clusters with centroids = tokens: P' is the exact attention (pinned above), so the top-p rule is
    # the oracle policy of Section 3.1 and the recall of its selection is at least p for every query
    r = _rng(54)
    N, d, p = 40, 8, 0.8
    Q = r.standard_normal((N, d)).astype(np.float32)
    K = r.standard_normal((N, d)).astype(np.float32)
    ident = np.arange(N, dtype=np.int32)
    s = oracle.select_topp(Q.astype(np.float64), K.astype(np.float64), np.ones(N, np.int32), np.ones(N, np.int32), p)
    rec = oracle.attention_recall(Q, K, ident, ident, N, N, s.row_ptr, s.col_idx)
    assert np.all(rec >= p - 1e-12)
    P = scipy.special.softmax((Q.astype(np.float64) @ K.astype(np.float64).T) / np.sqrt(d), axis=1)
    for n in range(N):                                       # minimal: dropping the weakest kept key falls below p
        kept = s.col_idx[s.row_ptr[n]: s.row_ptr[n + 1]]
        assert rec[n] - P[n, kept].min() < p


# ------------------------------------------------------------------ k-means++ seeding (Section 4.3)

def test_kmeans_pp_draws_in_proportion_to_squared_distance(oracle):
    # points on a line at 0, 1, 2, 3: after the first centre at 0 the squared distances are 0, 1, 4, 9, so the
    # second centre is token 1, 2, 3 for u in [0, 1/14), [1/14, 5/14), [5/14, 1)
    X = np.array([[0.0], [1.0], [2.0], [3.0]], dtype=np.float32)
    grid = (np.arange(14000) + 0.5) / 14000.0
    picks = np.array([oracle.kmeans_pp(X, 2, np.array([0.0, u]))[0][1] for u in grid])
    assert set(picks) == {1, 2, 3}
    np.testing.assert_array_equal(picks, np.where(grid < 1 / 14, 1, np.where(grid < 5 / 14, 2, 3)))
    # first centre: token floor(u0 * N)
    for u0, want in ((0.0, 0), (0.24, 0), (0.26, 1), (0.99, 3)):
        assert oracle.kmeans_pp(X, 1, np.array([u0]))[0][0] == want


def test_kmeans_pp_worked_example_three_centres(oracle):
    # tokens (0,0), (3,0), (0,4), (3,4); u = (0.3 -> token 1), then D2 = 9, 0, 25, 16 (sum 50):
    # u = 0.5 -> target 25 -> running sums 9, 9, 34 -> token 2; then D2 = 9, 0, 0, 9 (sum 18): u = 0.6 -> 10.8 -> token 3
    X = np.array([[0, 0], [3, 0], [0, 4], [3, 4]], dtype=np.float32)
    picked, centres = oracle.kmeans_pp(X, 3, np.array([0.3, 0.5, 0.6]))
    np.testing.assert_array_equal(picked, [1, 2, 3])
    np.testing.assert_array_equal(centres, X[[1, 2, 3]])


def test_kmeans_pp_invariants(oracle):
    r = _rng(60)
    X = r.standard_normal((500, 12)).astype(np.float32)
    u = r.random(40)
    picked, centres = oracle.kmeans_pp(X, 40, u)
    assert len(set(picked.tolist())) == 40                   # a chosen token has D2 = 0 and is never drawn again
    np.testing.assert_array_equal(centres, X[picked])
    pot = [np.min(((X[:, None, :] - X[picked[:k]][None]) ** 2).sum(-1), axis=1).sum() for k in range(1, 41)]
    assert np.all(np.diff(pot) <= 1e-9)                      # the potential never grows as centres are added
    # every D2 zero (all tokens identical): falls back to token floor(u * N)
    same = np.ones((10, 3), dtype=np.float32)
    np.testing.assert_array_equal(oracle.kmeans_pp(same, 3, np.array([0.05, 0.55, 0.95]))[0], [0, 5, 9])


# ------------------------------------------------------------------ FP8 E4M3 storage of the attention operands

def _e4m3_table():
    """All finite E4M3 values from the format's definition: sign, 4 exponent bits (bias 7), 3 mantissa bits,
    exponent field 0 subnormal, S.1111.111 not a number."""
    vals = {}
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            continue
        v = m * 2.0 ** -9 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
        vals[code] = -v if s else v
    return vals


def test_e4m3_every_code_is_a_fixed_point_and_encodes_to_itself(oracle):
    tab = _e4m3_table()
    assert len(tab) == 254 and max(tab.values()) == 448.0 and tab[0x38] == 1.0 and tab[0x01] == 2.0 ** -9
    codes = np.array(sorted(tab), dtype=np.uint8)
    vals = np.array([tab[c] for c in codes])
    np.testing.assert_array_equal(oracle.round_e4m3(vals), vals)
    got = oracle.encode_e4m3(vals)
    keep = vals != 0                                   # +0 and -0 compare equal as values
    np.testing.assert_array_equal(got[keep], codes[keep])
    assert oracle.encode_e4m3(np.array([0.0]))[0] == 0x00 and oracle.encode_e4m3(np.array([-0.0]))[0] == 0x80


def test_e4m3_rounding_is_nearest_by_brute_force_with_ties_to_even(oracle):
    tab = _e4m3_table()
    pos = np.array(sorted(v for v in tab.values() if v >= 0 and not (v == 0 and np.signbit(v))))
    pos = np.unique(pos)
    r = _rng(40)
    y = np.concatenate([r.uniform(-448, 448, 3000), r.standard_normal(3000) * 0.01, r.standard_normal(3000) * 3,
                        10.0 ** r.uniform(-5, 2.6, 3000)])
    got = oracle.round_e4m3(y)
    # brute force: scan the whole table for the nearest value
    d = np.abs(np.abs(y)[:, None] - pos[None, :])
    near = pos[np.argmin(d, axis=1)]
    not_tie = np.sort(d, axis=1)[:, 0] < np.sort(d, axis=1)[:, 1]
    np.testing.assert_array_equal(np.abs(got[not_tie]), near[not_tie])
    np.testing.assert_array_equal(np.sign(got[got != 0]), np.sign(y[got != 0]))
    # exact midpoints go to the neighbour with the even mantissa (even code)
    mids = (pos[:-1] + pos[1:]) / 2
    gm = oracle.round_e4m3(mids)
    code_of = {v: c for c, v in tab.items() if c < 0x80}
    for lo, hi, g in zip(pos[:-1], pos[1:], gm):
        want = lo if code_of[lo] % 2 == 0 else hi
        assert g == want, (lo, hi, g)
    np.testing.assert_array_equal(oracle.round_e4m3(-mids), -gm)
    # clamping
    np.testing.assert_array_equal(oracle.round_e4m3(np.array([448.1, 1e9, -500.0, 464.0])),
                                  np.array([448.0, 448.0, -448.0, 448.0]))


def test_e4m3_matches_the_library_conversion(oracle):
    r = _rng(41)
    y = np.concatenate([r.uniform(-440, 440, 4000), r.standard_normal(4000), r.standard_normal(2000) * 0.004,
                        np.array([0.0, 2.0 ** -10, 2.0 ** -10 * 1.0001, 3 * 2.0 ** -10, 447.9, -448.0])]).astype(np.float32)
    lib = torch.from_numpy(y).to(torch.float8_e4m3fn)
    np.testing.assert_array_equal(oracle.round_e4m3(y.astype(np.float64)), lib.to(torch.float64).numpy())
    nz = lib.to(torch.float64).numpy() != 0
    np.testing.assert_array_equal(oracle.encode_e4m3(oracle.round_e4m3(y.astype(np.float64)))[nz],
                                  lib.view(torch.uint8).numpy()[nz])


def test_quantize_e4m3_scale_and_error_bound(oracle):
    r = _rng(42)
    X = (r.standard_normal((300, 16)) * np.exp(r.standard_normal((300, 1)))).astype(np.float32)
    codes, dec, sc = oracle.quantize_e4m3(X)
    amax = np.abs(X).max()
    assert sc == np.float32(amax) / np.float32(448.0)
    assert np.abs(dec).max() == 448.0                  # the largest element lands on the largest code
    tab = _e4m3_table()
    np.testing.assert_array_equal(dec, np.array([tab[c] for c in codes.ravel()], dtype=np.float32).reshape(dec.shape))
    # library route: same single-precision scaling, library rounding
    inv = np.float32(448.0) / np.float32(amax)
    lib = torch.from_numpy((X * inv).astype(np.float32)).clamp(-448, 448).to(torch.float8_e4m3fn)
    np.testing.assert_array_equal(dec, lib.to(torch.float32).numpy())
    # relative error of a normal value is at most half a unit in the last of 3 mantissa bits (plus the fp32 product)
    y = X.astype(np.float64) * float(inv)
    normal = np.abs(y) >= 2.0 ** -6
    assert np.all(np.abs(dec[normal] - y[normal]) <= np.abs(y[normal]) * (2.0 ** -4 + 1e-6))
    assert np.all(np.abs(dec[~normal] - y[~normal]) <= 2.0 ** -10 + 1e-9)
    # all-zero input: scale 1, codes 0
    c0, d0, s0 = oracle.quantize_e4m3(np.zeros((4, 8), dtype=np.float32))
    assert s0 == 1.0 and not c0.any() and not d0.any()


# ------------------------------------------------------------------ error budget of rounded probabilities

def _budget_case(oracle, seed, N=90, d=6, Cq=4, Ck=7):
    r = _rng(seed)
    Q, K, V = (r.standard_normal((N, d)).astype(np.float32) for _ in range(3))
    Q *= 2.0
    lq, lk = _random_partition(r, N, Cq), _random_partition(r, N, Ck)
    pq, pk = oracle.permute(lq, Cq), oracle.permute(lk, Ck)
    sel = [np.sort(r.choice(Ck, size=r.integers(1, Ck), replace=False)) for _ in range(Cq)]
    row_ptr = np.concatenate([[0], np.cumsum([len(s) for s in sel])]).astype(np.int32)
    col_idx = np.concatenate(sel).astype(np.int32)
    args = (Q[pq.perm], K[pk.perm], V[pk.perm], pq.offsets, pk.offsets, row_ptr, col_idx)
    return r, Q, K, V, lq, lk, sel, pq, args


def test_rounded_weights_budget_bounds_every_perturbation_and_is_attained(oracle):
    # brute force: library softmax over the selected keys, weights perturbed by relative errors within eps and
    # renormalised by their own sum.  No perturbation may move an output by more than eps / (1 - eps) * dev1, and
    # the adversarial one (every weight pushed towards the side of its value) comes within 1 / (1 + eps) of it.
    r, Q, K, V, lq, lk, sel, pq, args = _budget_case(oracle, 31)
    eps, d = 2.0 ** -4, Q.shape[1]
    dev1, dev2, _, _, _ = oracle.rounded_weights_budget(*args, perm_q=pq.perm)
    O, _ = oracle.sparse_attention(*args, perm_q=pq.perm)
    for n in range(0, Q.shape[0], 7):
        keys = np.nonzero(np.isin(lk, sel[lq[n]]))[0]
        pi = scipy.special.softmax(K[keys].astype(np.float64) @ Q[n].astype(np.float64) / np.sqrt(d))
        v = V[keys].astype(np.float64)
        for trial in range(40):
            e = r.uniform(-eps, eps, size=keys.size)
            w = pi * (1 + e)
            err = (w @ v) / w.sum() - O[n]
            assert np.all(np.abs(err) <= eps / (1 - eps) * dev1[n] + 1e-15)
        for c in range(d):
            w = pi * (1 + eps * np.sign(v[:, c] - O[n, c]))
            err = (w @ v[:, c]) / w.sum() - O[n, c]
            assert err >= eps / (1 + eps) * dev1[n, c] - 1e-15
        # independent uniform errors: the spread is eps / sqrt(3) * sqrt(dev2) to first order in eps
        small = 1e-3
        errs = np.stack([((pi * (1 + e)) @ v) / (pi * (1 + e)).sum() - O[n]
                         for e in r.uniform(-small, small, size=(4000, keys.size))])
        np.testing.assert_allclose(errs.std(axis=0), small / np.sqrt(3) * np.sqrt(dev2[n]), rtol=0.08)


def test_rounded_weights_budget_closed_forms_and_tail(oracle):
    # two keys with probabilities a, 1 - a and values x, y: O = a x + (1 - a) y, so dev1 = 2 a (1 - a) |x - y|
    # and dev2 = (a^2 (1 - a)^2 + (1 - a)^2 a^2) (x - y)^2
    d = 4
    Q = np.zeros((1, d), np.float32); Q[0, 0] = 2.0
    K = np.zeros((2, d), np.float32); K[0, 0] = np.log(3.0)            # scores ln 3 and 0 at scale 1/2 -> a = 3/4
    V = np.array([[1.0, -2.0, 0.5, 0.0], [3.0, 2.0, 0.5, 0.0]], np.float32)
    one = np.array([0, 1], np.int32)
    two = np.array([0, 2], np.int32)
    dev1, dev2, t1, t2, tw = oracle.rounded_weights_budget(Q, K, V, one, two, one, np.zeros(1, np.int32),
                                                           tail_ratio=0.5, tail_abs=0.1)
    a, diff = 0.75, np.abs(V[0] - V[1]).astype(np.float64)         # ln 3 is stored as float32: a = 3/4 to ~1e-8
    np.testing.assert_allclose(dev1[0], 2 * a * (1 - a) * diff, rtol=1e-7)
    np.testing.assert_allclose(dev2[0], 2 * (a * (1 - a)) ** 2 * diff ** 2, rtol=1e-7)
    # the second key has a third of the largest probability: it is the tail at ratio 0.5; its |v - O| = a |x - y|
    # and its absolute weight error is min(1/4, 0.1 * 3/4) = 0.075
    np.testing.assert_allclose(t1[0], 0.075 * a * diff, rtol=1e-7)
    np.testing.assert_allclose(t2[0], (0.075 * a * diff) ** 2, rtol=1e-7)
    np.testing.assert_allclose(tw[0], 0.075, rtol=1e-7)
    # a weight cannot lose more than itself: with a huge absolute figure the error is capped at pi_j = 1/4
    _, _, t1, _, tw = oracle.rounded_weights_budget(Q, K, V, one, two, one, np.zeros(1, np.int32), tail_ratio=0.5,
                                                    tail_abs=10.0)
    np.testing.assert_allclose(tw[0], 0.25, rtol=1e-7)
    np.testing.assert_allclose(t1[0], 0.25 * a * diff, rtol=1e-7)
    # a weighted mean of equal values cannot be wrong whatever the weights: column 2 and 3 have no budget at all
    assert dev1[0, 2] == 0.0 and dev1[0, 3] == 0.0 and t1[0, 3] == 0.0
    # tail sums by brute force against library softmax; sampled rows leave the others untouched
    r, Q, K, V, lq, lk, sel, pq, args = _budget_case(oracle, 32)
    rows = np.array([1, 40, 77], dtype=np.int32)
    _, _, t1, t2, tw = oracle.rounded_weights_budget(*args, perm_q=pq.perm, rows=rows, tail_ratio=0.05, tail_abs=0.01)
    O, _ = oracle.sparse_attention(*args, perm_q=pq.perm)
    for n in pq.perm[rows]:
        keys = np.nonzero(np.isin(lk, sel[lq[n]]))[0]
        pi = scipy.special.softmax(K[keys].astype(np.float64) @ Q[n].astype(np.float64) / np.sqrt(Q.shape[1]))
        tail = pi < 0.05 * pi.max()
        a = np.minimum(pi[tail], 0.01 * pi.max())
        dv = np.abs(V[keys][tail].astype(np.float64) - O[n])
        np.testing.assert_allclose(t1[n], (a[:, None] * dv).sum(axis=0), rtol=1e-10, atol=1e-16)
        np.testing.assert_allclose(t2[n], ((a[:, None] * dv) ** 2).sum(axis=0), rtol=1e-10, atol=1e-18)
        np.testing.assert_allclose(tw[n], a.sum(), rtol=1e-10, atol=1e-16)
        # absolute errors within a_j on the tail keys, relative ones within eps on all: inside the combined bound
        eps = 2.0 ** -4
        dev1 = (pi[:, None] * np.abs(V[keys].astype(np.float64) - O[n])).sum(axis=0)
        for trial in range(20):
            w = pi * (1 + r.uniform(-eps, eps, size=pi.size))
            w[tail] += r.uniform(-1, 1, size=int(tail.sum())) * a
            err = (w @ V[keys].astype(np.float64)) / w.sum() - O[n]
            assert np.all(np.abs(err) <= (eps * dev1 + t1[n]) / (1 - eps - tw[n]) + 1e-15)
    assert np.isnan(np.delete(t1, pq.perm[rows], axis=0)).all()
