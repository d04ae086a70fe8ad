"""Pins for the oracle's model-selection part (Alg. 1, 5, 6): assignment against enumeration,
silhouettes against scikit-learn's routine (named by the paper as a dependency, called as a black
box), regression against non-negative least squares, medians, and the qualitative behaviour the
paper reports on planted data (silhouette near 1 and error low at the planted rank, silhouette
dropping beyond it)."""
import numpy as np
import pytest
from scipy.optimize import nnls
from sklearn.metrics import silhouette_samples

from oracle import mu, perturb, select
from synth import generators as gen


def test_assignment_matches_enumeration():
    rng = np.random.default_rng(0)
    for k in (1, 2, 3, 5, 7):
        for _ in range(5):
            G = rng.random((k, k))
            pi = select.lsa_max(G)
            pb, best, second = select.lsa_max_bruteforce(G)
            assert abs(G[np.arange(k), pi].sum() - best) < 1e-12
            if best - second > 1e-9:
                assert np.array_equal(pi, pb)


def test_cluster_recovers_planted_permutations():
    rng = np.random.default_rng(1)
    n, k, q = 60, 5, 7
    base = rng.random((n, k))
    perms = [rng.permutation(k) for _ in range(q)]
    perms[0] = np.arange(k)                        # the centroid starts from member 0
    A_ens = np.stack([base[:, p] + 1e-3 * rng.random((n, k)) for p in perms])
    R_ens = rng.random((q, 2, k, k))
    perm, A_perm, R_perm, med, rounds = select.custom_cluster(A_ens, R_ens)
    for r in range(q):
        # column s of member r is base[:, perms[r][s]]; cluster c must pick the s with perms[r][s] == c
        assert np.array_equal(perms[r][perm[r]], np.arange(k))
        assert np.array_equal(A_perm[r], A_ens[r][:, perm[r]])
        assert np.array_equal(R_perm[r], R_ens[r][:, perm[r]][:, :, perm[r]])
    assert np.abs(med - base).max() < 2e-3 and rounds <= 3
    # exactly one column of every member per cluster
    assert all(sorted(perm[r]) == list(range(k)) for r in range(q))


def test_assignment_uses_cosine_similarity():
    """The first round's assignment ignores the scale of every column (cosine similarity); later
    rounds depend on the medians, which are only invariant under one common factor."""
    rng = np.random.default_rng(2)
    A_ens = rng.random((4, 30, 3))
    scales = rng.random((4, 1, 3)) * 10 + 0.1
    p1 = select.custom_cluster(A_ens, max_rounds=1)[0]
    p2 = select.custom_cluster(A_ens * scales, max_rounds=1)[0]
    assert np.array_equal(p1, p2)
    assert np.array_equal(select.custom_cluster(A_ens)[0], select.custom_cluster(7.0 * A_ens)[0])


def test_median_convention():
    odd = np.array([[[1.0]], [[5.0]], [[2.0]]])
    even = np.array([[[1.0]], [[5.0]], [[2.0]], [[4.0]]])
    assert select.custom_cluster(odd)[3][0, 0] == 2.0
    assert select.custom_cluster(even)[3][0, 0] == 3.0          # mean of the two middle values


def test_silhouettes_match_sklearn_cosine():
    rng = np.random.default_rng(3)
    for (q, n, k) in [(5, 40, 3), (8, 25, 6), (2, 10, 2)]:
        A = rng.random((q, n, k))
        sil = select.silhouettes(A)
        pts = A.transpose(0, 2, 1).reshape(q * k, n)
        labels = np.tile(np.arange(k), q)
        ref = silhouette_samples(pts, labels, metric="cosine").reshape(q, k)
        np.testing.assert_allclose(sil, ref, atol=1e-12)
        assert np.all(sil >= -1) and np.all(sil <= 1)


def test_silhouette_special_cases():
    n, k, q = 12, 3, 4
    E = np.zeros((n, k))
    E[0:4, 0] = E[4:8, 1] = E[8:12, 2] = 1.0
    ident = np.stack([E] * q)                                   # identical members, orthogonal columns
    assert np.allclose(select.silhouettes(ident), 1.0)
    s_min, s_avg = select.cluster_stability(ident)
    assert s_min == pytest.approx(1.0) and s_avg == pytest.approx(1.0)
    same = np.stack([np.ones((n, 2))] * q)                      # two identical clusters
    assert np.allclose(select.silhouettes(same), 0.0)
    assert np.all(select.silhouettes(ident[:1]) == 0)           # q = 1


def test_regression_reaches_nnls_optimum():
    rng = np.random.default_rng(4)
    n, k, m = 15, 3, 2
    A = rng.random((n, k))
    X = np.einsum("ia,tab,jb->tij", A, rng.random((m, k, k)), A) + 0.05 * rng.random((m, n, n))
    R = select.regression(X, A, np.ones((m, k, k)), iters=20000, eps=0.0)
    K = np.kron(A, A)                                           # vec(A R A^T) = (A kron A) vec(R), row-major
    for t in range(m):
        want, _ = nnls(K, X[t].reshape(-1))
        np.testing.assert_allclose(R[t].reshape(-1), want, atol=2e-5)


def test_choose_k_rules():
    ks = [2, 3, 4, 5]
    assert select.choose_k(ks, [0.9, 0.95, 0.2, 0.1], [0.5, 0.1, 0.09, 0.08]) == 3
    assert select.choose_k(ks, [1.0, 1.0, 0.0, 0.0], [0.1, 0.1, 0.1, 0.1]) == 3      # tie -> larger k
    assert select.choose_k(ks, [0.9, 0.95, 0.8, 0.1], [0.5, 0.1, 0.1, 0.1], rule="threshold") == 4


def test_planted_rank_is_selected_on_community_data():
    """Community-structured tensor with planted rank 3: stable clusters and low error at k = 3,
    unstable clusters beyond, high error below (sections "Generic RESCALk" and "Synthetic Data")."""
    X, _, _ = gen.dense_community(n=72, m=3, rank=3, noise=0.01, seed=7)
    out = select.select_k(X, 2, 5, q=6, delta=0.03, iters=300, seed=2, regress_iters=200)
    s, e = dict(zip(out["ks"], out["s_min"])), dict(zip(out["ks"], out["err"]))
    assert out["k_opt"] == 3
    assert s[3] > 0.9 and e[3] < 0.05
    assert e[2] > 2 * e[3]
    assert s[4] < s[3] - 0.2 and s[5] < s[3] - 0.2
    assert all(-1 <= v <= 1 for v in out["s_min"] + out["s_avg"])
