"""Pins for the oracle's multiplicative updates (Eq. 2 / Alg. 3), independent of the oracle itself:
explicit index sums of Eq. 2 on tiny tensors, the planted factors as a fixed point, the k = 1 closed
form, the symmetries of the model, non-negativity and the monotone objective of Eq. 1."""
import numpy as np
import pytest

from oracle import mu, perturb
from synth import generators as gen


def _brute_step(X, A, R, eps):
    """Eq. 2 as explicit index sums (pure Python loops; Gauss-Seidel order of Alg. 3)."""
    m, n, k = len(X), len(A), len(A[0])
    G = [[sum(A[i][a] * A[i][b] for i in range(n)) for b in range(k)] for a in range(k)]
    Rn = [[[0.0] * k for _ in range(k)] for _ in range(m)]
    for t in range(m):
        for a in range(k):
            for b in range(k):
                num = sum(A[i][a] * X[t][i][j] * A[j][b] for i in range(n) for j in range(n))
                den = sum(G[a][c] * R[t][c][d] * G[d][b] for c in range(k) for d in range(k)) + eps
                Rn[t][a][b] = R[t][a][b] * num / den
    An = [[0.0] * k for _ in range(n)]
    for i in range(n):
        for s in range(k):
            num = 0.0
            for t in range(m):
                for j in range(n):
                    for b in range(k):
                        num += X[t][i][j] * A[j][b] * Rn[t][s][b]        # X_t A R_t^T
                        num += X[t][j][i] * A[j][b] * Rn[t][b][s]        # X_t^T A R_t
            den = 0.0
            for t in range(m):
                for a in range(k):
                    for c in range(k):
                        for d in range(k):
                            # A (R_t G R_t^T + R_t^T G R_t)
                            den += A[i][a] * (Rn[t][a][c] * G[c][d] * Rn[t][s][d] + Rn[t][c][a] * G[c][d] * Rn[t][d][s])
            An[i][s] = A[i][s] * num / (den + eps)
    return np.array(An), np.array(Rn)


@pytest.mark.parametrize("n,m,k", [(4, 1, 1), (5, 2, 2), (6, 3, 3)])
def test_matches_explicit_index_sums(n, m, k):
    rng = np.random.default_rng(n * 100 + k)
    X = rng.random((m, n, n))
    A, R = rng.random((n, k)) + 0.1, rng.random((m, k, k)) + 0.1
    A1, R1 = mu.mu_iteration(X, A, R, 1e-16)
    Ab, Rb = _brute_step(X.tolist(), A.tolist(), R.tolist(), 1e-16)
    np.testing.assert_allclose(R1, Rb, rtol=1e-12)
    np.testing.assert_allclose(A1, Ab, rtol=1e-12)


def test_planted_factors_are_a_fixed_point():
    rng = np.random.default_rng(0)
    A, R = rng.random((40, 4)), rng.random((3, 4, 4))
    X = np.einsum("ia,tab,jb->tij", A, R, A)
    A1, R1 = mu.mu_iteration(X, A, R, 0.0)
    np.testing.assert_allclose(A1, A, rtol=1e-12)
    np.testing.assert_allclose(R1, R, rtol=1e-12)


def test_rank_one_closed_form():
    """k = 1: one step gives R_t = a^T X_t a / (a^T a)^2 whatever R_t was (the least-squares value)."""
    rng = np.random.default_rng(1)
    X = rng.random((3, 9, 9))
    a = rng.random((9, 1)) + 0.1
    _, R1 = mu.mu_iteration(X, a, rng.random((3, 1, 1)) + 0.5, 0.0)
    want = np.array([(a.T @ X[t] @ a)[0, 0] / (a.T @ a)[0, 0] ** 2 for t in range(3)])
    np.testing.assert_allclose(R1[:, 0, 0], want, rtol=1e-13)


def test_symmetries():
    rng = np.random.default_rng(2)
    n, m, k = 12, 3, 3
    X = rng.random((m, n, n))
    A, R = rng.random((n, k)) + 0.1, rng.random((m, k, k)) + 0.1
    A1, R1 = mu.mu_iteration(X, A, R)
    # column permutation of the start permutes the result
    p = np.array([2, 0, 1])
    A2, R2 = mu.mu_iteration(X, A[:, p], R[:, p][:, :, p])
    np.testing.assert_allclose(A2, A1[:, p], rtol=1e-12)
    np.testing.assert_allclose(R2, R1[:, p][:, :, p], rtol=1e-12)
    # relabelling the entities
    e = rng.permutation(n)
    A3, R3 = mu.mu_iteration(X[:, e][:, :, e], A[e], R)
    np.testing.assert_allclose(A3, A1[e], rtol=1e-12)
    np.testing.assert_allclose(R3, R1, rtol=1e-12)
    # transposing every slice transposes every core slice and keeps A
    A4, R4 = mu.mu_iteration(X.transpose(0, 2, 1), A, R.transpose(0, 2, 1))
    np.testing.assert_allclose(A4, A1, rtol=1e-12)
    np.testing.assert_allclose(R4, R1.transpose(0, 2, 1), rtol=1e-12)
    # scaling X and R0 scales R and keeps A
    A5, R5 = mu.mu_iteration(3.0 * X, A, 3.0 * R, 0.0)
    A1z, R1z = mu.mu_iteration(X, A, R, 0.0)
    np.testing.assert_allclose(A5, A1z, rtol=1e-12)
    np.testing.assert_allclose(R5, 3.0 * R1z, rtol=1e-12)
    # an asymmetric X must give asymmetric R (catches a dropped transpose)
    assert np.abs(R1 - R1.transpose(0, 2, 1)).max() > 1e-3


def test_nonnegative_and_objective_monotone_dense_tiny():
    X, _, _ = gen.dense_tiny()
    for k in (2, 3, 5):
        A0, R0 = perturb.init_A(0, 1, 64, k), perturb.init_R(0, 1, 4, k)
        A, R, objs = mu.fit(X, A0, R0, 60, trace=True)
        assert A.min() >= 0 and R.min() >= 0
        objs = np.array([mu.objective(X, A0, R0)] + objs)
        assert np.all(np.diff(objs) <= 1e-9 * objs[:-1]), "objective increased"


def test_recovers_planted_model_noise_free():
    """At the planted rank the fit of a noise-free tensor keeps improving towards zero error."""
    X, _, _ = gen.dense_tiny()
    A0, R0 = perturb.init_A(0, 0, 64, 3), perturb.init_R(0, 0, 4, 3)
    A, R = mu.fit(X, A0, R0, 200)
    e200 = mu.relative_error(X, A, R)
    A, R = mu.fit(X, A, R, 1800)
    e2000 = mu.relative_error(X, A, R)
    assert e200 < 0.1 and e2000 < 0.02 and e2000 < 0.5 * e200


def test_recovers_community_columns():
    """Near-separable planted A (community generator): matched-column cosine close to 1."""
    X, A_true, _ = gen.dense_community(n=96, m=3, rank=3, noise=0.01, seed=3)
    A0, R0 = perturb.init_A(1, 0, 96, 3), perturb.init_R(1, 0, 3, 3)
    A, R = mu.fit(X, A0, R0, 500)
    An, _ = mu.normalise(A, R)
    At = A_true / np.linalg.norm(A_true, axis=0)
    C = At.T @ An
    assert C.max(axis=1).min() > 0.95
    assert mu.relative_error(X, A, R) < 0.05


def test_normalise_keeps_model_and_gives_unit_columns():
    rng = np.random.default_rng(4)
    A, R = rng.random((20, 3)), rng.random((2, 3, 3))
    An, Rn = mu.normalise(A, R)
    np.testing.assert_allclose(np.linalg.norm(An, axis=0), 1.0, rtol=1e-14)
    np.testing.assert_allclose(np.einsum("ia,tab,jb->tij", An, Rn, An), np.einsum("ia,tab,jb->tij", A, R, A), rtol=1e-12)
    A[:, 1] = 0
    An, Rn = mu.normalise(A, R)
    assert np.all(An[:, 1] == 0) and np.array_equal(Rn[:, 1, 1], R[:, 1, 1])


def test_objective_forms_and_sparse_path_agree():
    S, _, _ = gen.sparse_community(n=300, m=2, nnz_per_slice=3000, rank=3, communities=3, seed=5)
    Xd = S.to_dense()
    A0, R0 = perturb.init_A(2, 0, 300, 4), perturb.init_R(2, 0, 2, 4)
    f_direct = mu.objective(Xd, A0, R0)
    f_expand = mu.objective(S.to_scipy(), A0, R0)
    assert f_direct >= 0 and abs(f_direct - f_expand) < 1e-9 * f_direct
    a1, r1 = mu.mu_iteration(S.to_scipy(), A0, R0)
    a2, r2 = mu.mu_iteration(Xd, A0, R0)
    np.testing.assert_allclose(a1, a2, rtol=1e-12)
    np.testing.assert_allclose(r1, r2, rtol=1e-12)
    assert abs(mu.norm_sq(S.to_scipy()) - float((Xd.astype(np.float64) ** 2).sum())) < 1e-9


def test_zero_entries_stay_zero_and_guard_prevents_nan():
    rng = np.random.default_rng(6)
    X = rng.random((2, 8, 8))
    A, R = rng.random((8, 2)), rng.random((2, 2, 2))
    A[3, 1] = 0.0
    R[0, 0, 1] = 0.0
    A1, R1 = mu.mu_iteration(X, A, R)
    assert A1[3, 1] == 0 and R1[0, 0, 1] == 0
    A1, R1 = mu.mu_iteration(np.zeros_like(X), A, R)
    assert np.all(np.isfinite(A1)) and np.all(A1 == 0) and np.all(R1 == 0)


def test_fit_until_threshold_bookkeeping():
    """The threshold rule of section "Distributed RESCAL" against a scan of the plain per-iteration trace:
    which factors a check looks at, which iteration is the last, and the two ends of the threshold range."""
    X, _, _ = gen.dense_tiny()
    k, q, iters, every = 3, 3, 40, 4
    Xq = [np.stack(list(perturb.perturb_dense(X, 5, r, 0.03))) for r in range(q)]
    A0 = [perturb.init_A(5, r, 64, k) for r in range(q)]
    R0 = [perturb.init_R(5, r, 4, k) for r in range(q)]
    # the plain trace: f after 0, 1, ..., iters iterations, per member
    full = []
    for r in range(q):
        _, _, objs = mu.fit(Xq[r], A0[r], R0[r], iters, trace=True)
        full.append([mu.objective(Xq[r], A0[r], R0[r])] + objs)
    full = np.array(full)                                    # [q][iters + 1]
    worst = full.max(axis=0)                                 # the member that is furthest from the threshold
    assert np.all(np.diff(worst) < 0)
    # a threshold that the ensemble crosses between two checks, away from both
    tau = 0.5 * (worst[17] + worst[18])
    As, Rs, done, trace = mu.fit_until(Xq, A0, R0, iters, tau, every)
    # checks look at the factors after l - 1 iterations, l = 4, 8, ...: the first of them below tau is l - 1 = 19
    assert done == 20 and len(trace) == 5
    for c, row in enumerate(trace):
        assert np.allclose(row, full[:, every * (c + 1) - 1], rtol=1e-12)
    for r in range(q):
        A_ref, R_ref = mu.fit(Xq[r], A0[r], R0[r], done)
        assert np.array_equal(As[r], A_ref) and np.array_equal(Rs[r], R_ref)
    # never reached: all iterations, a check at every multiple; always reached: stops with the first check
    _, _, done0, trace0 = mu.fit_until(Xq, A0, R0, 10, 0.0, 3)
    assert done0 == 10 and np.allclose(trace0, full[:, [2, 5, 8]].T, rtol=1e-12)
    assert mu.fit_until(Xq, A0, R0, 10, np.inf, 3)[2] == 3
    # one member above the threshold keeps the whole ensemble going
    # (at the check of iteration 8 only the worst member is still above tau1; at the next check none is)
    tau1 = 0.5 * (np.sort(full[:, 7])[-1] + np.sort(full[:, 7])[-2])
    assert np.sort(full[:, 11])[-1] < tau1
    assert mu.fit_until(Xq, A0, R0, iters, tau1, every)[2] == 12
