"""Pins for the oracle's SVD-based start (section "Experiments", algorithmic parameters, option 2 of arxiv
2202.09512; NNDSVD of Boutsidis and Gallopoulos 2008): closed forms for a rank-one tensor and for planted
columns with disjoint supports, the split of a mixed-sign triplet recomputed from an independent
eigen-decomposition with explicit loops, and the invariances that the construction must have."""
import numpy as np

from oracle import mu, nndsvd, perturb


def test_rank_one_closed_form():
    """X_t = c_t x x^T: M = x [c_1 x^T ... c_m x^T  c_1 x^T ...], one singular value ||x||^2 sqrt(2 sum c_t^2)
    with u = x / ||x||, so a_0 = sqrt(s_0) x / ||x||.  (One unfolding alone would lose the factor sqrt 2.)"""
    rng = np.random.default_rng(0)
    x = rng.random(7) + 0.1
    c = np.array([0.5, 2.0, 1.5])
    Xs = [ct * np.outer(x, x) for ct in c]
    U, s, V = nndsvd.leading_triplets(nndsvd.concat_unfoldings(Xs), 1)
    s0 = (x @ x) * np.sqrt(2.0 * (c ** 2).sum())
    assert abs(s[0] - s0) <= 1e-12 * s0
    A = nndsvd.nndsvd_left(U, s, V)
    assert np.allclose(A[:, 0], np.sqrt(s0) * x / np.linalg.norm(x), rtol=1e-12)


def test_disjoint_columns_closed_form():
    """A with disjoint supports and X_t = A D_t A^T, D_t diagonal: M M^T = A (2 sum_t D_t A^T A D_t) A^T, so the
    left singular vectors are the normalised columns, s_j = ||a_j||^2 sqrt(2 sum_t d_tj^2), and (all parts
    non-negative) column j of the start is sqrt(s_j) a_j / ||a_j||, in the order of decreasing s_j."""
    rng = np.random.default_rng(1)
    n, k, m = 12, 3, 2
    A = np.zeros((n, k))
    for j in range(k):
        A[4 * j:4 * j + 4, j] = rng.random(4) + 0.2
    D = np.array([[3.0, 1.0, 0.3], [2.0, 1.5, 0.2]])
    Xs = [A @ np.diag(D[t]) @ A.T for t in range(m)]
    s_want = (A * A).sum(axis=0) * np.sqrt(2.0 * (D ** 2).sum(axis=0))
    order = np.argsort(-s_want)
    R0 = perturb.init_R(0, 0, m, k)
    A0, R = nndsvd.start(Xs, k, R0, r_iters=2000, floor_rel=0.0)
    for col, j in enumerate(order):
        assert np.allclose(A0[:, col], np.sqrt(s_want[j]) * A[:, j] / np.linalg.norm(A[:, j]), rtol=1e-9, atol=1e-12)
    # the start spans the planted model exactly, so the R-only updates drive the error of Eq. 1 towards zero
    assert mu.relative_error(np.stack(Xs), A0, R) < 1e-3
    errs = [mu.relative_error(np.stack(Xs), *nndsvd.start(Xs, k, R0, r_iters=it, floor_rel=0.0)) for it in (0, 1, 5, 50)]
    assert all(b <= a * (1 + 1e-12) for a, b in zip(errs, errs[1:]))


def test_mixed_sign_split_against_explicit_loops():
    """A random non-negative tensor: columns j >= 1 have mixed signs.  The triplets come from the symmetric
    eigenproblem of M M^T (another routine than the SVD), the right vectors from v = M^T u / s, the positive and
    negative parts and their norms from plain loops."""
    rng = np.random.default_rng(2)
    n, m, k = 6, 2, 4
    Xs = [rng.random((n, n)) for _ in range(m)]
    M = nndsvd.concat_unfoldings(Xs)
    assert M.shape == (n, 2 * n * m)
    assert np.array_equal(M[:, :n], Xs[0]) and np.array_equal(M[:, 2 * n:3 * n], Xs[0].T)
    lam, E = np.linalg.eigh(M @ M.T)
    idx = np.argsort(-lam)[:k]
    want = np.zeros((n, k))
    for col, e in enumerate(idx):
        s = np.sqrt(lam[e])
        u = [E[i, e] for i in range(n)]
        v = [sum(M[i, c] * u[i] for i in range(n)) / s for c in range(M.shape[1])]
        if col == 0:
            for i in range(n):
                want[i, 0] = np.sqrt(s) * abs(u[i])
            continue
        up = sum(a * a for a in u if a > 0) ** 0.5
        un = sum(a * a for a in u if a < 0) ** 0.5
        vp = sum(a * a for a in v if a > 0) ** 0.5
        vn = sum(a * a for a in v if a < 0) ** 0.5
        for i in range(n):
            if up * vp > un * vn:
                want[i, col] = np.sqrt(s * up * vp) * max(u[i], 0.0) / up
            else:
                want[i, col] = np.sqrt(s * un * vn) * max(-u[i], 0.0) / un
    U, s, V = nndsvd.leading_triplets(M, k)
    got = nndsvd.nndsvd_left(U, s, V)
    assert np.allclose(got, want, rtol=1e-9, atol=1e-12)
    # the sign a library gives a triplet must not matter
    flip = np.array([1.0, -1.0, 1.0, -1.0])
    assert np.allclose(nndsvd.nndsvd_left(U * flip, s, V * flip), got, rtol=1e-12, atol=1e-15)


def test_invariances_and_floor():
    rng = np.random.default_rng(3)
    n, m, k = 9, 3, 3
    Xs = [rng.random((n, n)) ** 2 for _ in range(m)]
    R0 = perturb.init_R(1, 0, m, k)
    A, R = nndsvd.start(Xs, k, R0)
    assert A.min() > 0 and R.min() >= 0
    # both unfoldings are in M: transposing every slice changes nothing in A
    A_t, _ = nndsvd.start([Xt.T for Xt in Xs], k, R0)
    assert np.allclose(A_t, A, rtol=1e-9)
    # relabelling the entities permutes the rows; scaling X by c scales A by sqrt(c)
    p = rng.permutation(n)
    A_p, _ = nndsvd.start([Xt[np.ix_(p, p)] for Xt in Xs], k, R0)
    assert np.allclose(A_p, A[p], rtol=1e-9)
    A_c, _ = nndsvd.start([4.0 * Xt for Xt in Xs], k, R0)
    assert np.allclose(A_c, 2.0 * A, rtol=1e-9)
    # column norms: ||a_j||^2 = s_j ||x+-|| ||y+-|| <= s_j before the floor
    U, s, V = nndsvd.leading_triplets(nndsvd.concat_unfoldings(Xs), k)
    A_raw = nndsvd.nndsvd_left(U, s, V)
    assert np.all((A_raw * A_raw).sum(axis=0) <= s * (1 + 1e-12))
    assert np.allclose((A_raw[:, 0] ** 2).sum(), s[0])
    # the floor: a hundredth of the mean of the unfloored factor, applied to the entries below it only
    assert (A_raw == 0).any() and np.array_equal(A, np.maximum(A_raw, 0.01 * A_raw.mean()))
    # sparse slices give what their dense copies give
    import scipy.sparse as sp
    Xsp = [sp.csr_matrix(np.where(Xt > 0.3, Xt, 0.0)) for Xt in Xs]
    A_s, R_s = nndsvd.start(Xsp, k, R0)
    A_d, R_d = nndsvd.start([Xt.toarray() for Xt in Xsp], k, R0)
    assert np.array_equal(A_s, A_d) and np.array_equal(R_s, R_d)
