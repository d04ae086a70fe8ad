"""GPU parity of the SVD-based start (section "Experiments", algorithmic parameters, option 2 of arxiv 2202.09512)
against the CPU oracle, through the C ABI.

Bar.  A is built from singular vectors, and an eigenvector of B = M M^T computed in fp32 moves by about
(rounding of B) / (gap to the neighbouring eigenvalues): with eps = 2^-24 the test allows
tol_A = 1e-6 + 2 eps lambda_0 / min_j gap_j per member (relative Frobenius error of A), computed from the oracle's own
spectrum, ten times that for R (ten R-only updates on top of A), and 1e-5 relative for the singular values.
Columns whose singular values are not separated (k above the planted rank: noise directions) are not comparable and
are checked by properties only."""
import numpy as np
import pytest
import torch

from oracle import mu, nndsvd, perturb, select
from synth import generators as gen
from tests.gpu_helpers import rel_fro

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
EPS = 2.0 ** -24


def _graded_tensor(n, m, k, seed):
    """Planted community columns with geometrically graded weights (separated singular values), 1 % noise."""
    rng = np.random.default_rng(seed)
    A = rng.random((n, k)) * 0.05
    A[np.arange(n), (np.arange(n) * k) // n] = 0.5 + 0.5 * rng.random(n)
    A *= 0.93 ** np.arange(k)[None, :]
    X = np.empty((m, n, n), dtype=np.float32)
    for t in range(m):
        R = np.eye(k) + 0.05 * rng.random((k, k))
        X0 = A @ R @ A.T
        X[t] = np.maximum(0.0, X0 * (1.0 + 0.01 * rng.standard_normal((n, n))))
    return X


def _check_start(lib, dx, X_host, k, q, seed, svd_iters, r_iters=10, floor_rel=0.01, csc_build=True):
    dense = isinstance(X_host, np.ndarray)
    m = X_host.shape[0] if dense else X_host.m
    Xq = select.perturbed_members(X_host if dense else X_host.to_scipy(), seed, q, 0.03)
    h = lib.nnrescal_init(dx, k=k, q=q, delta=0.03, seed=seed, csc_build=csc_build)
    lib.nnrescal_fit(h, 2)                                    # the start replaces whatever the handle holds
    sig = lib.nnrescal_start_nndsvd(h, svd_iters, r_iters, floor_rel)
    A, R = lib.nnrescal_get_factors(h)
    A, R = A.cpu().numpy(), R.cpu().numpy()
    assert np.all(np.isfinite(A)) and np.all(np.isfinite(R)) and A.min() > 0 and R.min() >= 0
    for r in range(q):
        Ao, Ro = nndsvd.start(Xq[r], k, perturb.init_R(seed, r, m, k), r_iters, floor_rel)
        s = np.linalg.svd(nndsvd.concat_unfoldings(Xq[r]), compute_uv=False)[:k + 1]
        lam = s ** 2
        gap = np.abs(np.diff(lam))                            # gap[j] = lam_j - lam_{j+1}, j = 0..k-1
        gap_min = min(gap[:k].min(), gap[:max(k - 1, 1)].min())
        tol = 1e-6 + 2 * EPS * lam[0] / gap_min
        assert tol < 2.5e-4, "the test data must have separated singular values"
        assert np.max(np.abs(np.array(sig[r]) - s[:k]) / s[:k]) <= 1e-5
        ea, er = rel_fro(A[r], Ao), rel_fro(R[r], Ro)
        assert ea <= tol and er <= 10 * tol, f"member {r}: relA={ea:.2e} relR={er:.2e} tol={tol:.2e}"
    return h, Xq, A, R


@pytest.mark.parametrize("n,m,k,q", [(200, 3, 4, 3), (97, 2, 1, 2), (150, 2, 9, 9), (130, 2, 17, 5)])
def test_start_dense_matches_oracle(lib, n, m, k, q):
    X = _graded_tensor(n, m, k, n + k)
    h, _, _, _ = _check_start(lib, lib.DenseX(torch.from_numpy(X).to(DEV).contiguous()), X, k, q, 2, 40)
    lib.nnrescal_destroy(h)


@pytest.mark.parametrize("with_csc,csc_build", [(True, True), (False, True), (False, False)])
def test_start_sparse_matches_oracle(lib, with_csc, csc_build):
    """CSC given, CSC built by the library from the CSR slices, and CSR slices alone (scatter form of X_t^T A)."""
    S, _, _ = gen.sparse_community(n=300, m=2, nnz_per_slice=12000, rank=3, communities=3, seed=4)
    h, _, _, _ = _check_start(lib, lib.SparseX.from_host(S, DEV, with_csc=with_csc), S, 3, 2, 1, 30, csc_build=csc_build)
    lib.nnrescal_destroy(h)


def test_start_then_fit_and_rank_above_planted(lib):
    """From the start the fit goes on as from any given factors (one iteration against the oracle's), reaches a
    lower error than the random start in the same number of iterations (the reason the paper gives for it), and a
    rank above the planted one (unseparated trailing singular values) still gives finite positive factors whose
    leading columns agree with the oracle."""
    X, _, _ = gen.dense_community(n=160, m=3, rank=4, noise=0.01, seed=1)
    dx = lib.DenseX(torch.from_numpy(X).to(DEV).contiguous())
    h, Xq, A, R = _check_start(lib, dx, X, 4, 3, 2, 15)
    lib.nnrescal_fit(h, 1)
    A1, R1 = lib.nnrescal_get_factors(h)
    for r in range(3):
        Ao, Ro = mu.mu_iteration(Xq[r], A[r].astype(np.float64), R[r].astype(np.float64))
        assert rel_fro(A1[r].cpu().numpy(), Ao) <= 1e-5 and rel_fro(R1[r].cpu().numpy(), Ro) <= 1e-5
    obj_svd = lib.nnrescal_fit(h, 19, objective=True)
    lib.nnrescal_destroy(h)
    h = lib.nnrescal_init(dx, k=4, q=3, delta=0.03, seed=2)
    obj_rand = lib.nnrescal_fit(h, 20, objective=True)
    lib.nnrescal_destroy(h)
    assert all(a < 0.5 * b for a, b in zip(obj_svd, obj_rand))
    # k = 7 > 4: the columns of the four separated singular values agree, the others are only checked for sanity
    h = lib.nnrescal_init(dx, k=7, q=2, delta=0.03, seed=3)
    sig = lib.nnrescal_start_nndsvd(h, 40, 5, 0.01)
    A7, R7 = lib.nnrescal_get_factors(h)
    lib.nnrescal_destroy(h)
    A7, R7 = A7.cpu().numpy(), R7.cpu().numpy()
    assert np.all(np.isfinite(A7)) and A7.min() > 0 and np.all(np.isfinite(R7)) and R7.min() >= 0
    Xq7 = select.perturbed_members(X, 3, 2, 0.03)
    for r in range(2):
        Ao, _ = nndsvd.start(Xq7[r], 7, perturb.init_R(3, r, 3, 7), 5, 0.01)
        # the floor depends on all columns' mean, so compare above it only
        big = Ao[:, :4] > 10 * Ao.min()
        assert np.max(np.abs(A7[r][:, :4] - Ao[:, :4])[big] / Ao[:, :4][big]) <= 1e-3
        assert all(sig[r][j] >= sig[r][j + 1] for j in range(6))


def test_start_through_init_and_model_selection(lib):
    """start = 1 in the parameters: nnrescal_init makes the same factors as the explicit call, and Alg. 1 run
    with that start for every fit (section "RESCAL with Automatic Model Selection": random or NNDSVD
    initialisation) selects the planted rank, with the oracle's curves up to that rank."""
    from tests.test_gpu_select import _check_select
    X, _, _ = gen.dense_community(n=72, m=3, rank=3, noise=0.01, seed=7)
    dx = lib.DenseX(torch.from_numpy(X).to(DEV).contiguous())
    h = lib.nnrescal_init(dx, k=3, q=4, delta=0.03, seed=2, start=(20, 10, 0.01))
    A1, R1 = lib.nnrescal_get_factors(h)
    lib.nnrescal_destroy(h)
    h = lib.nnrescal_init(dx, k=3, q=4, delta=0.03, seed=2)
    lib.nnrescal_start_nndsvd(h, 20, 10, 0.01)
    A2, R2 = lib.nnrescal_get_factors(h)
    lib.nnrescal_destroy(h)
    # (not bit for bit: partial sums are added to memory in an order that varies from run to run)
    assert rel_fro(A1.cpu().numpy(), A2.cpu().numpy()) <= 1e-6 and rel_fro(R1.cpu().numpy(), R2.cpu().numpy()) <= 1e-5
    got, want = _check_select(lib, dx, X, 2, 5, 6, 0.03, 100, 2, s_tol=2e-2, e_tol=5e-4, tight_up_to=3,
                              start=(30, 10, 0.01))
    assert want["k_opt"] == 3 and got["k_opt"] == 3
    with pytest.raises(lib.NNRescalError) as ei:
        lib.nnrescal_init(dx, k=3, q=2, delta=0.03, seed=2, start=(0, 10, 0.01))
    assert ei.value.status == 1


def test_start_rejects_bad_arguments(lib):
    X, _, _ = gen.dense_tiny()
    h = lib.nnrescal_init(lib.DenseX(torch.from_numpy(X).to(DEV).contiguous()), k=3, q=2, delta=0.03, seed=0)
    for kw in (dict(svd_iters=0, r_iters=1, floor_rel=0.01), dict(svd_iters=5, r_iters=-1, floor_rel=0.01),
               dict(svd_iters=5, r_iters=1, floor_rel=-0.5)):
        with pytest.raises(lib.NNRescalError) as ei:
            lib.nnrescal_start_nndsvd(h, **kw)
        assert ei.value.status == 1
    lib.nnrescal_destroy(h)
