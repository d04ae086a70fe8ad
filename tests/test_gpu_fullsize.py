"""GPU parity at the full sizes of the five benchmark configurations, in the launch configuration bench.py times.

Every configuration gets a factor-level comparison with the CPU oracle at its own size:
  * dense medium (n = 2048, m = 16, q = 20, k = 16): 100 iterations of two members (one of a full member group, one
    of the tail group): A, R within 1e-4 relative Frobenius error, relative reconstruction error within 1e-4;
  * dense large (n = 16384, m = 32, 34 GB, q = 8), sparse (n = 1e6, m = 8, ~1e7 non-zeros per slice, q = 4, k = 32) and
    sparse power-law as configured (n = 1e7, m = 4, ~2e8 non-zeros in all, q = 2, k = 64): ONE whole iteration of the
    oracle for one member, A and R within 1e-5, beside sampled rows of the two products of the pass over X, and a
    non-increasing objective over a few iterations (nnrescal_fit_until's trace).
The oracle's update rules are the NumPy ones (oracle/mu.py) on slices that are produced one at a time; the perturbed
values and the random start at these sizes come from the oracle's compiled twin (oracle/fast.py), which is pinned bit
for bit to the NumPy definition.  The large tensors are drawn on the device (synth/device_generators.py) and copied
to the host for the oracle, so both sides see the same arrays.

Property checked where no oracle run is affordable (dense large, noise-free): the planted factors are a fixed point
of the update rules (section "Multiplicative Update Algorithm", Eq. 2).  Its bar is 3e-5: fp32 sums of n = 16384 terms
against their exact value, rounding ~ sqrt(n) * 2^-24 ~ 8e-6 per sum, one quotient of two such sums per rule.
"""
import numpy as np
import pytest
import torch

from oracle import fast, mu, perturb
from synth import generators as gen
from tests.gpu_helpers import rel_fro, row_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SEED = 0


def _oracle_P_row(x_row, A0, seed, member, t, i, n, delta):
    """P[i, :] = sum_j X^q[t, i, j] A[j, :] for one row of X (fp32 perturbation, fp64 sum)."""
    xq = x_row * perturb.delta_field(seed, member, t, i, np.arange(n), n, delta) if delta else x_row
    return xq.astype(np.float64) @ A0.astype(np.float64)


def _oracle_Q_row(x_col, A0, seed, member, t, j, n, delta):
    """Q[j, :] = sum_i X^q[t, i, j] A[i, :] for one column of X."""
    xq = x_col * perturb.delta_field(seed, member, t, np.arange(n), j, n, delta) if delta else x_col
    return xq.astype(np.float64) @ A0.astype(np.float64)


def _check_dense_products(lib, h, X_dev, n, k, delta, slices, members, rows):
    for t in slices:
        P, Q = lib.nnrescal_products(h, t)
        for member in members:
            A0 = perturb.init_A(SEED, member, n, k)
            for i in rows:
                x_row = X_dev[t, i, :].cpu().numpy()
                x_col = X_dev[t, :, i].cpu().numpy()
                want_p = _oracle_P_row(x_row, A0, SEED, member, t, i, n, delta)
                want_q = _oracle_Q_row(x_col, A0, SEED, member, t, i, n, delta)
                assert rel_fro(P[member, i].cpu().numpy(), want_p) <= 1e-5, (t, member, i)
                assert rel_fro(Q[member, i].cpu().numpy(), want_q) <= 1e-5, (t, member, i)


def _dense_member_slices(X_dev, member, delta, progress):
    """The perturbed slices of one member, one at a time, from a tensor that lives on the device."""
    for t in range(X_dev.shape[0]):
        if t % 8 == 0:
            progress(f"oracle iteration: slice {t} of {X_dev.shape[0]}")
        yield fast.perturb_dense_slice(X_dev[t].cpu().numpy(), t, SEED, member, delta)


def _sparse_member_slices(S, member, delta, progress):
    """The perturbed slices of one member of a host SparseTensor as scipy CSR matrices, one at a time."""
    import scipy.sparse as sp
    for t in range(S.m):
        progress(f"oracle iteration: slice {t} of {S.m}")
        lo, hi = int(S.csr_slice_off[t]), int(S.csr_slice_off[t + 1])
        rows, cols, vals = S.slice_coo(t)
        vq = fast.perturb_coo(rows, cols, vals, t, S.n, SEED, member, delta)
        del rows, cols
        yield sp.csr_matrix((vq, S.csr_col[lo:hi], S.csr_rowptr[t]), shape=(S.n, S.n))


def _check_one_iteration(lib, h, slices, member, n, m, k, tol=1e-5):
    """nnrescal_mu_step on a fresh handle against one oracle iteration of `member` from the same random start."""
    Ao, Ro = mu.mu_iteration(slices, fast.init_A(SEED, member, n, k), fast.init_R(SEED, member, m, k))
    lib.nnrescal_mu_step(h)
    A, R = lib.nnrescal_get_factors(h)
    assert bool(torch.isfinite(A).all()) and bool(torch.isfinite(R).all()) and float(A.min()) >= 0 and float(R.min()) >= 0
    A, R = A[member].cpu().numpy(), R[member].cpu().numpy()
    ea, er, em = rel_fro(A, Ao), rel_fro(R, Ro), row_err(A, Ao)
    assert ea <= tol and er <= tol and em <= 10 * tol, (member, ea, er, em)


def _check_monotone(lib, h, iters=6):
    """The objective of Eq. 1 at the start of each of the next iterations, for every member: non-increasing."""
    done, trace = lib.nnrescal_fit_until(h, iters, 0.0, 1)
    tr = np.array(trace)
    assert done == iters and tr.shape[0] == iters and np.isfinite(tr).all()
    assert np.all(tr[1:] <= tr[:-1] * (1 + 1e-6)), tr


# ------------------------------------------------------------------------------------------ dense medium
def test_dense_medium_full_size(lib):
    """benchmark configuration 2 at k = 16: sampled products, then 100 iterations against the oracle for a member of
    the first full group and one of the tail group (q = 20 = 8 + 8 + 4)."""
    n, m, k, q, delta = 2048, 16, 16, 20, 0.03
    X, _, _ = gen.dense_community(n=n, m=m, rank=8, noise=0.01, seed=0)
    X_dev = torch.from_numpy(X).to(DEV)
    h = lib.nnrescal_init(lib.DenseX(X_dev), k=k, q=q, delta=delta, seed=SEED)
    _check_dense_products(lib, h, X_dev, n, k, delta, slices=(0, 15), members=(3, 12, 19), rows=(0, 1, 777, 2047))
    obj = lib.nnrescal_fit(h, 100, objective=True)
    A, R = (v.cpu().numpy() for v in lib.nnrescal_get_factors(h))
    lib.nnrescal_destroy(h)
    assert A.min() >= 0 and R.min() >= 0 and np.isfinite(A).all() and np.isfinite(R).all()
    for member in (3, 19):
        Xq = np.stack([fast.perturb_dense_slice(X[t], t, SEED, member, delta) for t in range(m)])
        Ao, Ro = mu.fit(Xq, perturb.init_A(SEED, member, n, k), perturb.init_R(SEED, member, m, k), 100)
        ea, er, em = rel_fro(A[member], Ao), rel_fro(R[member], Ro), row_err(A[member], Ao)
        assert ea <= 1e-4 and er <= 1e-4 and em <= 1e-3, (member, ea, er, em)
        xn = mu.norm_sq(Xq)
        e_gpu, e_or = np.sqrt(max(obj[member], 0) / xn), np.sqrt(mu.objective(Xq, Ao, Ro) / xn)
        assert abs(e_gpu - e_or) <= 1e-4, (member, e_gpu, e_or)


def test_dense_medium_selects_planted_rank(lib):
    """benchmark configuration 2 with its own iteration count (500) and ensemble (q = 20), on the ranks around the planted
    one: the planted rank 8 is selected, with stable clusters and a small error there, an error ten times larger
    below it and unstable clusters above it (sections "Generic RESCALk" and "Synthetic Data").  The oracle cannot
    run this size (hours); its own selection is pinned on a small tensor and compared with the library there."""
    X, _, _ = gen.dense_community(n=2048, m=16, rank=8, noise=0.01, seed=0)
    out = lib.nnrescal_select_k(lib.DenseX(torch.from_numpy(X).to(DEV)), 6, 10, 20, 0.03, 500, seed=0, regress_iters=200)
    s, e = dict(zip(out["ks"], out["s_min"])), dict(zip(out["ks"], out["err"]))
    assert out["k_opt"] == 8
    assert s[8] > 0.8 and e[8] < 0.05
    assert e[7] > 5 * e[8] and e[6] > 5 * e[8]
    assert s[9] < s[8] - 0.5 and s[10] < s[8] - 0.5
    assert tuple(out["A_med"].shape) == (2048, 8) and float(out["A_med"].min()) >= 0


# ------------------------------------------------------------------------------------------ dense large
def test_dense_large_full_size(lib, progress):
    """benchmark configuration 3 (n = 16384, m = 32, 34 GB, built on the device) at k = 16, q = 8."""
    from synth.device_generators import dense_community_device
    n, m, k, q, delta = 16384, 32, 16, 8, 0.03
    # ---- fixed point on the noise-free tensor: member r starts from the planted factors with its own column
    #      order and column scaling, all of which are exact fixed points
    X_dev, A, R = dense_community_device(n, m, 16, 0.0, 0, DEV)
    rng = np.random.default_rng(1)
    A0 = np.empty((q, n, k), dtype=np.float32)
    R0 = np.empty((q, m, k, k), dtype=np.float32)
    for r in range(q):
        pi, sc = rng.permutation(k), 0.5 + rng.random(k)
        A0[r] = A[:, pi] * sc[None, :]
        R0[r] = R[:, pi][:, :, pi] / (sc[None, :, None] * sc[None, None, :])
    h = lib.nnrescal_init(lib.DenseX(X_dev), k=k, q=q, delta=0.0, seed=SEED, A0=torch.from_numpy(A0).to(DEV),
                          R0=torch.from_numpy(R0).to(DEV))
    lib.nnrescal_mu_step(h)
    A1, R1 = (v.cpu().numpy() for v in lib.nnrescal_get_factors(h))
    lib.nnrescal_destroy(h)
    for r in range(q):
        assert rel_fro(A1[r], A0[r]) <= 3e-5 and rel_fro(R1[r], R0[r]) <= 3e-5, r
    del X_dev, h
    torch.cuda.empty_cache()
    # ---- the noisy tensor of the benchmark, perturbation on: sampled rows of both products, then one whole iteration
    #      of the oracle for one member (the slices come back from the device one at a time), then the objective
    progress("fixed point ok; the noisy tensor: products on sampled rows")
    X_dev, _, _ = dense_community_device(n, m, 16, 0.01, 0, DEV)
    h = lib.nnrescal_init(lib.DenseX(X_dev), k=k, q=q, delta=delta, seed=SEED)
    _check_dense_products(lib, h, X_dev, n, k, delta, slices=(0, 31), members=(0, 7), rows=(0, 8191, 16383))
    _check_one_iteration(lib, h, _dense_member_slices(X_dev, 5, delta, progress), 5, n, m, k)
    _check_monotone(lib, h, 4)
    lib.nnrescal_destroy(h)


def test_dense_large_selects_planted_rank(lib):
    """benchmark configuration 3 at full size, Alg. 1 around the planted rank 16 (k = 15, 16, 17, q = 8) with the SVD-based
    start and 40 iterations per fit: the clusters are stable at the planted rank only.  (No oracle at this size: the
    selection rule itself is compared with the oracle at small sizes.)"""
    from synth.device_generators import dense_community_device
    X_dev, _, _ = dense_community_device(16384, 32, 16, 0.01, 0, DEV)
    torch.cuda.synchronize()
    out = lib.nnrescal_select_k(lib.DenseX(X_dev), 15, 17, 8, 0.03, 40, seed=0, regress_iters=200, start=(5, 10, 0.01))
    s = dict(zip(out["ks"], out["s_min"]))
    e = dict(zip(out["ks"], out["err"]))
    assert out["k_opt"] == 16 and s[16] > 0.9 and s[15] < 0.5 and s[17] < 0.5
    assert e[16] < e[15] - 0.01 and abs(e[17] - e[16]) < 0.01
    del X_dev
    torch.cuda.empty_cache()


# ------------------------------------------------------------------------------------------ sparse
def _check_sparse_products(lib, h, S, k, delta, slices, members, rows):
    """Sampled rows of X_t A (from the CSR rows) and of X_t^T A (from the CSC columns) against the oracle, which
    forms them entry by entry from the stored non-zeros and the rows of the initial A that they refer to."""
    n = S.n
    A0 = {member: fast.init_A(SEED, member, n, k) for member in members}
    for t in slices:
        P, Q = lib.nnrescal_products(h, t)
        lo, lo2 = int(S.csr_slice_off[t]), int(S.csc_slice_off[t])
        for member in members:
            for i in rows:
                a, b = lo + int(S.csr_rowptr[t, i]), lo + int(S.csr_rowptr[t, i + 1])
                cols, vals = S.csr_col[a:b].astype(np.int64), S.csr_val[a:b]
                xq = fast.perturb_coo(np.full(cols.size, i), cols, vals, t, n, SEED, member, delta)
                want = xq.astype(np.float64) @ A0[member][cols].astype(np.float64)
                got = P[member, i].cpu().numpy()
                assert (rel_fro(got, want) <= 1e-5) if cols.size else (not got.any()), (t, member, i)
                a, b = lo2 + int(S.csc_colptr[t, i]), lo2 + int(S.csc_colptr[t, i + 1])
                rws, vals = S.csc_row[a:b].astype(np.int64), S.csc_val[a:b]
                xq = fast.perturb_coo(rws, np.full(rws.size, i), vals, t, n, SEED, member, delta)
                want = xq.astype(np.float64) @ A0[member][rws].astype(np.float64)
                got = Q[member, i].cpu().numpy()
                assert (rel_fro(got, want) <= 1e-5) if rws.size else (not got.any()), (t, member, i)
        del P, Q


def test_sparse_full_size(lib, progress):
    """benchmark configuration 4 (n = 1e6, m = 8, ~1e7 non-zeros per slice) at k = 32, q = 4, given as CSR: the library
    builds its CSC copy, as in the benchmark."""
    from synth.device_generators import sparse_community_device
    n, m, k, q, delta = 1_000_000, 8, 32, 4, 0.03
    progress("drawing the tensor on the device")
    D, _, _ = sparse_community_device(n, m, 10_000_000, 32, 32, 0, DEV)
    S = D.to_host()
    progress(f"{S.nnz} stored non-zeros; products on sampled rows")
    assert S.nnz > 7.9e7
    h = lib.nnrescal_init(lib.SparseX.from_device(D, with_csc=False), k=k, q=q, delta=delta, seed=SEED)
    deg = np.diff(S.csr_rowptr[0])
    _check_sparse_products(lib, h, S, k, delta, (0, 7), (0, 3), [0, int(np.argmax(deg)), n // 2 + 17, n - 1])
    _check_one_iteration(lib, h, _sparse_member_slices(S, 3, delta, progress), 3, n, m, k)
    _check_monotone(lib, h)
    lib.nnrescal_destroy(h)


def _check_powerlaw(lib, progress, m, draws_per_slice, whole_iteration):
    from synth.device_generators import sparse_powerlaw_device
    n, k, q, delta = 10_000_000, 64, 2, 0.03
    progress(f"drawing {m} x {draws_per_slice} Zipf positions on the device")
    D, _, _ = sparse_powerlaw_device(n, m, draws_per_slice, 64, 0, DEV)
    S = D.to_host()
    progress(f"{S.nnz} stored non-zeros; products on sampled rows")
    h = lib.nnrescal_init(lib.SparseX.from_device(D), k=k, q=q, delta=delta, seed=SEED)
    deg_r, deg_c = np.diff(S.csr_rowptr[0]), np.diff(S.csc_colptr[0])
    assert deg_r.max() > 100_000 and deg_c.max() > 100_000 and (deg_r == 0).any()
    rows = [int(np.argmax(deg_r)), int(np.argmax(deg_c)), int(np.argmin(deg_r)), int(np.flatnonzero(deg_r == 1)[0]),
            0, n - 1]
    _check_sparse_products(lib, h, S, k, delta, (0, m - 1), (0, 1), rows)
    if whole_iteration:
        _check_one_iteration(lib, h, _sparse_member_slices(S, 1, delta, progress), 1, n, m, k)
        _check_monotone(lib, h, 4)
    else:
        lib.nnrescal_mu_step(h)
        A1, R1 = lib.nnrescal_get_factors(h)
        assert bool(torch.isfinite(A1).all()) and bool(torch.isfinite(R1).all()) and float(A1.min()) >= 0
    lib.nnrescal_destroy(h)
    return S


def test_sparse_powerlaw_full_entity_count(lib, progress):
    """The shape of benchmark configuration 5 (n = 1e7 entities, k = 64, q = 2) with ONE slice of 1e7 Zipf(1.1) draws: most
    entity rows and columns are empty here (the heaviest hold more than 1e5 non-zeros each, spread over hundreds
    of wavefronts)."""
    _check_powerlaw(lib, progress, 1, 10_000_000, whole_iteration=False)


def test_sparse_powerlaw_full_size(lib, progress):
    """benchmark configuration 5 itself: n = 1e7, m = 4, about 2e8 stored non-zeros in all (1.27e8 Zipf(1.1) draws per slice
    leave about 5e7 distinct coordinates each), CSR + CSC, k = 64, q = 2."""
    S = _check_powerlaw(lib, progress, 4, 127_000_000, whole_iteration=True)
    assert 1.9e8 < S.nnz < 2.1e8, S.nnz
