"""GPU parity of the model-selection calls (Alg. 1, 5, 6 of arxiv 2202.09512) against the CPU oracle, through the C ABI.

Bars: cluster permutations bit-exact (where the best assignment is unique by a margin), medians and
silhouettes to fp32 rounding, relative errors to 1e-4 absolute, the selected k equal to the oracle's.
"""
import numpy as np
import pytest
import torch

from oracle import mu, select
from synth import generators as gen
from tests.gpu_helpers import rel_fro

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dense(lib, X):
    return lib.DenseX(torch.from_numpy(X).to(DEV).contiguous())


def _assignment_margin(A_ens, perm):
    """Smallest gap between the best and the second-best assignment over the members, measured on the
    similarity to the final median (the oracle's own matrices): ties would make several permutations valid."""
    q, n, k = A_ens.shape
    if k > 7:
        return 1.0
    A_perm = np.stack([A_ens[r][:, perm[r]] for r in range(q)])
    Mh = select.unit_columns(np.median(A_perm, axis=0))
    gap = np.inf
    for r in range(q):
        _, best, second = select.lsa_max_bruteforce(Mh.T @ select.unit_columns(A_ens[r]))
        gap = min(gap, best - second)
    return gap


def _planted_ensemble(n, m, k, q, noise, seed):
    rng = np.random.default_rng(seed)
    A0 = rng.random((n, k)) ** 3 + 1e-3
    R0 = rng.random((m, k, k))
    A_ens, R_ens, perms = [], [], []
    for r in range(q):
        pi = rng.permutation(k)
        scale = 0.5 + rng.random(k)                      # clustering must not depend on the column scaling
        A = (A0 * (1 + noise * rng.standard_normal((n, k))))[:, pi] * scale[None, :]
        A_ens.append(np.abs(A))
        R_ens.append(R0[:, pi][:, :, pi] * (1 + noise * rng.standard_normal((m, k, k))))
        perms.append(pi)
    # fancy indexing leaves Fortran-ordered members behind: the binding must cope with non-contiguous tensors
    return (np.stack(A_ens).astype(np.float32), np.abs(np.stack(R_ens)).astype(np.float32), np.stack(perms))


@pytest.mark.parametrize("n,m,k,q", [(200, 3, 4, 5), (333, 2, 7, 8), (1000, 1, 16, 4), (150, 2, 3, 20), (97, 2, 1, 3),
                                      (500, 2, 20, 6)])
def test_cluster_matches_oracle(lib, n, m, k, q):
    A_ens, R_ens, _ = _planted_ensemble(n, m, k, q, 0.05, n + k)
    got = lib.nnrescal_cluster(torch.from_numpy(A_ens).to(DEV), torch.from_numpy(R_ens).to(DEV))
    perm, A_perm, R_perm, A_med, rounds = select.custom_cluster(A_ens, R_ens)
    assert _assignment_margin(A_ens.astype(np.float64), perm) > 1e-3
    assert np.array_equal(np.array(got["perm"]), perm)                      # bit-exact assignments
    assert got["rounds"] == rounds
    assert rel_fro(got["A_med"].cpu().numpy(), A_med) < 1e-6
    assert rel_fro(got["R_med"].cpu().numpy(), np.median(R_perm, axis=0)) < 1e-6
    s_min, s_avg = select.cluster_stability(A_perm)
    assert abs(got["s_min"] - s_min) < 2e-5 and abs(got["s_avg"] - s_avg) < 2e-5


def test_cluster_recovers_planted_permutations(lib):
    A_ens, R_ens, perms = _planted_ensemble(400, 2, 6, 7, 0.02, 3)
    got = lib.nnrescal_cluster(torch.from_numpy(A_ens).to(DEV), None)
    perm = np.array(got["perm"])
    # member r holds planted column pi_r[c] at position c; aligned to member 0, cluster s must pick the position
    # of planted column pi_0[s]
    for r in range(7):
        want = [int(np.where(perms[r] == perms[0][s])[0][0]) for s in range(6)]
        assert list(perm[r]) == want
    assert got["s_min"] > 0.9


def test_cluster_degenerate_members(lib):
    # one member only: silhouettes are defined as 0; identical members: every silhouette is 1 for orthogonal columns
    A = np.zeros((1, 64, 4), dtype=np.float32)
    for c in range(4):
        A[0, 16 * c:16 * (c + 1), c] = 1.0
    got = lib.nnrescal_cluster(torch.from_numpy(A).to(DEV), None)
    assert got["s_min"] == 0.0 and got["perm"] == [[0, 1, 2, 3]]
    got = lib.nnrescal_cluster(torch.from_numpy(np.repeat(A, 3, axis=0)).to(DEV), None)
    assert abs(got["s_min"] - 1.0) < 1e-6 and abs(got["s_avg"] - 1.0) < 1e-6


def _check_select(lib, X_dev, X_host, k_lo, k_hi, q, delta, iters, seed, regress_iters=200, s_tol=5e-3, e_tol=1e-4,
                  tight_up_to=None, start=None):
    """tight_up_to: compare the per-k curves only for k <= this rank.  Above the planted rank the factorisation
    is not identifiable and long fp32 / fp64 trajectories drift apart; there only the selected k is compared.
    start: None or (svd_iters, r_iters, floor_rel) for the SVD-based start of every fit."""
    got = lib.nnrescal_select_k(X_dev, k_lo, k_hi, q, delta, iters, seed=seed, regress_iters=regress_iters, start=start)
    want = select.select_k(X_host, k_lo, k_hi, q, delta, iters, seed, regress_iters=regress_iters,
                           start=None if start is None else (start[1], start[2]))
    for i, k in enumerate(want["ks"]):
        if tight_up_to is not None and k > tight_up_to:
            continue
        assert abs(got["err"][i] - want["err"][i]) <= e_tol, (k, got["err"][i], want["err"][i])
        assert abs(got["s_min"][i] - want["s_min"][i]) <= s_tol, (k, got["s_min"][i], want["s_min"][i])
        assert abs(got["s_avg"][i] - want["s_avg"][i]) <= s_tol, (k, got["s_avg"][i], want["s_avg"][i])
    score = np.array(want["s_min"]) - np.array(want["err"])
    top2 = np.sort(score)[-2:]
    if top2[1] - top2[0] > 4 * (s_tol + e_tol):           # the oracle's own choice is clear-cut
        assert got["k_opt"] == want["k_opt"]
    ko = got["k_opt"]
    if ko == want["k_opt"]:
        assert rel_fro(got["A_med"].cpu().numpy(), want["A_med"][ko]) < 5e-3
    return got, want


def test_select_k_dense_tiny_config(lib):
    """benchmark configuration 1 (reduced iteration count so that fp32 and fp64 trajectories stay comparable)."""
    X, _, _ = gen.dense_tiny()
    _check_select(lib, _dense(lib, X), X, 2, 5, 5, 0.03, 40, 0)


def test_select_k_dense_tiny_config_200_iterations(lib):
    """benchmark configuration 1 as configured: k = 2..5, q = 5, delta = 0.03, 200 iterations, seed 0.  The curves are
    compared up to the planted rank 3; above it the factorisation is not identifiable and 200 iterations of fp32 and
    fp64 arithmetic drift apart, there the selected k is what is compared."""
    X, _, _ = gen.dense_tiny()
    _check_select(lib, _dense(lib, X), X, 2, 5, 5, 0.03, 200, 0, s_tol=2e-2, e_tol=5e-4, tight_up_to=3)


def test_select_k_community_finds_planted_rank(lib):
    """The configuration that pins the oracle's own selection (planted rank 3, 300 iterations)."""
    X, _, _ = gen.dense_community(n=72, m=3, rank=3, noise=0.01, seed=7)
    got, want = _check_select(lib, _dense(lib, X), X, 2, 5, 6, 0.03, 300, 2, s_tol=2e-2, e_tol=5e-4, tight_up_to=3)
    assert want["k_opt"] == 3 and got["k_opt"] == 3
    s = dict(zip(got["ks"], got["s_min"]))
    assert s[3] > 0.9 and s[4] < s[3] - 0.2 and s[5] < s[3] - 0.2


def test_select_k_sparse(lib):
    S, _, _ = gen.sparse_community(n=300, m=2, nnz_per_slice=12000, rank=3, communities=3, seed=4)
    _check_select(lib, lib.SparseX.from_host(S, DEV), S.to_scipy(), 2, 4, 4, 0.03, 30, 2)


@pytest.mark.parametrize("kind,k_lo,k_hi", [("dense", 2, 16), ("dense", 9, 24), ("sparse", 2, 7)])
def test_select_k_two_ranks_per_handle(lib, kind, k_lo, k_hi):
    """Two ranks that fit one 16-column block together are fitted side by side (same starts, same rules, the sums
    taken in another order): the curves must agree with those of one handle per rank to rounding, over ranges in
    which ranks pair up within one block (2..16: 14+2, 13+3, ...), across two blocks (9..24: 24+... none, 23+9, ...)
    and stay alone (16, 15, 8)."""
    if kind == "dense":
        X, _, _ = gen.dense_community(n=150, m=3, rank=5, noise=0.01, seed=3)
        dx = _dense(lib, X)
    else:
        S, _, _ = gen.sparse_community(n=300, m=2, nnz_per_slice=12000, rank=3, communities=3, seed=4)
        dx = lib.SparseX.from_host(S, DEV)
    a = lib.nnrescal_select_k(dx, k_lo, k_hi, 4, 0.03, 25, seed=5, regress_iters=50)
    b = lib.nnrescal_select_k(dx, k_lo, k_hi, 4, 0.03, 25, seed=5, regress_iters=50, rank_packing=False)
    assert a["ks"] == b["ks"]
    for i, k in enumerate(a["ks"]):
        assert abs(a["err"][i] - b["err"][i]) <= 1e-5, (k, a["err"][i], b["err"][i])
        assert abs(a["s_min"][i] - b["s_min"][i]) <= 2e-3, (k, a["s_min"][i], b["s_min"][i])
        assert abs(a["s_avg"][i] - b["s_avg"][i]) <= 2e-3, (k, a["s_avg"][i], b["s_avg"][i])
    assert a["k_opt"] == b["k_opt"]
    assert rel_fro(a["A_med"].cpu().numpy(), b["A_med"].cpu().numpy()) <= 1e-4


def test_select_k_rejects_bad_arguments(lib):
    X, _, _ = gen.dense_tiny()
    dx = _dense(lib, X)
    for kw in (dict(k_lo=0, k_hi=3), dict(k_lo=4, k_hi=3), dict(k_lo=2, k_hi=65)):
        with pytest.raises(lib.NNRescalError) as ei:
            lib.nnrescal_select_k(dx, kw["k_lo"], kw["k_hi"], 3, 0.03, 2)
        assert ei.value.status == 1
