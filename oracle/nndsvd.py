"""SVD-based start for the multiplicative updates (arxiv 2202.09512, section "Experiments", algorithmic
parameters, option 2; mentioned with Alg. 1 and Alg. 3 as the alternative to the random start).

Test infrastructure only (see package docstring).  fp64 throughout.

The paper's description, restated: the unfoldings of X along its first and its second axis are
concatenated, a non-negative double SVD of that matrix gives A, and the R statements of Alg. 3's loop
(with A held fixed) then give the R_t that go with it.  The steps below are the published NNDSVD of
Boutsidis and Gallopoulos (Pattern Recognition 41, 2008) applied to that matrix, of which only the left
factor is kept.

Readings taken here (the paper calls its variant "custom" and gives no detail):
  * the concatenation is M = [X_1 ... X_m  X_1^T ... X_m^T], n x 2nm (both unfoldings have n rows);
  * the truncated SVD is the exact one (a library routine here);
  * entries of the resulting A below floor_rel times its mean are raised to that value: an exact zero can
    never leave zero under a multiplicative rule;
  * R starts from the random R of Alg. 3 step 1 and takes r_iters R-only updates of Eq. 2.
Parity with the paper's own code is unpinned (it prints no numbers for its start); the steps are pinned by
closed forms and invariants in tests/test_oracle_nndsvd.py.
"""
import numpy as np

from . import mu


def concat_unfoldings(Xs):
    """M = [X_1 ... X_m  X_1^T ... X_m^T] as a dense fp64 array (small cases only)."""
    dense = [np.asarray(Xt.toarray() if hasattr(Xt, "toarray") else Xt, dtype=np.float64) for Xt in Xs]
    return np.concatenate(dense + [D.T for D in dense], axis=1)


def leading_triplets(M, k):
    """The k leading singular triplets (U [n,k], s [k], V [cols,k]) of M, by the library's SVD."""
    U, s, Vt = np.linalg.svd(M, full_matrices=False)
    return U[:, :k], s[:k], Vt[:k].T


def nndsvd_left(U, s, V):
    """Left factor of NNDSVD from singular triplets: column 0 is sqrt(s_0) |u_0|; for j >= 1 the triplet's
    rank-one term is split into its positive and negative parts, x = u_j, y = v_j, x+ = max(x, 0),
    x- = max(-x, 0), and the part with the larger ||x||.||y|| is kept:
    a_j = sqrt(s_j ||x+-|| ||y+-||) x+- / ||x+-||."""
    n, k = U.shape
    A = np.zeros((n, k))
    A[:, 0] = np.sqrt(s[0]) * np.abs(U[:, 0])
    for j in range(1, k):
        x, y = U[:, j], V[:, j]
        xp, xn = np.maximum(x, 0.0), np.maximum(-x, 0.0)
        yp, yn = np.maximum(y, 0.0), np.maximum(-y, 0.0)
        nxp, nxn, nyp, nyn = (np.linalg.norm(v) for v in (xp, xn, yp, yn))
        mp, mn = nxp * nyp, nxn * nyn
        if mp > mn:
            A[:, j] = np.sqrt(s[j] * mp) * xp / nxp
        elif mn > 0:
            A[:, j] = np.sqrt(s[j] * mn) * xn / nxn
    return A


def start(Xs, k, R0, r_iters=10, floor_rel=0.01, eps=1e-16):
    """(A, R) to start Alg. 3 from, for one (perturbed) tensor given as its m slices.
    R0: the random R [m, k, k] the R-only updates begin with."""
    M = concat_unfoldings(Xs)
    U, s, V = leading_triplets(M, k)
    A = nndsvd_left(U, s, V)
    A = np.maximum(A, floor_rel * A.mean())
    ATA = A.T @ A
    ATXA = np.stack([A.T @ (np.asarray(Xt.toarray() if hasattr(Xt, "toarray") else Xt, dtype=np.float64) @ A)
                     for Xt in Xs])
    R = mu.r_update_only(ATXA, ATA, R0, r_iters, eps)
    return A, R
