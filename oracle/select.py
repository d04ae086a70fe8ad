"""Model selection by ensemble stability (Alg. 1 "Rescalk", Alg. 5 "customCluster",
Alg. 6 "clusterStability", section "RESCAL with Automatic Model Selection" steps 1-6).

Test infrastructure only (see package docstring).  fp64 arithmetic.

Readings of the paper taken here:
  * similarity in the assignment step is the cosine similarity of columns (section "Generic RESCALk":
    the reordering maximises cosine similarity); Alg. 5 prints a raw M^T A, which is the same thing
    once both operands have unit columns, so both are normalised before the product;
  * the assignment maximises the summed similarity (= minimises summed cosine distance);
  * "median": element-wise median over the members; for an even count the mean of the two middle
    values; the loop stops when no member's permutation changes (at most `max_rounds` rounds);
  * silhouettes: the standard definition on cosine DISTANCE with the point itself left out of its own
    cluster's mean (the text after Alg. 6 says "cosine distance"; the listing's Gram matrices are
    similarities and its means include the point itself);
  * regression: R-only multiplicative updates on the unperturbed X with A fixed to the median
    (Alg. 1's comment on its regression statement), started from the element-wise median of the
    permuted member cores, floored at 1e-12;
  * k_opt: largest separation s_min(k) - e(k), ties to the larger k (section "Synthetic Data",
    selection criteria); the threshold rule of step 6 is offered as an alternative.
"""
import itertools

import numpy as np
from scipy.optimize import linear_sum_assignment

from . import mu, nndsvd, perturb


def unit_columns(A):
    A = np.asarray(A, dtype=np.float64)
    d = np.sqrt((A * A).sum(axis=0))
    return A / np.where(d > 0, d, 1.0)[None, :]


def lsa_max(G):
    """Permutation pi maximising sum_s G[s, pi[s]] (library routine; Alg. 5's LSA statement)."""
    rows, cols = linear_sum_assignment(np.asarray(G, dtype=np.float64), maximize=True)
    pi = np.empty(G.shape[0], dtype=np.int64)
    pi[rows] = cols
    return pi


def lsa_max_bruteforce(G):
    """Same by enumeration of all k! permutations (k <= 8); returns (pi, best, second_best)."""
    k = G.shape[0]
    best, second, arg = -np.inf, -np.inf, None
    for p in itertools.permutations(range(k)):
        v = sum(G[s, p[s]] for s in range(k))
        if v > best:
            best, second, arg = v, best, p
        elif v > second:
            second = v
    return np.array(arg, dtype=np.int64), best, second


def custom_cluster(A_ens, R_ens=None, max_rounds=50):
    """Alg. 5.  A_ens: [q, n, k] (any column scaling), R_ens: [q, m, k, k] or None.

    Returns (perm [q, k], A_perm [q, n, k], R_perm or None, median [n, k], rounds).
    perm[q, s] = index of the column of member q placed in cluster s.
    """
    A_ens = np.asarray(A_ens, dtype=np.float64)
    q, n, k = A_ens.shape
    M = A_ens[0].copy()                                    # centroid = first member's solution
    prev = None
    rounds = 0
    for rounds in range(1, max_rounds + 1):
        Mh = unit_columns(M)
        perm = np.empty((q, k), dtype=np.int64)
        for r in range(q):
            G = Mh.T @ unit_columns(A_ens[r])              # similarity of centroid s with column c
            perm[r] = lsa_max(G)
        A_perm = np.stack([A_ens[r][:, perm[r]] for r in range(q)])
        M = np.median(A_perm, axis=0)
        if prev is not None and np.array_equal(prev, perm):
            break
        prev = perm
    R_perm = None
    if R_ens is not None:
        R_ens = np.asarray(R_ens, dtype=np.float64)
        R_perm = np.stack([R_ens[r][:, perm[r]][:, :, perm[r]] for r in range(q)])
    return perm, A_perm, R_perm, M, rounds


def silhouettes(A_perm):
    """Silhouette value of each of the q*k columns (cluster label = column position), cosine distance.

    Returns sil [q, k].  a = mean distance to the other q-1 members of the own cluster, b = smallest
    mean distance to the q members of another cluster, sil = (b - a) / max(a, b); 0 if max(a,b) = 0,
    if q = 1 or if k = 1.
    """
    A_perm = np.asarray(A_perm, dtype=np.float64)
    q, n, k = A_perm.shape
    sil = np.zeros((q, k))
    if q == 1 or k == 1:
        return sil
    U = np.stack([unit_columns(A_perm[r]) for r in range(q)])      # [q, n, k]
    P = U.transpose(1, 0, 2).reshape(n, q * k)                     # point index = r*k + s
    D = 1.0 - P.T @ P                                              # cosine distances
    D = D.reshape(q, k, q, k)
    for r in range(q):
        for s in range(k):
            a = (D[r, s, :, s].sum() - D[r, s, r, s]) / (q - 1)
            b = min(D[r, s, :, c].mean() for c in range(k) if c != s)
            den = max(a, b)
            sil[r, s] = 0.0 if den == 0 else (b - a) / den
    return sil


def cluster_stability(A_perm):
    """(s_min, s_avg): minimum over clusters of the cluster's mean silhouette, and the overall mean
    (Alg. 6 last statement and the remark after it)."""
    sil = silhouettes(A_perm)
    return float(sil.mean(axis=0).min()), float(sil.mean())


def regression(X, A_med, R_init, iters=1000, eps=1e-16):
    """R-only updates on the unperturbed X with A fixed (model-selection step 3)."""
    Xs = mu._as_slices(X)
    A = np.asarray(A_med, dtype=np.float64)
    ATA = A.T @ A
    ATXA = np.stack([A.T @ np.asarray(Xt @ A) for Xt in Xs])
    R0 = np.maximum(np.asarray(R_init, dtype=np.float64), 1e-12)
    return mu.r_update_only(ATXA, ATA, R0, iters, eps)


def choose_k(ks, s_min, err, rule="separation", s_thresh=0.75, e_slack=1.1):
    ks = list(ks)
    s_min = np.asarray(s_min, dtype=np.float64)
    err = np.asarray(err, dtype=np.float64)
    if rule == "separation":
        score = s_min - err
        best = max(range(len(ks)), key=lambda i: (score[i], ks[i]))
        return ks[best]
    ok = [i for i in range(len(ks)) if s_min[i] >= s_thresh and err[i] <= e_slack * err.min()]
    return ks[max(ok, key=lambda i: ks[i])] if ok else ks[int(np.argmin(err))]


def member_fit(X_pert, seed, member, k, iters, eps=1e-16, start=None):
    """Alg. 1's inner statement: RESCAL(X^q, k) from the member's own start, then normalise.  start: None for
    the random start of Alg. 3 step 1, or (r_iters, floor_rel) for the SVD-based start of the member's own
    perturbed tensor (section "RESCAL with Automatic Model Selection": "a random or NNDSVD initialization")."""
    m = len(X_pert)
    n = X_pert[0].shape[0]
    R0 = perturb.init_R(seed, member, m, k)
    if start is None:
        A0 = perturb.init_A(seed, member, n, k)
    else:
        A0, R0 = nndsvd.start(X_pert, k, R0, start[0], start[1], eps)
    A, R = mu.fit(X_pert, A0, R0, iters, eps)
    return mu.normalise(A, R)


def perturbed_members(X, seed, q, delta):
    """List over members of the perturbed tensor as a list of fp64-ready slices (Alg. 1, Perturb)."""
    out = []
    for member in range(q):
        if isinstance(X, np.ndarray):
            out.append(list(perturb.perturb_dense(X, seed, member, delta)))
        else:
            sl = []
            for t, Xt in enumerate(X):
                coo = Xt.tocoo()
                v = perturb.perturb_coo(coo.row, coo.col, coo.data.astype(np.float32), t, Xt.shape[0], seed,
                                        member, delta)
                sl.append(type(Xt)((v, (coo.row, coo.col)), shape=Xt.shape))
            out.append(sl)
    return out


def select_k(X, k_lo, k_hi, q, delta, iters, seed, eps=1e-16, regress_iters=1000, rule="separation", start=None):
    """Alg. 1.  Returns dict with per-k s_min, s_avg, err, k_opt and the per-k (A_med, R_reg, perm)."""
    Xq = perturbed_members(X, seed, q, delta)
    ks = list(range(k_lo, k_hi + 1))
    out = {"ks": ks, "s_min": [], "s_avg": [], "err": [], "A_med": {}, "R_reg": {}, "perm": {}}
    for k in ks:
        fits = [member_fit(Xq[r], seed, r, k, iters, eps, start) for r in range(q)]
        A_ens = np.stack([f[0] for f in fits])
        R_ens = np.stack([f[1] for f in fits])
        perm, A_perm, R_perm, A_med, _ = custom_cluster(A_ens, R_ens)
        s_min, s_avg = cluster_stability(A_perm)
        R_reg = regression(X, A_med, np.median(R_perm, axis=0), regress_iters, eps)
        out["s_min"].append(s_min)
        out["s_avg"].append(s_avg)
        out["err"].append(mu.relative_error(X, A_med, R_reg))
        out["A_med"][k], out["R_reg"][k], out["perm"][k] = A_med, R_reg, perm
    out["k_opt"] = choose_k(ks, out["s_min"], out["err"], rule)
    return out
