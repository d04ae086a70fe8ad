"""Multiplicative updates for non-negative RESCAL (Eq. 2; sequencing of Alg. 3 "Distributed RESCAL" with p = 1).

Test infrastructure only (see package docstring).  fp64 arithmetic throughout; inputs are the fp32
tensors the HIP library receives, widened.  With one process every distributed product of Alg. 3 is
a plain product and both broadcasts vanish, so what is left is Eq. 2 applied slice by slice:

  core rule    R_t <- R_t (*) (A^T X_t A) (/) (G R_t G + eps),                       G = A^T A
  factor rule  A   <- A (*) sum_t (X_t A R_t^T + X_t^T A R_t)
                        (/) (sum_t (A R_t G R_t^T + A R_t^T G R_t) + eps)

written as two functions of one slice each (`core_rule`, `factor_terms`) and a driver that fixes the
order in which Alg. 3 applies them.  No blocking, fusion or re-association beyond that: every
n-sized product the paper forms is formed, in particular the second pass over the slice,
X_t^T (A R_t).

Readings of the paper taken here (the text is silent or inconsistent):
  * the factor rule sums over all m slices in numerator AND denominator (Alg. 3 accumulates both
    inside the slice loop; Eq. 2 prints the sum over the numerator only);
  * the division guard eps is added once per denominator, after the sum (Eq. 2), not once per slice
    (Alg. 3's accumulation would add m*eps); it must be positive for an entry with vanishing
    numerator and denominator to stay 0 rather than become NaN;
  * the factor rule sees the R_t already updated in this iteration and the A and A^T A from the start
    of the iteration (order of Alg. 3: a slice's core is updated, then its terms are accumulated);
  * column norm for the final normalisation: Euclidean.
"""
import numpy as np


def _as_slices(X):
    """Accept a dense array [m, n, n] or an iterable of m (dense or scipy.sparse) n x n slices; yield them one at a
    time, widened to fp64.  (Lazily, so that a caller whose tensor does not fit in host memory twice can hand over
    a generator that produces slice t on demand; such a generator serves one pass, i.e. one call.)"""
    if isinstance(X, np.ndarray):
        for t in range(X.shape[0]):
            yield X[t].astype(np.float64)
    else:
        for Xt in X:
            yield Xt.astype(np.float64)


def core_rule(Xt, A, Rt, G, eps):
    """Eq. 2, first rule, for one slice: returns the updated core and X_t A (which the factor rule needs again)."""
    slice_times_factor = np.asarray(Xt @ A)                     # n x k, first pass over the slice
    projected = A.T @ slice_times_factor                        # A^T X_t A
    model_gram = G @ (Rt @ G)                                   # A^T (A R_t A^T) A = G R_t G
    return Rt * projected / (model_gram + eps), slice_times_factor


def factor_terms(Xt, A, Rt, G, slice_times_factor):
    """One slice's share of the numerator and of the denominator of Eq. 2's second rule, for the core Rt given
    (Alg. 3 hands over the core it has just updated)."""
    right = A @ Rt                                              # A R_t
    left = A @ Rt.T                                             # A R_t^T
    numerator = slice_times_factor @ Rt.T + np.asarray(Xt.T @ right)      # X_t A R_t^T + X_t^T (A R_t): second pass
    denominator = left @ (G @ Rt) + right @ (G @ Rt.T)          # A R_t^T G R_t + A R_t G R_t^T
    return numerator, denominator


def mu_iteration(X, A, R, eps=1e-16):
    """One iteration of Alg. 3's outer loop for one ensemble member.

    X: slices (see _as_slices), A: [n, k], R: [m, k, k]; returns new (A, R) as fp64 arrays.
    """
    Xs = _as_slices(X)
    A = np.asarray(A, dtype=np.float64)
    R = np.array(R, dtype=np.float64)           # copy: updated slice by slice
    G = A.T @ A                                 # of the A the iteration starts from, for both rules
    num = np.zeros_like(A)
    den = np.zeros_like(A)
    for t, Xt in enumerate(Xs):
        R[t], XtA = core_rule(Xt, A, R[t], G, eps)
        n_t, d_t = factor_terms(Xt, A, R[t], G, XtA)
        num += n_t
        den += d_t
    return A * num / (den + eps), R


def fit(X, A0, R0, iters, eps=1e-16, trace=False):
    """`iters` iterations from (A0, R0).  With trace=True also returns the objective after every iteration."""
    A = np.asarray(A0, dtype=np.float64)
    R = np.asarray(R0, dtype=np.float64)
    objs = []
    for _ in range(iters):
        A, R = mu_iteration(X, A, R, eps)
        if trace:
            objs.append(objective(X, A, R))
    return (A, R, objs) if trace else (A, R)


def fit_until(Xs, A0s, R0s, max_iters, tau, check_every=1, eps=1e-16):
    """Alg. 3 run for an ensemble until the threshold of section "Distributed RESCAL" (last paragraph):
    the alternating updates go on until the reconstruction error of Eq. 1 is below tau, or max_iters is reached.

    Xs, A0s, R0s: one (perturbed) tensor and one start per ensemble member.  Reading taken here (the paper
    names neither how often nor for which factors the error is evaluated, nor what an ensemble does):
    the error is evaluated for the factors at the START of every check_every-th iteration l = check_every,
    2*check_every, ... (iterations count from 1); that iteration is still carried out; if every member's
    value was below tau it is the last one.  Returns (As, Rs, iterations done, trace) with trace[c][r] the
    value of member r at check c.
    """
    As = [np.asarray(A, dtype=np.float64) for A in A0s]
    Rs = [np.asarray(R, dtype=np.float64) for R in R0s]
    trace = []
    for l in range(1, max_iters + 1):
        check = l % check_every == 0
        if check:
            trace.append([objective(Xs[r], As[r], Rs[r]) for r in range(len(As))])
        for r in range(len(As)):
            As[r], Rs[r] = mu_iteration(Xs[r], As[r], Rs[r], eps)
        if check and max(trace[-1]) < tau:
            return As, Rs, l, trace
    return As, Rs, max_iters, trace


def normalise(A, R):
    """Unit Euclidean columns for A with the inverse scaling moved into R, done once after the
    optimisation (section "Multiplicative Update Algorithm", last sentence): with D = diag(||A_:,s||),
    A <- A D^-1 and R_t <- D R_t D leave A R_t A^T unchanged.  A zero column is left as it is."""
    A = np.asarray(A, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    d = np.sqrt((A * A).sum(axis=0))
    d = np.where(d > 0, d, 1.0)
    return A / d[None, :], R * d[None, :, None] * d[None, None, :]


def objective(X, A, R):
    """sum_t || X_t - A R_t A^T ||_F^2 (Eq. 1).

    Dense slices: the residual is formed directly.  Sparse slices: the square is expanded,
    ||X_t||^2 - 2 <X_t, A R_t A^T> + <G R_t G, R_t> with G = A^T A, and the middle term is summed over
    the stored non-zeros only; the two forms are compared on small dense cases in the tests.
    """
    Xs = _as_slices(X)
    A = np.asarray(A, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    f = 0.0
    G = None
    for t, Xt in enumerate(Xs):
        if isinstance(Xt, np.ndarray):
            D = Xt - A @ R[t] @ A.T
            f += float((D * D).sum())
        else:
            if G is None:
                G = A.T @ A
            coo = Xt.tocoo()
            AR = A @ R[t]
            cross = float((coo.data * np.einsum("ij,ij->i", AR[coo.row], A[coo.col])).sum())
            f += float((coo.data ** 2).sum()) - 2.0 * cross + float(((G @ R[t] @ G) * R[t]).sum())
    return f


def norm_sq(X):
    """sum_t ||X_t||_F^2."""
    tot = 0.0
    for Xt in _as_slices(X):
        tot += float((Xt * Xt).sum()) if isinstance(Xt, np.ndarray) else float((Xt.data ** 2).sum())
    return tot


def relative_error(X, A, R):
    """e = ||X - A R A^T||_F / ||X||_F (section "RESCAL with Automatic Model Selection", step 5)."""
    return float(np.sqrt(max(objective(X, A, R), 0.0) / norm_sq(X)))


def r_update_only(ATXA, ATA, R0, iters, eps=1e-16):
    """Repeated R-rule of Eq. 2 with A held fixed: A^T X_t A and A^T A are then constants, so each
    iteration is k x k work.  Used by the regression step of model selection."""
    R = np.array(R0, dtype=np.float64)
    for _ in range(iters):
        for t in range(R.shape[0]):
            R[t] = R[t] * ATXA[t] / (ATA @ (R[t] @ ATA) + eps)
    return R
