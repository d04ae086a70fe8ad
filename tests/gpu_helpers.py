"""Helpers shared by the GPU parity tests: run the oracle and the HIP library on the same inputs."""
import numpy as np

from oracle import mu, perturb


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def row_err(a, b):
    """Largest error of a single row of a factor, relative to that row's own norm in the reference or to the
    root-mean-square row norm, whichever is larger (rows of power-law tensors differ in norm by orders of
    magnitude; a nearly empty row is measured against the typical one).  A local mistake (a few rows of a product
    lost) shows here long before it moves a Frobenius norm over n rows."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    norms = np.sqrt((b * b).sum(axis=-1))
    rms = np.sqrt((b * b).sum() / max(b.shape[0], 1))
    scale = np.maximum(norms, rms)
    scale[scale == 0] = 1.0
    return float((np.sqrt(((a - b) ** 2).sum(axis=-1)) / scale).max())


def oracle_members(X_host, q, delta, seed):
    """Perturbed tensors of all members: dense ndarray [m,n,n] -> list of ndarrays; SparseTensor -> scipy lists."""
    from oracle import select
    if isinstance(X_host, np.ndarray):
        return select.perturbed_members(X_host, seed, q, delta)
    return select.perturbed_members(X_host.to_scipy(), seed, q, delta)


def oracle_fit(X_host, k, q, delta, seed, iters, eps=1e-16, A0=None, R0=None):
    """fp64 oracle factors after `iters` iterations for every member: (A [q,n,k], R [q,m,k,k])."""
    Xq = oracle_members(X_host, q, delta, seed)
    n = X_host.shape[1] if isinstance(X_host, np.ndarray) else X_host.n
    m = X_host.shape[0] if isinstance(X_host, np.ndarray) else X_host.m
    As, Rs = [], []
    for r in range(q):
        a0 = perturb.init_A(seed, r, n, k) if A0 is None else A0[r]
        r0 = perturb.init_R(seed, r, m, k) if R0 is None else R0[r]
        A, R = mu.fit(Xq[r], a0, r0, iters, eps)
        As.append(A)
        Rs.append(R)
    return np.stack(As), np.stack(Rs), Xq
