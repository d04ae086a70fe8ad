"""Seeded synthetic relational tensors shaped like the workloads of arxiv 2202.09512.

This module only draws inputs.  It holds none of the method's arithmetic (no update rule, no
perturbation, no clustering) and is shared by the CPU oracle's tests, the GPU parity tests and the
benchmark, so that both sides always see the same arrays.  Everything is generated from
`numpy.random.default_rng(seed)`; a planted non-negative model X_t = A R_t A^T supplies the values
(section "Synthetic Data": a planted feature matrix, a random core tensor, a small relative noise).

Dense tensors are returned as float32 [m, n, n] (slice-major, the layout Alg. 1 states).
Sparse tensors are returned as `SparseTensor`: per-slice CSR and CSC arrays, int64 row/column
pointers, int32 indices, float32 values, rows sorted by column, no duplicates, no stored zeros.
"""
from dataclasses import dataclass

import numpy as np


# --------------------------------------------------------------------------- planted factors
def uniform_factors(rng, n, rank, m):
    """A ~ U[0,1)^{n x rank}, R_t ~ U[0,1)^{rank x rank} (dense tiny workload)."""
    A = rng.random((n, rank))
    R = rng.random((m, rank, rank))
    return A, R


def community_factors(rng, n, rank, m):
    """Block-community A: row i has one dominant column (i*rank//n, contiguous blocks) drawn from
    U[0.5,1); all other columns U[0,0.05).  R_t ~ U[0,1)."""
    A = rng.random((n, rank)) * 0.05
    dom = (np.arange(n) * rank) // n
    A[np.arange(n), dom] = 0.5 + 0.5 * rng.random(n)
    R = rng.random((m, rank, rank))
    return A, R


# --------------------------------------------------------------------------- dense tensors
def dense_tiny(n=64, m=4, rank=3, seed=0):
    """Noise-free X_t = A R_t A^T with uniform factors.  Returns (X float32 [m,n,n], A, R)."""
    rng = np.random.default_rng(seed)
    A, R = uniform_factors(rng, n, rank, m)
    X = np.einsum("ia,tab,jb->tij", A, R, A).astype(np.float32)
    return X, A, R


def dense_community(n=2048, m=16, rank=8, noise=0.01, seed=0):
    """Community-structured planted model with relative Gaussian noise, clamped at zero:
    X = max(0, X0 * (1 + noise * N(0,1))).  Returns (X float32 [m,n,n], A, R)."""
    rng = np.random.default_rng(seed)
    A, R = community_factors(rng, n, rank, m)
    X = np.empty((m, n, n), dtype=np.float32)
    for t in range(m):
        X0 = (A @ R[t]) @ A.T
        if noise > 0:
            X0 *= 1.0 + noise * rng.standard_normal((n, n))
        np.maximum(X0, 0.0, out=X0)
        X[t] = X0
    return X, A, R


# --------------------------------------------------------------------------- sparse tensors
@dataclass
class SparseTensor:
    n: int
    m: int
    csr_rowptr: np.ndarray      # int64 [m, n+1], offsets local to the slice
    csr_col: np.ndarray         # int32 [nnz_total]
    csr_val: np.ndarray         # float32 [nnz_total]
    csr_slice_off: np.ndarray   # int64 [m+1]
    csc_colptr: np.ndarray      # int64 [m, n+1]
    csc_row: np.ndarray         # int32 [nnz_total]
    csc_val: np.ndarray         # float32 [nnz_total]
    csc_slice_off: np.ndarray   # int64 [m+1]
    binary: bool = False        # every stored value is 1 (an adjacency tensor): the library may be given no value arrays

    @property
    def nnz(self):
        return int(self.csr_slice_off[-1])

    def slice_coo(self, t):
        """(rows, cols, vals) of slice t in CSR order."""
        lo, hi = int(self.csr_slice_off[t]), int(self.csr_slice_off[t + 1])
        rows = np.repeat(np.arange(self.n, dtype=np.int64), np.diff(self.csr_rowptr[t]))
        return rows, self.csr_col[lo:hi].astype(np.int64), self.csr_val[lo:hi]

    def to_scipy(self):
        """List of m scipy.sparse.csr_matrix (float32)."""
        import scipy.sparse as sp
        out = []
        for t in range(self.m):
            lo, hi = int(self.csr_slice_off[t]), int(self.csr_slice_off[t + 1])
            out.append(sp.csr_matrix((self.csr_val[lo:hi], self.csr_col[lo:hi], self.csr_rowptr[t]),
                                     shape=(self.n, self.n)))
        return out

    def to_dense(self):
        return np.stack([s.toarray() for s in self.to_scipy()]).astype(np.float32)


def _assemble(n, per_slice):
    """per_slice: list of (rows int64, cols int64, vals float32), unique coordinates, any order."""
    m = len(per_slice)
    csr_rowptr = np.zeros((m, n + 1), dtype=np.int64)
    csc_colptr = np.zeros((m, n + 1), dtype=np.int64)
    off = np.zeros(m + 1, dtype=np.int64)
    cc, cv, rr, rv = [], [], [], []
    for t, (rows, cols, vals) in enumerate(per_slice):
        keep = vals > 0
        rows, cols, vals = rows[keep], cols[keep], vals[keep].astype(np.float32)
        o = np.lexsort((cols, rows))                        # row-major order
        csr_rowptr[t, 1:] = np.cumsum(np.bincount(rows, minlength=n))
        cc.append(cols[o].astype(np.int32))
        cv.append(vals[o])
        o2 = np.lexsort((rows, cols))                       # column-major order
        csc_colptr[t, 1:] = np.cumsum(np.bincount(cols, minlength=n))
        rr.append(rows[o2].astype(np.int32))
        rv.append(vals[o2])
        off[t + 1] = off[t] + rows.size
    cat = lambda xs, dt: np.concatenate(xs) if xs else np.zeros(0, dtype=dt)
    return SparseTensor(n, m, csr_rowptr, cat(cc, np.int32), cat(cv, np.float32), off,
                        csc_colptr, cat(rr, np.int32), cat(rv, np.float32), off.copy())


def _unique_coords(rows, cols, n):
    key = np.unique(rows.astype(np.int64) * n + cols.astype(np.int64))
    return key // n, key % n


def _planted_values(A, Rt, rows, cols, chunk=1 << 20):
    out = np.empty(rows.size, dtype=np.float64)
    for lo in range(0, rows.size, chunk):
        hi = min(lo + chunk, rows.size)
        out[lo:hi] = np.einsum("ia,ia->i", A[rows[lo:hi]] @ Rt, A[cols[lo:hi]])
    return out


def sparse_community(n=1_000_000, m=8, nnz_per_slice=10_000_000, rank=32, communities=32,
                     inside=0.9, seed=0, shuffle_ids=False):
    """Positions: `inside` of them uniform inside one of `communities` diagonal blocks of contiguous
    entities (block chosen uniformly), the rest uniform over n x n; duplicates dropped.  Values:
    (A R_t A^T)_ij from a planted community-structured A.  Returns (SparseTensor, A, R)."""
    rng = np.random.default_rng(seed)
    A, R = community_factors(rng, n, rank, m)
    relabel = rng.permutation(n) if shuffle_ids else None
    bsz = n // communities
    slices = []
    for t in range(m):
        n_in = int(round(nnz_per_slice * inside))
        blk = rng.integers(0, communities, n_in)
        rows = np.concatenate([blk * bsz + rng.integers(0, bsz, n_in), rng.integers(0, n, nnz_per_slice - n_in)])
        cols = np.concatenate([blk * bsz + rng.integers(0, bsz, n_in), rng.integers(0, n, nnz_per_slice - n_in)])
        rows, cols = _unique_coords(rows, cols, n)
        vals = _planted_values(A, R[t], rows, cols)
        if relabel is not None:
            rows, cols = relabel[rows], relabel[cols]
        slices.append((rows, cols, vals.astype(np.float32)))
    if relabel is not None:
        Ap = np.empty_like(A)
        Ap[relabel] = A
        A = Ap
    return _assemble(n, slices), A, R


def sparse_binary(n=1_000_000, m=8, nnz_per_slice=10_000_000, communities=32, inside=0.9, seed=0):
    """Binary relational tensor (Introduction: slice t holds a 1 where relation t links entity i to entity j):
    the positions of `sparse_community` (`inside` of them within one of `communities` diagonal blocks, the rest
    anywhere, duplicates dropped), every stored value 1.  Returns a SparseTensor with binary=True (its value
    arrays hold ones, for the oracle; the library is given none)."""
    rng = np.random.default_rng(seed)
    bsz = n // communities
    slices = []
    for t in range(m):
        n_in = int(round(nnz_per_slice * inside))
        blk = rng.integers(0, communities, n_in)
        rows = np.concatenate([blk * bsz + rng.integers(0, bsz, n_in), rng.integers(0, n, nnz_per_slice - n_in)])
        cols = np.concatenate([blk * bsz + rng.integers(0, bsz, n_in), rng.integers(0, n, nnz_per_slice - n_in)])
        rows, cols = _unique_coords(rows, cols, n)
        slices.append((rows, cols, np.ones(rows.size, dtype=np.float32)))
    S = _assemble(n, slices)
    S.binary = True
    return S


def sparse_powerlaw(n=10_000_000, m=4, draws_per_slice=50_000_000, rank=64, exponent=1.1, seed=0):
    """Row and column of every position drawn independently from Zipf(exponent) over a random
    permutation of the entity ids; duplicates dropped.  Values: U(0,1] times the planted
    (A R_t A^T)_ij.  Returns (SparseTensor, A, R)."""
    rng = np.random.default_rng(seed)
    A, R = community_factors(rng, n, rank, m)
    w = np.arange(1, n + 1, dtype=np.float64) ** (-exponent)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    ids = rng.permutation(n)
    slices = []
    for t in range(m):
        rows = ids[np.minimum(np.searchsorted(cdf, rng.random(draws_per_slice)), n - 1)]
        cols = ids[np.minimum(np.searchsorted(cdf, rng.random(draws_per_slice)), n - 1)]
        rows, cols = _unique_coords(rows, cols, n)
        u = 1.0 - rng.random(rows.size)                       # (0, 1]
        vals = u * _planted_values(A, R[t], rows, cols)
        slices.append((rows, cols, vals.astype(np.float32)))
    return _assemble(n, slices), A, R


def dense_to_sparse(X):
    """CSR+CSC view of a dense tensor (tests: dense and sparse paths must agree on the same data)."""
    m, n, _ = X.shape
    slices = []
    for t in range(m):
        r, c = np.nonzero(X[t])
        slices.append((r.astype(np.int64), c.astype(np.int64), X[t][r, c]))
    return _assemble(n, slices)
