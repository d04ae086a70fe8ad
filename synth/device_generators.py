"""The dense generators of `generators.py` evaluated on the GPU, for tensors too large to build on the host
(dense large workload: n = 16384, m = 32, 34 GB).  Input drawing only: the planted factors come from the same
host routine (`community_factors`, numpy `default_rng(seed)`), the slices X_t = A R_t A^T and the relative
Gaussian noise are formed with torch on the device (`torch.Generator` seeded with `seed`).  Same recipe as
`generators.dense_community`; the noise stream differs from the host generator's, which does not matter because
oracle and library always receive the very same array.
"""
import numpy as np

from .generators import community_factors


def dense_community_device(n, m, rank, noise, seed, device):
    """Returns (X torch.float32 [m, n, n] on `device`, A float64 [n, rank], R float64 [m, rank, rank])."""
    import torch
    rng = np.random.default_rng(seed)
    A, R = community_factors(rng, n, rank, m)
    At = torch.from_numpy(A).to(device=device, dtype=torch.float32)
    Rt = torch.from_numpy(R).to(device=device, dtype=torch.float32)
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    X = torch.empty((m, n, n), dtype=torch.float32, device=device)
    for t in range(m):
        X0 = (At @ Rt[t]) @ At.T
        if noise > 0:
            X0.mul_(1.0 + noise * torch.randn((n, n), generator=g, device=device, dtype=torch.float32))
        X[t] = X0.clamp_(min=0.0)
        del X0
    return X, A, R


# --------------------------------------------------------------------------- sparse tensors, built on the device
class DeviceSparseTensor:
    """Per-slice CSR and CSC arrays as torch tensors on the GPU (the layout of `generators.SparseTensor`: int64
    pointers local to the slice, int32 indices, float32 values, rows sorted by column, no duplicates, no stored
    zeros); the slice offsets are host arrays.  `to_host()` gives the same tensor as a `generators.SparseTensor`,
    so that the oracle and the library always see the very same arrays."""

    def __init__(self, n, m, csr_rowptr, csr_col, csr_val, csr_slice_off, csc_colptr, csc_row, csc_val, binary=False):
        self.n, self.m = int(n), int(m)
        self.binary = binary    # every stored value is 1: the library may be given no value arrays
        self.csr_rowptr, self.csr_col, self.csr_val = csr_rowptr, csr_col, csr_val
        self.csc_colptr, self.csc_row, self.csc_val = csc_colptr, csc_row, csc_val
        self.csr_slice_off = np.asarray(csr_slice_off, dtype=np.int64)
        self.csc_slice_off = self.csr_slice_off.copy()

    @property
    def nnz(self):
        return int(self.csr_slice_off[-1])

    def to_host(self):
        from .generators import SparseTensor
        h = lambda t: t.cpu().numpy()
        return SparseTensor(self.n, self.m, h(self.csr_rowptr), h(self.csr_col), h(self.csr_val), self.csr_slice_off.copy(),
                            h(self.csc_colptr), h(self.csc_row), h(self.csc_val), self.csc_slice_off.copy(), self.binary)


def _planted_values_device(A, Rt, rows, cols, chunk=1 << 22):
    """(A R_t A^T)[rows, cols] in fp64 on the device, a chunk of positions at a time."""
    import torch
    out = torch.empty(rows.numel(), dtype=torch.float64, device=rows.device)
    for lo in range(0, rows.numel(), chunk):
        hi = min(lo + chunk, rows.numel())
        out[lo:hi] = ((A[rows[lo:hi]] @ Rt) * A[cols[lo:hi]]).sum(dim=1)
    return out


def _assemble_device(n, per_slice):
    """per_slice: list of (key int64 = row * n + col, sorted and unique; vals float32) on the device."""
    import torch
    m = len(per_slice)
    dev = per_slice[0][0].device
    csr_rowptr = torch.zeros((m, n + 1), dtype=torch.int64, device=dev)
    csc_colptr = torch.zeros((m, n + 1), dtype=torch.int64, device=dev)
    off = np.zeros(m + 1, dtype=np.int64)
    cc, cv, rr, rv = [], [], [], []
    for t, (key, vals) in enumerate(per_slice):
        keep = vals > 0
        key, vals = key[keep], vals[keep]
        rows, cols = key // n, key % n                      # row-major order already (the keys are sorted)
        csr_rowptr[t, 1:] = torch.cumsum(torch.bincount(rows, minlength=n), 0)
        cc.append(cols.to(torch.int32))
        cv.append(vals)
        order = torch.argsort(cols * n + rows)              # column-major order
        csc_colptr[t, 1:] = torch.cumsum(torch.bincount(cols, minlength=n), 0)
        rr.append(rows[order].to(torch.int32))
        rv.append(vals[order])
        off[t + 1] = off[t] + int(key.numel())
        del rows, cols, order, key, vals, keep
    return DeviceSparseTensor(n, m, csr_rowptr, torch.cat(cc), torch.cat(cv), off, csc_colptr, torch.cat(rr), torch.cat(rv))


def _community_keys_device(n, nnz_per_slice, communities, inside, g, device):
    """Sorted unique keys row * n + col of one slice's positions (see sparse_community_device)."""
    import torch
    bsz = n // communities
    n_in = int(round(nnz_per_slice * inside))
    ri = lambda hi, cnt: torch.randint(0, hi, (cnt,), generator=g, device=device, dtype=torch.int64)
    blk = ri(communities, n_in)
    rows = torch.cat([blk * bsz + ri(bsz, n_in), ri(n, nnz_per_slice - n_in)])
    cols = torch.cat([blk * bsz + ri(bsz, n_in), ri(n, nnz_per_slice - n_in)])
    return torch.unique(rows * n + cols)


def sparse_community_device(n, m, nnz_per_slice, rank, communities, seed, device, inside=0.9, shuffle_ids=False):
    """The recipe of `generators.sparse_community` on the device: `inside` of the positions uniform inside one of
    `communities` diagonal blocks of contiguous entities (block chosen uniformly), the rest uniform over n x n,
    duplicates dropped; values (A R_t A^T)_ij of a planted community-structured A; shuffle_ids relabels the entities
    by a random permutation afterwards (no locality left in the ids).  Planted factors from the host routine;
    positions from `torch.Generator(seed)`.  Returns (DeviceSparseTensor, A, R)."""
    import torch
    rng = np.random.default_rng(seed)
    A, R = community_factors(rng, n, rank, m)
    Ad = torch.from_numpy(A).to(device)
    Rd = torch.from_numpy(R).to(device)
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    relabel = torch.randperm(n, generator=g, device=device) if shuffle_ids else None
    slices = []
    for t in range(m):
        key = _community_keys_device(n, nnz_per_slice, communities, inside, g, device)
        vals = _planted_values_device(Ad, Rd[t], key // n, key % n).to(torch.float32)
        if relabel is not None:
            key, order = torch.sort(relabel[key // n] * n + relabel[key % n])
            vals = vals[order]
        slices.append((key, vals))
    del Ad
    if relabel is not None:
        Ap = np.empty_like(A)
        Ap[relabel.cpu().numpy()] = A
        A = Ap
    return _assemble_device(n, slices), A, R


def sparse_binary_device(n, m, nnz_per_slice, communities, seed, device, inside=0.9):
    """The recipe of `generators.sparse_binary` on the device: the positions of the community tensor, every stored
    value 1 (a binary relational tensor).  Returns (DeviceSparseTensor with binary=True, None, None)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    slices = []
    for t in range(m):
        key = _community_keys_device(n, nnz_per_slice, communities, inside, g, device)
        slices.append((key, torch.ones(key.numel(), dtype=torch.float32, device=device)))
    D = _assemble_device(n, slices)
    D.binary = True
    return D, None, None


def sparse_powerlaw_device(n, m, draws_per_slice, rank, seed, device, exponent=1.1):
    """The recipe of `generators.sparse_powerlaw` on the device: row and column of every position drawn
    independently from Zipf(exponent) over a random permutation of the entity ids (inverse of the cumulative
    distribution at a uniform draw), duplicates dropped; values U(0,1] times the planted (A R_t A^T)_ij.
    Returns (DeviceSparseTensor, A, R)."""
    import torch
    rng = np.random.default_rng(seed)
    A, R = community_factors(rng, n, rank, m)
    Ad = torch.from_numpy(A).to(device)
    Rd = torch.from_numpy(R).to(device)
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    cdf = torch.cumsum(torch.arange(1, n + 1, dtype=torch.float64, device=device) ** (-exponent), 0)
    cdf /= cdf[-1].clone()
    ids = torch.randperm(n, generator=g, device=device)
    draw = lambda: ids[torch.searchsorted(cdf, torch.rand(draws_per_slice, generator=g, device=device,
                                                          dtype=torch.float64)).clamp_(max=n - 1)]
    slices = []
    for t in range(m):
        rows = draw()
        key = rows * n
        del rows
        key += draw()
        key = torch.unique(key)
        u = 1.0 - torch.rand(key.numel(), generator=g, device=device, dtype=torch.float64)      # (0, 1]
        vals = (u * _planted_values_device(Ad, Rd[t], key // n, key % n)).to(torch.float32)
        slices.append((key, vals))
        del u
    del Ad, cdf, ids
    return _assemble_device(n, slices), A, R
