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
