"""The reproducible mode (nnrescal_params.deterministic): sums that several workgroups share are stored in pieces
and added up in a fixed order instead of atomically, so two runs on the same input must agree bit for bit: factors,
objective, products.  The mode must also still be right: against the oracle at the usual bars, and against the
default path to rounding."""
import numpy as np
import pytest
import torch

from synth import generators as gen
from tests.gpu_helpers import oracle_fit, rel_fro

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(lib, dx, k, q, iters, deterministic, **kw):
    h = lib.nnrescal_init(dx, k=k, q=q, delta=0.03, seed=3, deterministic=deterministic, fused_small=False, **kw)
    obj = lib.nnrescal_fit(h, iters, objective=True)
    A, R = lib.nnrescal_get_factors(h)
    P, Q = lib.nnrescal_products(h, dx.m - 1)
    torch.cuda.synchronize()
    out = (A.cpu().numpy(), R.cpu().numpy(), np.array(obj), P.cpu().numpy(), Q.cpu().numpy())
    lib.nnrescal_destroy(h)
    return out


def _same_bits(a, b):
    return all(np.array_equal(x.view(np.uint8), y.view(np.uint8)) for x, y in zip(a, b))


@pytest.mark.parametrize("n,m,k,q", [(300, 2, 16, 9), (685, 3, 44, 5), (1000, 2, 5, 20), (130, 5, 64, 2), (70, 80, 9, 2)])
def test_dense_two_runs_same_bits(lib, n, m, k, q):
    """Shapes with several column panels, several member groups and a tail group, wide ranks (the Gram pass of its
    own) and so many slices that the A rule stages R_t slice by slice."""
    X, _, _ = gen.dense_community(n=n, m=m, rank=4, noise=0.01, seed=n)
    dx = lib.DenseX(torch.from_numpy(X).to(DEV))
    a = _run(lib, dx, k, q, 4, True)
    b = _run(lib, dx, k, q, 4, True)
    assert _same_bits(a, b)
    Ao, Ro, _ = oracle_fit(X, k, q, 0.03, 3, 4)
    c = _run(lib, dx, k, q, 4, False)
    for r in range(q):
        assert rel_fro(a[0][r], Ao[r]) <= 3e-5 and rel_fro(a[1][r], Ro[r]) <= 3e-5
    assert rel_fro(a[0], c[0]) <= 5e-6 and rel_fro(a[1], c[1]) <= 5e-6 and np.allclose(a[2], c[2], rtol=1e-5)


@pytest.mark.parametrize("gather_form", [1, 2])
@pytest.mark.parametrize("with_csc", [True, False])
def test_sparse_two_runs_same_bits(lib, with_csc, gather_form):
    """A power-law tensor (rows of thousands of non-zeros cross many chunk borders) and a community tensor; given
    with its CSC copy, or as CSR with the copy built by the library; both forms of the products."""
    for S, k, q in ((gen.sparse_powerlaw(n=3000, m=3, draws_per_slice=60000, rank=4, seed=2)[0], 8, 3),
                    (gen.sparse_community(n=1000, m=2, nnz_per_slice=20000, rank=4, communities=4, seed=1)[0], 33, 4)):
        sx = lib.SparseX.from_host(S, DEV, with_csc=with_csc)
        a = _run(lib, sx, k, q, 3, True, gather_form=gather_form)
        b = _run(lib, sx, k, q, 3, True, gather_form=gather_form)
        assert _same_bits(a, b)
        Ao, Ro, _ = oracle_fit(S, k, q, 0.03, 3, 3)
        for r in range(q):
            assert rel_fro(a[0][r], Ao[r]) <= 3e-5 and rel_fro(a[1][r], Ro[r]) <= 3e-5
        c = _run(lib, sx, k, q, 3, False)
        assert rel_fro(a[0], c[0]) <= 5e-6 and rel_fro(a[1], c[1]) <= 5e-6
        assert rel_fro(a[3], c[3]) <= 5e-6 and rel_fro(a[4], c[4]) <= 5e-6


def test_reproducible_mode_needs_a_csc_copy(lib):
    S, _, _ = gen.sparse_community(n=300, m=2, nnz_per_slice=2000, rank=3, communities=3, seed=1)
    with pytest.raises(lib.NNRescalError) as ei:
        lib.nnrescal_init(lib.SparseX.from_host(S, DEV, with_csc=False), k=3, q=2, deterministic=True, csc_build=False)
    assert ei.value.status == 1 and "CSC" in str(ei.value)


def test_dense_medium_full_size_two_runs_same_bits(lib):
    """benchmark configuration 2 (n = 2048, m = 16, q = 20, k = 16: 16 panels, two full member groups and a tail group)."""
    X, _, _ = gen.dense_community(n=2048, m=16, rank=8, noise=0.01, seed=0)
    dx = lib.DenseX(torch.from_numpy(X).to(DEV))
    a = _run(lib, dx, 16, 20, 3, True)
    b = _run(lib, dx, 16, 20, 3, True)
    assert _same_bits(a, b)
    c = _run(lib, dx, 16, 20, 3, False)
    assert rel_fro(a[0], c[0]) <= 5e-6 and rel_fro(a[1], c[1]) <= 5e-6
