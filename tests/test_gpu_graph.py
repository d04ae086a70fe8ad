"""nnrescal_mu_step inside a HIP graph: an iteration enqueues kernels only (no allocation, no memset node, no
synchronisation), so a caller may capture it on the handle's stream and replay it.  The graph is replayed several
times, with eager work of the same library and synchronisations between the replays, and every replay is checked
against a handle that made the same iterations eagerly."""
import numpy as np
import pytest
import torch

from synth import generators as gen
from tests.gpu_helpers import rel_fro

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _factors(lib, h):
    A, R = lib.nnrescal_get_factors(h)
    torch.cuda.synchronize()
    return A.cpu().numpy(), R.cpu().numpy()


@pytest.mark.parametrize("kind", ["dense", "sparse"])
def test_iterations_replayed_from_a_graph(lib, kind):
    if kind == "dense":
        X, _, _ = gen.dense_community(n=200, m=3, rank=4, noise=0.01, seed=1)
        dx = lib.DenseX(torch.from_numpy(X).to(DEV))
        k, q = 16, 9                                   # a full member group and a tail group
    else:
        S, _, _ = gen.sparse_powerlaw(n=3000, m=2, draws_per_slice=40000, rank=4, seed=2)
        dx = lib.SparseX.from_host(S, DEV)
        k, q = 8, 3
    s = torch.cuda.Stream(device=DEV)
    kw = dict(k=k, q=q, delta=0.03, seed=5, fused_small=False)
    h = lib.nnrescal_init(dx, stream=s, **kw)
    ref = lib.nnrescal_init(dx, **kw)
    lib.nnrescal_fit(h, 2)                             # the first iterations differ from the later ones (A^T A, cleared rows)
    lib.nnrescal_fit(ref, 2)
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        lib.nnrescal_mu_step(h)
        lib.nnrescal_mu_step(h)
    torch.cuda.synchronize()
    a0, _ = _factors(lib, h)
    aref, _ = _factors(lib, ref)
    assert rel_fro(a0, aref) <= 1e-6                   # capturing has not run anything
    for replay in range(3):
        with torch.cuda.stream(s):                     # (a replay runs on the current stream: the handle's)
            g.replay()
        lib.nnrescal_fit(ref, 2)
        A, R = _factors(lib, h)
        Ar, Rr = _factors(lib, ref)
        assert np.isfinite(A).all() and A.min() >= 0
        assert rel_fro(A, Ar) <= 1e-5 and rel_fro(R, Rr) <= 1e-5, (kind, replay, rel_fro(A, Ar), rel_fro(R, Rr))
        # eager work of the same handle between the replays: one more iteration on both sides, and an objective
        lib.nnrescal_mu_step(h)
        lib.nnrescal_mu_step(ref)
        o1, _ = lib.nnrescal_objective(h)
        o2, _ = lib.nnrescal_objective(ref)
        assert np.allclose(o1, o2, rtol=1e-4)
    lib.nnrescal_destroy(h)
    lib.nnrescal_destroy(ref)
