"""The entry point that allocates nothing (nnrescal_mu_step_static: one iteration with every workspace in the
library's static device array) against the existing path (nnrescal_init with the same factors, nnrescal_mu_step,
nnrescal_get_factors), through the C ABI: two calls in a row on the same GPU, the second with a smaller input, so
that whatever the first call left in the shared array would show; then sparse tensors in both forms.  The two paths
run the same kernels, so they agree to the rounding of sums taken in another order (atomic adds); the bar is the
one-iteration bar of the parity tests, 1e-5 relative Frobenius error, and the first case is also held against the
CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import mu, perturb
from synth import generators as gen
from tests.gpu_helpers import rel_fro

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _handle_step(lib, dx, A0, R0, delta, seed, **kw):
    q, _, k = A0.shape
    h = lib.nnrescal_init(dx, k=k, q=q, delta=delta, seed=seed, A0=A0, R0=R0, **kw)
    lib.nnrescal_mu_step(h)
    A, R = lib.nnrescal_get_factors(h)
    torch.cuda.synchronize()
    lib.nnrescal_destroy(h)
    return A.cpu().numpy(), R.cpu().numpy()


def _static_step(lib, dx, A0, R0, delta, seed):
    A, R = A0.clone(), R0.clone()
    status = torch.full((1,), 7, dtype=torch.int32, device=DEV)
    # number of allocations torch's caching allocator has served so far (it only ever grows): the binding of this
    # call must not add to it (the library itself never uses that allocator here: it gets no callbacks)
    count = lambda: torch.cuda.memory_stats().get("allocation.all.allocated", 0)
    before = count()
    lib.nnrescal_mu_step_static(dx, A, R, delta=delta, seed=seed, status=status)
    assert count() == before
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    return A.cpu().numpy(), R.cpu().numpy()


def _starts(rng, q, n, m, k):
    A0 = torch.from_numpy(rng.random((q, n, k)).astype(np.float32) + 0.01).to(DEV)
    R0 = torch.from_numpy(rng.random((q, m, k, k)).astype(np.float32) + 0.01).to(DEV)
    return A0, R0


def test_static_step_equals_handle_step(lib):
    rng = np.random.default_rng(42)
    # ---- dense, then a smaller dense problem right behind it (fewer rows, slices, members and columns)
    for n, m, k, q, seed in ((300, 2, 16, 9, 3), (100, 1, 5, 3, 4)):
        X, _, _ = gen.dense_community(n=n, m=m, rank=4, noise=0.01, seed=n)
        dx = lib.DenseX(torch.from_numpy(X).to(DEV))
        A0, R0 = _starts(rng, q, n, m, k)
        As, Rs = _static_step(lib, dx, A0, R0, 0.03, seed)
        Ah, Rh = _handle_step(lib, dx, A0, R0, 0.03, seed)
        assert rel_fro(As, Ah) <= 1e-5 and rel_fro(Rs, Rh) <= 1e-5, (n, rel_fro(As, Ah), rel_fro(Rs, Rh))
        assert np.isfinite(As).all() and As.min() >= 0 and Rs.min() >= 0
        for r in range(q):      # and against the oracle
            Xq = list(perturb.perturb_dense(X, seed, r, 0.03))
            Ao, Ro = mu.mu_iteration(Xq, A0[r].cpu().numpy(), R0[r].cpu().numpy())
            assert rel_fro(As[r], Ao) <= 1e-5 and rel_fro(Rs[r], Ro) <= 1e-5, (n, r)
    # ---- sparse with both formats given, then CSR alone (X_t^T A by atomic adds: no copy is built)
    for n, m, nnz, k, q, with_csc in ((1000, 3, 9000, 17, 4, True), (400, 2, 3000, 4, 2, False)):
        S, _, _ = gen.sparse_community(n=n, m=m, nnz_per_slice=nnz, rank=4, communities=4, seed=n)
        sx = lib.SparseX.from_host(S, DEV, with_csc=with_csc)
        A0, R0 = _starts(rng, q, n, m, k)
        As, Rs = _static_step(lib, sx, A0, R0, 0.03, 9)
        Ah, Rh = _handle_step(lib, sx, A0, R0, 0.03, 9, csc_build=False)
        assert rel_fro(As, Ah) <= 1e-5 and rel_fro(Rs, Rh) <= 1e-5, (n, with_csc)


def test_static_step_rejects_what_does_not_fit(lib):
    """8 slices of 4096 entities at q = 8, k = 16 need 2 * 8 * 4096 * 128 * 4 bytes for the two products alone: more
    than the static array holds.  Rejected before any device work, with both figures in the message."""
    X = torch.zeros((8, 4096, 4096), dtype=torch.float32, device=DEV)
    A = torch.ones((8, 4096, 16), dtype=torch.float32, device=DEV)
    R = torch.ones((8, 8, 16, 16), dtype=torch.float32, device=DEV)
    with pytest.raises(lib.NNRescalError) as ei:
        lib.nnrescal_mu_step_static(lib.DenseX(X), A, R)
    assert ei.value.status == 1 and "static array" in str(ei.value) and str(32 << 20) in str(ei.value)
    assert float(A.min()) == 1.0 and float(R.max()) == 1.0     # outputs untouched
    with pytest.raises(lib.NNRescalError) as ei:
        lib.nnrescal_mu_step_static(lib.DenseX(X[:1, :64, :64].contiguous()), A[:, :64].contiguous(), R[:, :1].contiguous(),
                                    delta=1.5)
    assert ei.value.status == 1
