"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI.

Bars: random stream, perturbed values and initial factors bit-exact; A, R, objective within 1e-5
relative Frobenius error after one iteration and 1e-4 after 100 iterations.
"""
import numpy as np
import pytest
import torch

from oracle import mu, perturb
from synth import generators as gen
from tests.gpu_helpers import oracle_fit, rel_fro, row_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL1, TOL100 = 1e-5, 1e-4


def _dense(lib, X):
    return lib.DenseX(torch.from_numpy(X).to(DEV).contiguous())


# ------------------------------------------------------------------------------------------ random stream
@pytest.mark.parametrize("n,m", [(64, 4), (77, 2), (130, 1)])
def test_perturb_dense_bit_exact(lib, n, m):
    rng = np.random.default_rng(n)
    X = rng.random((m, n, n)).astype(np.float32)
    dx = _dense(lib, X)
    for member in (0, 1, 6, 7, 8, 13, 19):
        got = lib.nnrescal_perturb(dx, member, 0.03, 0x1234567890ABCDEF).cpu().numpy()
        want = perturb.perturb_dense(X, 0x1234567890ABCDEF, member, 0.03)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (n, m, member)
    assert np.array_equal(lib.nnrescal_perturb(dx, 3, 0.0, 5).cpu().numpy(), X)
    # other amplitudes (a power of two, a large one, one with a full significand) and values far from 1
    Xw = (X * np.float32(3.0e4)).astype(np.float32)
    Xw[0, 0, :8] = [0.0, 1e-30, 1.0, 2.5e-7, 65504.0, 3.4e37, 1e-37, 7.0]
    dw = _dense(lib, Xw)
    for delta in (0.25, 0.5, 0.001, 0.0123456789):
        got = lib.nnrescal_perturb(dw, 5, delta, 99).cpu().numpy()
        want = perturb.perturb_dense(Xw, 99, 5, delta)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), delta


def test_perturb_sparse_bit_exact_csr_and_csc(lib):
    S, _, _ = gen.sparse_community(n=500, m=3, nnz_per_slice=6000, rank=4, communities=4, seed=1)
    sx = lib.SparseX.from_host(S, DEV)
    for member in (0, 5, 9):
        got = lib.nnrescal_perturb(sx, member, 0.03, 77).cpu().numpy()
        got_csc = lib.nnrescal_perturb(sx, member, 0.03, 77, from_csc=True).cpu().numpy()
        for t in range(S.m):
            r, c, v = S.slice_coo(t)
            lo, hi = int(S.csr_slice_off[t]), int(S.csr_slice_off[t + 1])
            want = perturb.perturb_coo(r, c, v, t, S.n, 77, member, 0.03)
            assert np.array_equal(got[lo:hi].view(np.uint32), want.view(np.uint32))
            # CSC order: column-major sort of the same coordinates
            o = np.lexsort((r, c))
            assert np.array_equal(got_csc[lo:hi].view(np.uint32), want[o].view(np.uint32))


@pytest.mark.parametrize("k", [1, 3, 16, 17])
def test_initial_factors_bit_exact(lib, k):
    X, _, _ = gen.dense_tiny(n=70, m=3, rank=3, seed=1)
    h = lib.nnrescal_init(_dense(lib, X), k=k, q=6, delta=0.03, seed=99)
    A, R = lib.nnrescal_get_factors(h)
    for r in range(6):
        assert np.array_equal(A[r].cpu().numpy(), perturb.init_A(99, r, 70, k))
        assert np.array_equal(R[r].cpu().numpy(), perturb.init_R(99, r, 3, k))
    lib.nnrescal_destroy(h)


# ------------------------------------------------------------------------------------------ one iteration
def _check_fit(lib, dx, X_host, k, q, delta, seed, iters, tol, A0=None, R0=None, **kw):
    """Dense tensors small enough for the single-launch kernel are fitted twice: by it and by the general kernels."""
    kw = dict(kw)
    if A0 is not None:
        kw.update(A0=torch.from_numpy(A0).to(DEV), R0=torch.from_numpy(R0).to(DEV))
    Ao, Ro, Xq = oracle_fit(X_host, k, q, delta, seed, iters, A0=A0, R0=R0)
    small = isinstance(X_host, np.ndarray) and X_host.shape[1] <= 64
    # a CSR-only tensor is fitted twice as well: with the CSC copy the library builds, and from the CSR slices alone
    csr_only = not isinstance(X_host, np.ndarray) and dx.c.format == 1
    for fused_small in ((True, False) if small or csr_only else (True,)):
        if csr_only:
            kw["csc_build"] = fused_small
        h = lib.nnrescal_init(dx, k=k, q=q, delta=delta, seed=seed, fused_small=fused_small, **kw)
        obj = lib.nnrescal_fit(h, iters, objective=True)
        A, R = lib.nnrescal_get_factors(h)
        A, R = A.cpu().numpy(), R.cpu().numpy()
        lib.nnrescal_destroy(h)
        assert np.all(np.isfinite(A)) and np.all(np.isfinite(R)) and A.min() >= 0 and R.min() >= 0
        for r in range(q):
            ea, er, em = rel_fro(A[r], Ao[r]), rel_fro(R[r], Ro[r]), row_err(A[r], Ao[r])
            assert ea <= tol and er <= tol, f"member {r}: relA={ea:.3e} relR={er:.3e} (k={k}, iters={iters}, {fused_small})"
            # no single row off by more than ten times the bar (in units of the typical row norm)
            assert em <= 10 * tol, f"member {r}: worst row {em:.3e} (k={k}, iters={iters}, {fused_small})"
            f_or = mu.objective(Xq[r], Ao[r], Ro[r])
            xn = mu.norm_sq(Xq[r])
            # compare relative errors sqrt(f/||X||^2) with an absolute tolerance (f itself cancels near a perfect fit)
            e_gpu, e_or = np.sqrt(max(obj[r], 0) / xn), np.sqrt(f_or / xn)
            assert abs(e_gpu - e_or) <= 1e-4, f"member {r}: objective {obj[r]} vs {f_or}"
    return A, R


@pytest.mark.parametrize("k", [2, 3, 4, 5])
def test_dense_tiny_one_iteration(lib, k):
    X, _, _ = gen.dense_tiny()
    _check_fit(lib, _dense(lib, X), X, k, 5, 0.03, 0, 1, TOL1)


@pytest.mark.parametrize("n,m,k,q", [(77, 2, 1, 1), (130, 3, 5, 3), (200, 2, 16, 9), (97, 2, 17, 8), (300, 1, 33, 5),
                                      (129, 2, 64, 2), (256, 1, 8, 20), (40, 2, 24, 12)])
def test_dense_odd_shapes_one_iteration(lib, n, m, k, q):
    X, _, _ = gen.dense_community(n=n, m=m, rank=4, noise=0.01, seed=n)
    _check_fit(lib, _dense(lib, X), X, k, q, 0.03, 3, 1, TOL1)


@pytest.mark.parametrize("n,m,k,q", [(685, 3, 44, 13), (685, 3, 32, 13), (300, 2, 16, 19), (1000, 2, 40, 6)])
def test_dense_ragged_chunks_several_member_groups(lib, n, m, k, q):
    """Row chunks whose last round has strips for only some of the waves, several member groups and slices in one
    launch: a wave without a strip still is a link in the hand-over of the tile columns (a version in which it was
    not lost single strips' contributions to X_t^T A, 1e-3 relative, on exactly these shapes)."""
    X, _, _ = gen.dense_community(n=n, m=m, rank=6, noise=0.01, seed=5)
    _check_fit(lib, _dense(lib, X), X, k, q, 0.03, 5, 3, 3e-5)


def test_dense_no_perturbation_and_given_start(lib):
    X, _, _ = gen.dense_community(n=150, m=2, rank=3, noise=0.01, seed=5)
    rng = np.random.default_rng(0)
    A0 = rng.random((2, 150, 4)).astype(np.float32) + 0.01
    R0 = rng.random((2, 2, 4, 4)).astype(np.float32) + 0.01
    _check_fit(lib, _dense(lib, X), X, 4, 2, 0.0, 1, 2, TOL1, A0=A0, R0=R0)


def test_dense_zero_rows_and_columns(lib):
    X, _, _ = gen.dense_community(n=90, m=2, rank=3, noise=0.0, seed=6)
    X[:, 10:20, :] = 0
    X[:, :, 50:55] = 0
    _check_fit(lib, _dense(lib, X), X, 3, 4, 0.03, 2, 3, TOL1 * 3)


@pytest.mark.parametrize("k", [2, 3, 5])
def test_dense_tiny_100_iterations(lib, k):
    X, _, _ = gen.dense_tiny()
    _check_fit(lib, _dense(lib, X), X, k, 5, 0.03, 0, 100, TOL100)


def test_dense_medium_reduced_100_iterations(lib):
    X, _, _ = gen.dense_community(n=384, m=4, rank=8, noise=0.01, seed=0)
    _check_fit(lib, _dense(lib, X), X, 8, 20, 0.03, 0, 100, TOL100)


# ------------------------------------------------------------------------------------------ sparse
@pytest.mark.parametrize("with_csc", [True, False])
@pytest.mark.parametrize("n,m,nnz,k,q", [(400, 2, 4000, 4, 4), (1000, 3, 9000, 16, 4), (333, 2, 2000, 17, 2),
                                          (600, 1, 20000, 48, 4), (500, 2, 3000, 64, 2), (300, 2, 1500, 3, 9)])
def test_sparse_one_iteration(lib, n, m, nnz, k, q, with_csc):
    S, _, _ = gen.sparse_community(n=n, m=m, nnz_per_slice=nnz, rank=4, communities=4, seed=n)
    sx = lib.SparseX.from_host(S, DEV, with_csc=with_csc)
    _check_fit(lib, sx, S, k, q, 0.03, 5, 1, TOL1)


def test_sparse_built_csc_copy_equals_given_one(lib):
    """The CSC copy that the library builds from CSR slices (columns ascending, rows ascending inside a column) gives the
    products of the copy made on the host, on a power-law tensor with empty rows and columns and an empty slice."""
    S, _, _ = gen.sparse_powerlaw(n=3000, m=3, draws_per_slice=40000, rank=4, seed=2)
    lo, hi = int(S.csr_slice_off[1]), int(S.csr_slice_off[2])
    keep = np.r_[0:lo, hi:S.nnz]
    for name in ("csr_col", "csr_val", "csc_row", "csc_val"):
        setattr(S, name, getattr(S, name)[keep])
    S.csr_rowptr[1] = 0
    S.csc_colptr[1] = 0
    S.csr_slice_off[2:] -= hi - lo
    S.csc_slice_off[2:] -= hi - lo
    hs = [lib.nnrescal_init(lib.SparseX.from_host(S, DEV, with_csc=w), k=5, q=3, delta=0.03, seed=1) for w in (True, False)]
    for t in range(3):
        (P0, Q0), (P1, Q1) = (lib.nnrescal_products(h, t) for h in hs)
        # (not bit for bit: rows that cross a chunk border are summed with atomic adds)
        assert torch.allclose(P0, P1, rtol=2e-6, atol=0)
        assert torch.allclose(Q0, Q1, rtol=2e-6, atol=0)
        assert (Q0 != 0).sum() == (Q1 != 0).sum() and ((Q0 != 0).sum() > 0) == (t != 1)
    for h in hs:
        lib.nnrescal_destroy(h)


def test_sparse_built_csc_copy_many_sort_blocks(lib):
    """A slice whose sort takes three digit passes (n > 2^16) and more blocks than one trip of the per-digit scan
    holds (2.4e6 entries per slice: 293 blocks of 8192 against 256 counters per trip): the products of the built copy against those of the host's copy."""
    S, _, _ = gen.sparse_community(n=70000, m=2, nnz_per_slice=2_400_000, rank=4, communities=8, seed=3)
    assert S.nnz > 2 * 256 * 8192
    hs = [lib.nnrescal_init(lib.SparseX.from_host(S, DEV, with_csc=w), k=4, q=2, delta=0.03, seed=1) for w in (True, False)]
    for t in range(2):
        (P0, Q0), (P1, Q1) = (lib.nnrescal_products(h, t) for h in hs)
        assert torch.allclose(P0, P1, rtol=2e-6, atol=0) and torch.allclose(Q0, Q1, rtol=2e-6, atol=0)
        assert float(Q0.abs().sum()) > 0
    for h in hs:
        lib.nnrescal_destroy(h)


GATHER_SHAPES = [(4, 4), (17, 4), (64, 2), (16, 5), (33, 3), (5, 20), (33, 9), (16, 1)]


@pytest.mark.parametrize("k,q", GATHER_SHAPES)
def test_sparse_gather_forms(lib, k, q, form=2):
    """Both forms of the sparse products (whole rows; one 128-byte line of every row per pass) against the
    oracle, on a power-law tensor (rows of thousands of non-zeros that cross many chunks, rows with one non-zero, empty
    rows, a ragged last chunk) and a community tensor.  The shapes cover: a row of one line and less (the form falls
    back), lines shared by two members (kp = 16, 48), a half-filled last line (q kp = 80), two members of one line on
    both sides of a block of 8 of the random stream (kp = 48, members 7 and 8), more than 256 columns."""
    for S in (gen.sparse_powerlaw(n=3000, m=2, draws_per_slice=50000, rank=4, seed=5)[0],
              gen.sparse_community(n=1500, m=2, nnz_per_slice=30011, rank=4, communities=4, seed=6)[0]):
        sx = lib.SparseX.from_host(S, DEV)
        _check_fit(lib, sx, S, k, q, 0.03, 11, 1, TOL1, gather_form=1)
        _check_fit(lib, sx, S, k, q, 0.03, 11, 1, TOL1, gather_form=form)
        # and the products themselves against those of the rows form
        hs = [lib.nnrescal_init(sx, k=k, q=q, delta=0.03, seed=11, gather_form=f) for f in (1, form)]
        assert lib.nnrescal_gather_form(hs[1]) == (form if q * 16 * ((k + 15) // 16) > 32 else 1)   # one line: rows
        for t in range(2):
            (P0, Q0), (P1, Q1) = (lib.nnrescal_products(h, t) for h in hs)
            assert torch.allclose(P0, P1, rtol=3e-6, atol=1e-30) and torch.allclose(Q0, Q1, rtol=3e-6, atol=1e-30)
            assert ((P0 != 0) == (P1 != 0)).all() and ((Q0 != 0) == (Q1 != 0)).all()
        for h in hs:
            lib.nnrescal_destroy(h)


def test_sparse_lines_form_empty_slice_and_short_chunks(lib):
    """The lines form on a tensor with an empty slice (a segment without workgroups between two others) and on tensors
    whose slices are shorter than one chunk of 256 non-zeros (groups of lanes without any work)."""
    S, _, _ = gen.sparse_powerlaw(n=3000, m=3, draws_per_slice=40000, rank=4, seed=2)
    lo, hi = int(S.csr_slice_off[1]), int(S.csr_slice_off[2])
    keep = np.r_[0:lo, hi:S.nnz]
    for name in ("csr_col", "csr_val", "csc_row", "csc_val"):
        setattr(S, name, getattr(S, name)[keep])
    S.csr_rowptr[1] = 0
    S.csc_colptr[1] = 0
    S.csr_slice_off[2:] -= hi - lo
    S.csc_slice_off[2:] -= hi - lo
    _check_fit(lib, lib.SparseX.from_host(S, DEV), S, 17, 4, 0.03, 4, 2, TOL1 * 2, gather_form=2)
    for nnz in (37, 255, 257):
        T, _, _ = gen.sparse_community(n=60, m=2, nnz_per_slice=nnz, rank=3, communities=2, seed=nnz)
        _check_fit(lib, lib.SparseX.from_host(T, DEV), T, 20, 3, 0.03, 1, 1, TOL1, gather_form=2)


def test_sparse_gather_form_chosen_at_init(lib):
    """A tensor above the size from which the library asks the tensor itself: some admissible form is chosen, the
    iteration agrees with the one of the rows form; the reproducible mode keeps the rows form; a small tensor too."""
    S, _, _ = gen.sparse_community(n=70000, m=2, nnz_per_slice=2_400_000, rank=4, communities=8, seed=3)
    sx = lib.SparseX.from_host(S, DEV)
    assert S.nnz >= 1 << 22
    out = []
    for kw in (dict(), dict(gather_form=1), dict(deterministic=True), dict(deterministic=True, gather_form=2)):
        h = lib.nnrescal_init(sx, k=32, q=4, delta=0.03, seed=2, **kw)
        form = lib.nnrescal_gather_form(h)
        assert form == kw.get("gather_form", form) and form in (1, 2) and (form == 1 or kw != dict(deterministic=True))
        lib.nnrescal_mu_step(h)
        out.append([v.cpu().numpy() for v in lib.nnrescal_get_factors(h)])
        lib.nnrescal_destroy(h)
    for A, R in out[1:]:
        assert rel_fro(A, out[0][0]) <= 5e-6 and rel_fro(R, out[0][1]) <= 5e-6
    small, _, _ = gen.sparse_community(n=500, m=2, nnz_per_slice=3000, rank=3, communities=3, seed=1)
    h = lib.nnrescal_init(lib.SparseX.from_host(small, DEV), k=32, q=4)
    assert lib.nnrescal_gather_form(h) == 1
    lib.nnrescal_destroy(h)
    with pytest.raises(lib.NNRescalError) as ei:
        lib.nnrescal_init(lib.SparseX.from_host(small, DEV), k=4, q=2, gather_form=7)
    assert ei.value.status == 1 and "gather_form" in str(ei.value)


@pytest.mark.parametrize("k,q,iters", [(5, 4, 1), (40, 3, 1), (64, 2, 1), (20, 5, 1), (6, 3, 100)])
def test_sparse_typed_relations(lib, k, q, iters):
    """Relations between entity types: a slice touches only the id ranges of its two types, so whole 16-row tiles of
    X_t A and X_t^T A do not exist (the kernels that stream them leave those tiles out, loads and products), others
    exist in part, and the products X_t A and X_t^T A of one slice exist on different ranges."""
    rng = np.random.default_rng(9)
    n, m = 420, 3
    X = np.zeros((m, n, n), dtype=np.float32)
    blocks = [((0, 200), (0, 200)), ((200, 420), (200, 420)), ((0, 200), (200, 420))]   # (rows, columns) of every slice
    for t, ((r0, r1), (c0, c1)) in enumerate(blocks):
        B = rng.random((r1 - r0, c1 - c0)).astype(np.float32)
        B[rng.random(B.shape) > 0.1] = 0
        X[t, r0:r1, c0:c1] = B
    S = gen.dense_to_sparse(X)
    assert (np.diff(S.csr_rowptr[0])[208:] == 0).all() and (np.diff(S.csc_colptr[2])[:192] == 0).all()
    _check_fit(lib, lib.SparseX.from_host(S, DEV), S, k, q, 0.03, 3, iters, TOL1 if iters == 1 else TOL100)
    _check_fit(lib, _dense(lib, X), X, k, q, 0.03, 3, iters, TOL1 if iters == 1 else TOL100)


def test_sparse_powerlaw_rows_and_empty_rows(lib):
    S, _, _ = gen.sparse_powerlaw(n=3000, m=2, draws_per_slice=40000, rank=8, seed=2)
    deg = np.diff(S.csr_rowptr[0])
    assert deg.max() > 20 * max(1, int(deg.mean())) and (deg == 0).any()
    sx = lib.SparseX.from_host(S, DEV)
    _check_fit(lib, sx, S, 8, 2, 0.03, 1, 1, TOL1)


def test_sparse_equals_dense_path(lib):
    X, _, _ = gen.dense_community(n=120, m=2, rank=3, noise=0.01, seed=8)
    X[X < np.quantile(X, 0.7)] = 0
    S = gen.dense_to_sparse(X)
    hd = lib.nnrescal_init(_dense(lib, X), k=5, q=3, delta=0.03, seed=4)
    hs = lib.nnrescal_init(lib.SparseX.from_host(S, DEV), k=5, q=3, delta=0.03, seed=4)
    lib.nnrescal_fit(hd, 3)
    lib.nnrescal_fit(hs, 3)
    Ad, Rd = lib.nnrescal_get_factors(hd)
    As, Rs = lib.nnrescal_get_factors(hs)
    assert rel_fro(As.cpu().numpy(), Ad.cpu().numpy()) < 1e-5 and rel_fro(Rs.cpu().numpy(), Rd.cpu().numpy()) < 1e-5
    lib.nnrescal_destroy(hd)
    lib.nnrescal_destroy(hs)


def test_sparse_100_iterations(lib):
    S, _, _ = gen.sparse_community(n=800, m=3, nnz_per_slice=16000, rank=4, communities=4, seed=3)
    _check_fit(lib, lib.SparseX.from_host(S, DEV), S, 4, 4, 0.03, 0, 100, TOL100)


# ------------------------------------------------------------------------------------------ edge cases
def test_dense_smaller_than_a_tile(lib):
    """n below the 16-row tile, k = n (the largest admissible rank), one slice."""
    rng = np.random.default_rng(3)
    X = rng.random((1, 5, 5)).astype(np.float32)
    _check_fit(lib, _dense(lib, X), X, 5, 3, 0.03, 7, 2, TOL1 * 2)


def test_dense_maximum_rank_and_ensemble(lib):
    """k = 64 and q = 64: the largest rank and ensemble the library accepts (tail groups of every size occur)."""
    X, _, _ = gen.dense_community(n=96, m=1, rank=4, noise=0.01, seed=11)
    _check_fit(lib, _dense(lib, X), X, 64, 64, 0.03, 1, 1, TOL1)


@pytest.mark.parametrize("n,m,k,q", [(70, 80, 9, 2), (90, 20, 30, 2), (100, 8, 40, 3), (130, 5, 64, 2)])
def test_dense_many_slices_one_iteration(lib, n, m, k, q):
    """So many slices that their R_t no longer fit the A rule's on-chip operand store together: the slice-by-slice
    variant of the rule runs (the other tests of these ranks take the all-resident one)."""
    X, _, _ = gen.dense_community(n=n, m=m, rank=4, noise=0.01, seed=n + m)
    _check_fit(lib, _dense(lib, X), X, k, q, 0.03, 5, 2, TOL1 * 2)


def test_sparse_empty_slice_and_empty_tensor_rows(lib):
    """A slice without any non-zero between two ordinary slices: its R_t becomes zero and stays finite."""
    S, _, _ = gen.sparse_community(n=200, m=3, nnz_per_slice=1500, rank=3, communities=2, seed=9)
    lo, hi = int(S.csr_slice_off[1]), int(S.csr_slice_off[2])
    keep = np.r_[0:lo, hi:S.nnz]
    for name in ("csr_col", "csr_val", "csc_row", "csc_val"):
        setattr(S, name, getattr(S, name)[keep])
    S.csr_rowptr[1] = 0
    S.csc_colptr[1] = 0
    S.csr_slice_off[2:] -= hi - lo
    S.csc_slice_off[2:] -= hi - lo
    for with_csc in (True, False):
        A, R = _check_fit(lib, lib.SparseX.from_host(S, DEV, with_csc=with_csc), S, 3, 2, 0.03, 4, 2, TOL1 * 2)
        assert np.all(R[:, 1] == 0)


def test_random_shapes_sweep(lib):
    """Shapes drawn at random (seeded): n, m, k, q and the iteration count, dense (small and larger ragged ones) and
    sparse with and without CSC."""
    rng = np.random.default_rng(123)
    for trial in range(24):
        n, m = int(rng.integers(17, 700)), int(rng.integers(1, 5))
        k, q, iters = int(rng.integers(1, min(n, 48))), int(rng.integers(1, 21)), int(rng.integers(1, 4))
        X, _, _ = gen.dense_community(n=n, m=m, rank=max(2, min(6, n // 8)), noise=0.01, seed=trial)
        _check_fit(lib, _dense(lib, X), X, k, q, 0.03, trial, iters, 3e-5)
    # larger ragged shapes with several member groups and slices per launch
    for trial in range(6):
        n, m = int(rng.integers(600, 1500)), int(rng.integers(2, 5))
        k, q, iters = int(rng.integers(1, 65)), int(rng.integers(9, 25)), int(rng.integers(2, 4))
        X, _, _ = gen.dense_community(n=n, m=m, rank=6, noise=0.01, seed=100 + trial)
        _check_fit(lib, _dense(lib, X), X, k, q, 0.03, trial, iters, 3e-5)
    for trial in range(8):
        n, m = int(rng.integers(50, 3000)), int(rng.integers(1, 4))
        k, q, nnz = int(rng.integers(1, 40)), int(rng.integers(1, 9)), int(rng.integers(n, 20 * n))
        S, _, _ = gen.sparse_community(n=n, m=m, nnz_per_slice=nnz, rank=4, communities=3, seed=trial)
        for with_csc in (True, False):
            _check_fit(lib, lib.SparseX.from_host(S, DEV, with_csc=with_csc), S, k, q, 0.03, trial, 2, 3e-5)


# ------------------------------------------------------------------------------------------ threshold stopping
def _oracle_members(X_host, k, q, delta, seed):
    from oracle import select
    dense = isinstance(X_host, np.ndarray)
    n, m = (X_host.shape[1], X_host.shape[0]) if dense else (X_host.n, X_host.m)
    Xq = select.perturbed_members(X_host if dense else X_host.to_scipy(), seed, q, delta)
    A0 = [perturb.init_A(seed, r, n, k) for r in range(q)]
    R0 = [perturb.init_R(seed, r, m, k) for r in range(q)]
    return Xq, A0, R0


@pytest.mark.parametrize("kind", ["dense", "sparse"])
def test_fit_until_threshold(lib, kind):
    """Section "Distributed RESCAL", termination by a threshold on the error of Eq. 1: the same number of
    iterations as the oracle for thresholds that the oracle's own trace crosses with a margin, the traced values
    (relative errors within 1e-4 absolute) and the factors at the stop (the bar of a plain fit of that length)."""
    if kind == "dense":
        X, _, _ = gen.dense_tiny()
        dx, k, q, seed = _dense(lib, X), 3, 3, 5
    else:
        X, _, _ = gen.sparse_community(n=300, m=2, nnz_per_slice=6000, rank=3, communities=3, seed=2)
        dx, k, q, seed = lib.SparseX.from_host(X, DEV), 3, 2, 1
    Xq, A0, R0 = _oracle_members(X, k, q, 0.03, seed)
    every, iters = 4, 40
    _, _, _, full = mu.fit_until(Xq, A0, R0, iters, 0.0, every)       # never stops: the whole trace
    worst = np.max(np.array(full), axis=1)
    xn = np.array([mu.norm_sq(Xq[r]) for r in range(q)])
    for c in (1, 4, 8):
        if not worst[c] < 0.999 * worst[c - 1]:
            continue                                                  # no margin between these two checks
        tau = 0.5 * (worst[c] + worst[c - 1])
        Ao, Ro, done_o, trace_o = mu.fit_until(Xq, A0, R0, iters, tau, every)
        assert done_o == every * (c + 1)
        h = lib.nnrescal_init(dx, k=k, q=q, delta=0.03, seed=seed)
        done, trace = lib.nnrescal_fit_until(h, iters, tau, every)
        A, R = lib.nnrescal_get_factors(h)
        lib.nnrescal_destroy(h)
        assert done == done_o and len(trace) == len(trace_o)
        e_gpu = np.sqrt(np.maximum(np.array(trace), 0) / xn[None, :])
        e_or = np.sqrt(np.array(trace_o) / xn[None, :])
        assert np.max(np.abs(e_gpu - e_or)) <= 1e-4
        tol = TOL1 if done <= 4 else TOL100
        for r in range(q):
            assert rel_fro(A[r].cpu().numpy(), Ao[r]) <= tol and rel_fro(R[r].cpu().numpy(), Ro[r]) <= tol
    # the two ends of the threshold range, and the traced values against a plain objective call
    h = lib.nnrescal_init(dx, k=k, q=q, delta=0.03, seed=seed)
    assert lib.nnrescal_fit_until(h, 6, float("inf"), 3)[0] == 3
    obj3, _ = lib.nnrescal_objective(h)                               # after 3 iterations
    done, trace = lib.nnrescal_fit_until(h, 5, 0.0, 1)                # its first check sees the same factors
    assert done == 5 and len(trace) == 5
    assert np.allclose(trace[0], obj3, rtol=1e-6)
    assert all(max(trace[c + 1]) <= max(trace[c]) * (1 + 1e-6) for c in range(4))
    for bad in (dict(max_iters=-1, tau=1.0, check_every=1), dict(max_iters=3, tau=1.0, check_every=0),
                dict(max_iters=3, tau=float("nan"), check_every=1)):
        with pytest.raises(lib.NNRescalError) as ei:
            lib.nnrescal_fit_until(h, bad["max_iters"], bad["tau"], bad["check_every"])
        assert ei.value.status == 1
    lib.nnrescal_destroy(h)


def test_small_tensor_single_launch_kernel(lib):
    """n <= 64: nnrescal_fit runs all iterations in one launch; calls can be chained with single steps of the general
    kernels in any order, and the maximum sizes the kernel accepts (n = 64, k = 64, q = 64) go through."""
    X, _, _ = gen.dense_tiny()
    dx = _dense(lib, X)
    Ao, Ro, _ = oracle_fit(X, 3, 5, 0.03, 0, 7)
    h = lib.nnrescal_init(dx, k=3, q=5, delta=0.03, seed=0)
    lib.nnrescal_fit(h, 2)          # fused
    lib.nnrescal_mu_step(h)         # general kernels
    lib.nnrescal_fit(h, 3)          # fused again
    lib.nnrescal_mu_step(h)
    A, R = lib.nnrescal_get_factors(h)
    lib.nnrescal_destroy(h)
    for r in range(5):
        assert rel_fro(A[r].cpu().numpy(), Ao[r]) <= 2e-5 and rel_fro(R[r].cpu().numpy(), Ro[r]) <= 2e-5
    X64, _, _ = gen.dense_community(n=64, m=2, rank=4, noise=0.01, seed=3)
    _check_fit(lib, _dense(lib, X64), X64, 64, 64, 0.03, 1, 1, TOL1)


# ------------------------------------------------------------------------------------------ API behaviour
def test_normalised_copy_and_resume(lib):
    X, _, _ = gen.dense_tiny()
    dx = _dense(lib, X)
    h = lib.nnrescal_init(dx, k=3, q=5, delta=0.03, seed=0)
    lib.nnrescal_fit(h, 10)
    A, R = (t.cpu().numpy() for t in lib.nnrescal_get_factors(h))
    An, Rn = (t.cpu().numpy() for t in lib.nnrescal_get_factors(h, normalised=True))
    for r in range(5):
        Ao, Ro = mu.normalise(A[r], R[r])
        assert rel_fro(An[r], Ao) < 1e-6 and rel_fro(Rn[r], Ro) < 1e-6
        assert np.allclose(np.linalg.norm(An[r].astype(np.float64), axis=0), 1.0, atol=1e-6)
    # the handle's own factors are untouched: stepping on equals a fresh handle fed the un-normalised factors
    lib.nnrescal_fit(h, 1)
    A1, R1 = (t.cpu().numpy() for t in lib.nnrescal_get_factors(h))
    h2 = lib.nnrescal_init(dx, k=3, q=5, delta=0.03, seed=0)
    lib.nnrescal_set_factors(h2, torch.from_numpy(A).to(DEV), torch.from_numpy(R).to(DEV))
    lib.nnrescal_mu_step(h2)
    A2, R2 = (t.cpu().numpy() for t in lib.nnrescal_get_factors(h2))
    assert rel_fro(A2, A1) < 1e-6 and rel_fro(R2, R1) < 1e-6
    lib.nnrescal_destroy(h)
    lib.nnrescal_destroy(h2)


def test_errors_are_reported_not_thrown(lib):
    X, _, _ = gen.dense_tiny()
    dx = _dense(lib, X)
    for kw in (dict(k=0, q=2), dict(k=65, q=2), dict(k=3, q=0), dict(k=3, q=65), dict(k=3, q=2, delta=1.0),
               dict(k=3, q=2, delta=-0.1), dict(k=3, q=2, eps_div=-1.0), dict(k=3, q=2, eps_div=0.0)):
        with pytest.raises(lib.NNRescalError) as ei:
            lib.nnrescal_init(dx, **kw)
        assert ei.value.status == 1 and len(str(ei.value)) > 20
    # allocator failure -> ENOMEM, nothing leaked
    from paper_2202_09512_amd.binding import _TorchAllocator
    al = _TorchAllocator(torch.device(DEV))
    al.fail_after = 3
    with pytest.raises(lib.NNRescalError) as ei:
        lib.nnrescal_init(dx, k=3, q=2, allocator=al)
    assert ei.value.status == 2 and len(al.live) == 0


def test_profile_classes(lib):
    X, _, _ = gen.dense_tiny()
    h = lib.nnrescal_init(_dense(lib, X), k=3, q=5, delta=0.03, seed=0)
    lib.nnrescal_profile(h, True)
    lib.nnrescal_fit(h, 4)
    pr = lib.nnrescal_profile(h, False)
    assert pr["matrix_mul"][1] == 0 and pr["matrix_mul_tail"][1] == 4     # q = 5: one tail group of 8 slots
    # A^T A once (later iterations get it from the A update), A^T X_t A once per iteration
    assert pr["gram_mul"][1] == 5 and pr["gram_mul"][0] > 0
    # mode 2: only the passes over X are timed
    lib.nnrescal_profile(h, 2)
    lib.nnrescal_fit(h, 3)
    pr = lib.nnrescal_profile(h, False)
    assert pr["matrix_mul_tail"][1] == 3 and pr["matrix_mul_tail"][0] > 0
    assert pr["gram_mul"][1] == 0 and pr["elementwise"][1] == 0
    lib.nnrescal_destroy(h)


def test_handover_timeout_is_reported_not_passed_over(lib):
    """Dense pass: a wave that waits in vain for the tile column of its neighbour must not go on silently.  The host
    forces the condition (no poll allowed at all): the kernel still ends normally, the first synchronising call
    returns NNRESCAL_EDEVICE, and so does every later call on the handle.  With the default limit the same shape
    fits as usual (every other test of this file would fail with that status otherwise)."""
    X, _, _ = gen.dense_community(n=685, m=2, rank=6, noise=0.01, seed=5)
    dx = _dense(lib, X)
    h = lib.nnrescal_init(dx, k=16, q=9, delta=0.03, seed=5, handover_spin_limit=-1)
    with pytest.raises(lib.NNRescalError) as ei:
        lib.nnrescal_fit(h, 2, objective=True)
    assert ei.value.status == 3 and "wait" in str(ei.value)
    for call in (lambda: lib.nnrescal_mu_step(h), lambda: lib.nnrescal_get_factors(h), lambda: lib.nnrescal_objective(h)):
        with pytest.raises(lib.NNRescalError) as ei:
            call()
        assert ei.value.status == 3
    lib.nnrescal_destroy(h)
    _check_fit(lib, dx, X, 16, 9, 0.03, 5, 2, 3e-5)


def test_check_input_finds_what_breaks_the_method(lib):
    """nnrescal_params.check_input: a negative entry would silently break non-negativity (section "Multiplicative Update
    Algorithm"), a NaN poisons every factor, and the sparse kernels rely on sorted rows without duplicates."""
    X, _, _ = gen.dense_community(n=90, m=2, rank=3, noise=0.01, seed=6)
    h = lib.nnrescal_init(_dense(lib, X), k=3, q=2, check_input=True)          # a valid tensor passes
    lib.nnrescal_destroy(h)
    for bad, status, word in ((-1e-3, 1, "negative"), (np.nan, 5, "NaN"), (np.inf, 5, "NaN")):
        Xb = X.copy()
        Xb[1, 57, 13] = bad
        with pytest.raises(lib.NNRescalError) as ei:
            lib.nnrescal_init(_dense(lib, Xb), k=3, q=2, check_input=True)
        assert ei.value.status == status and word in str(ei.value)
        with pytest.raises(lib.NNRescalError) as ei:
            lib.nnrescal_select_k(_dense(lib, Xb), 2, 3, 2, 0.03, 2, check_input=True)
        assert ei.value.status == status
    S, _, _ = gen.sparse_community(n=300, m=2, nnz_per_slice=2500, rank=3, communities=3, seed=9)
    h = lib.nnrescal_init(lib.SparseX.from_host(S, DEV), k=3, q=2, check_input=True)
    lib.nnrescal_destroy(h)
    import copy
    row = int(np.argmax(np.diff(S.csr_rowptr[1])))                             # a row of slice 1 with several entries
    a = int(S.csr_slice_off[1] + S.csr_rowptr[1, row])

    def broken(edit):
        B = copy.deepcopy(S)
        edit(B)
        with pytest.raises(lib.NNRescalError) as ei:
            lib.nnrescal_init(lib.SparseX.from_host(B, DEV), k=3, q=2, check_input=True)
        return ei.value

    def swap(B):
        B.csr_col[a], B.csr_col[a + 1] = B.csr_col[a + 1], B.csr_col[a]
    err = broken(swap)
    assert err.status == 1 and "sorted" in str(err)

    def duplicate(B):
        B.csr_col[a + 1] = B.csr_col[a]
    err = broken(duplicate)
    assert err.status == 1 and "twice" in str(err)

    def outside(B):
        B.csc_row[5] = 300
    err = broken(outside)
    assert err.status == 1 and "outside" in str(err)

    def pointers(B):
        B.csr_rowptr[0, 10] = B.csr_rowptr[0, 11] + 1
    err = broken(pointers)
    assert err.status == 1 and "pointers" in str(err)

    def negative(B):
        B.csc_val[7] = -2.0
    err = broken(negative)
    assert err.status == 1 and "negative" in str(err)
