"""Binary relational tensors (Introduction: X[t][i][j] = 1 iff relation t links entity i to entity j): CSR / CSC index
arrays with NO value array, every stored entry 1.  Parity bars as for every other tensor: perturbed values bit for
bit, A and R within 1e-5 after one iteration and 1e-4 after 100; the oracle is given the same pattern with explicit
ones."""
import numpy as np
import pytest
import torch

from oracle import perturb
from paper_2202_09512_amd import triples
from synth import generators as gen
from tests.gpu_helpers import rel_fro
from tests.test_gpu_parity import TOL1, TOL100, _check_fit

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_binary_perturbed_values_bit_exact(lib):
    S = gen.sparse_binary(n=600, m=3, nnz_per_slice=7000, communities=4, seed=2)
    assert S.binary and np.all(S.csr_val == 1)
    sx = lib.SparseX.from_host(S, DEV)
    assert sx.c.csr_val is None and sx.c.csc_val is None            # no value arrays cross the boundary
    for member in (0, 5, 9):
        got = lib.nnrescal_perturb(sx, member, 0.03, 77).cpu().numpy()
        got_csc = lib.nnrescal_perturb(sx, member, 0.03, 77, from_csc=True).cpu().numpy()
        for t in range(S.m):
            r, c, v = S.slice_coo(t)
            lo, hi = int(S.csr_slice_off[t]), int(S.csr_slice_off[t + 1])
            want = perturb.perturb_coo(r, c, v, t, S.n, 77, member, 0.03)
            assert np.array_equal(got[lo:hi].view(np.uint32), want.view(np.uint32))
            assert np.array_equal(got_csc[lo:hi].view(np.uint32), want[np.lexsort((r, c))].view(np.uint32))


@pytest.mark.parametrize("with_csc", [True, False])
@pytest.mark.parametrize("n,m,nnz,k,q", [(400, 2, 4000, 4, 4), (1000, 3, 9000, 17, 4), (500, 2, 3000, 64, 2)])
def test_binary_one_iteration(lib, n, m, nnz, k, q, with_csc):
    """with_csc False: given as CSR alone, fitted with the CSC copy the library builds (no values there either) and
    from the CSR slices alone."""
    S = gen.sparse_binary(n=n, m=m, nnz_per_slice=nnz, communities=4, seed=n)
    _check_fit(lib, lib.SparseX.from_host(S, DEV, with_csc=with_csc), S, k, q, 0.03, 5, 1, TOL1)


def test_binary_100_iterations(lib):
    S = gen.sparse_binary(n=800, m=3, nnz_per_slice=16000, communities=4, seed=3)
    _check_fit(lib, lib.SparseX.from_host(S, DEV), S, 4, 4, 0.03, 0, 100, TOL100)


def test_binary_equals_explicit_ones(lib):
    """The same pattern handed over with value arrays of ones gives the same factors (sums in the same order up to the
    atomic adds of rows that cross a chunk border)."""
    S = gen.sparse_binary(n=700, m=2, nnz_per_slice=9000, communities=3, seed=4)
    out = []
    for binary in (True, False):
        S.binary = binary
        h = lib.nnrescal_init(lib.SparseX.from_host(S, DEV), k=6, q=3, delta=0.03, seed=1)
        lib.nnrescal_fit(h, 3)
        out.append([v.cpu().numpy() for v in lib.nnrescal_get_factors(h)])
        lib.nnrescal_destroy(h)
    assert rel_fro(out[0][0], out[1][0]) <= 2e-6 and rel_fro(out[0][1], out[1][1]) <= 2e-6
    # a value array for only one of the two formats is refused
    S.binary = False
    sx = lib.SparseX.from_host(S, DEV)
    sx.c.csc_val = None
    with pytest.raises(lib.NNRescalError) as ei:
        lib.nnrescal_init(sx, k=3, q=2)
    assert ei.value.status == 1 and "binary" in str(ei.value)


def test_triple_file_to_fit(lib, tmp_path):
    """A triple file read by the package's reader, fitted, against the oracle on the same facts."""
    rng = np.random.default_rng(5)
    n, m = 120, 3
    names = [f"e{i}" for i in range(n)]
    lines = []
    for _ in range(2500):
        i, j = rng.integers(0, n, 2)
        if i // 40 == j // 40 or rng.random() < 0.1:             # three communities and some background
            lines.append(f"{names[i]}\trel{rng.integers(0, m)}\t{names[j]}")
    p = tmp_path / "facts.tsv"
    p.write_text("\n".join(lines) + "\n")
    T = triples.load_triples(str(p))
    assert T.m == m and T.n <= n and T.nnz > 500
    ones = np.ones(T.nnz, dtype=np.float32)
    S = gen.SparseTensor(T.n, T.m, T.csr_rowptr, T.csr_col, ones, T.csr_slice_off, T.csc_colptr, T.csc_row, ones.copy(),
                         T.csc_slice_off, binary=True)
    _check_fit(lib, lib.SparseX.from_host(T, DEV), S, 3, 4, 0.03, 2, 2, TOL1 * 2)
