"""The triple-file reader (paper_2202_09512_amd/triples.py): host-side input preparation, no GPU needed."""
import numpy as np
import pytest

from paper_2202_09512_amd import triples


def _dense(T):
    X = np.zeros((T.m, T.n, T.n), dtype=np.float32)
    for t in range(T.m):
        lo = int(T.csr_slice_off[t])
        for i in range(T.n):
            a, b = lo + int(T.csr_rowptr[t, i]), lo + int(T.csr_rowptr[t, i + 1])
            X[t, i, T.csr_col[a:b]] = 1
    return X


def test_reads_names_comments_tabs_and_drops_duplicates(tmp_path):
    p = tmp_path / "facts.txt"
    p.write_text("# a comment\n"
                 "usa allies uk\n"
                 "uk allies usa\n"
                 "\n"
                 "usa\ttrades with\tnew zealand\n"
                 "usa allies uk\n"
                 "  china   trades_with usa \n")
    T = triples.load_triples(str(p))
    assert T.entities == ["usa", "uk", "new zealand", "china"] and T.relations == ["allies", "trades with", "trades_with"]
    assert (T.n, T.m, T.nnz) == (4, 3, 4) and T.binary and T.csr_val is None
    X = _dense(T)
    want = np.zeros((3, 4, 4), dtype=np.float32)
    want[0, 0, 1] = want[0, 1, 0] = want[1, 0, 2] = want[2, 3, 0] = 1
    assert np.array_equal(X, want)
    # the CSC arrays describe the same slices
    for t in range(T.m):
        lo = int(T.csc_slice_off[t])
        Y = np.zeros((T.n, T.n), dtype=np.float32)
        for j in range(T.n):
            a, b = lo + int(T.csc_colptr[t, j]), lo + int(T.csc_colptr[t, j + 1])
            rows = T.csc_row[a:b]
            assert np.all(np.diff(rows) > 0)
            Y[rows, j] = 1
        assert np.array_equal(Y, want[t])


def test_index_triples_random_against_dense(tmp_path):
    rng = np.random.default_rng(0)
    n, m, cnt = 37, 5, 900
    s, r, o = rng.integers(0, n, cnt), rng.integers(0, m, cnt), rng.integers(0, n, cnt)
    T = triples.from_index_triples(s, r, o, n, m)
    want = np.zeros((m, n, n), dtype=np.float32)
    want[r, s, o] = 1
    assert np.array_equal(_dense(T), want) and T.nnz == int(want.sum())
    for t in range(m):          # rows sorted by column inside every row
        lo = int(T.csr_slice_off[t])
        for i in range(n):
            a, b = lo + int(T.csr_rowptr[t, i]), lo + int(T.csr_rowptr[t, i + 1])
            assert np.all(np.diff(T.csr_col[a:b]) > 0)


def test_malformed_lines_are_refused(tmp_path):
    p = tmp_path / "bad.txt"
    p.write_text("a likes b\nonly two\n")
    with pytest.raises(ValueError, match="bad.txt:2"):
        triples.load_triples(str(p))
    p.write_text("# nothing here\n")
    with pytest.raises(ValueError, match="no triples"):
        triples.load_triples(str(p))
    with pytest.raises(ValueError):
        triples.from_index_triples([0, 5], [0, 0], [1, 1], n=3)
