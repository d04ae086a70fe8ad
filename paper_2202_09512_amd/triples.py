"""Reader for relational data given as a plain triple file, the form in which knowledge-graph data sets such as the
ones of section "Real-world Data" (Nations, Trade) are commonly distributed: one fact per line,

    subject <TAB or blanks> relation <TAB or blanks> object

Empty lines and lines that start with '#' are skipped; if a line holds a tab, fields are cut at tabs (names may then
contain blanks), otherwise at blanks.  Entities and relations are numbered in the order of their first appearance.
The result is the binary tensor of the paper's Introduction, X[t][i][j] = 1 iff relation t links entity i to entity
j, as per-slice CSR and CSC index arrays WITHOUT value arrays (every stored entry is 1: the library then reads 4
bytes per stored entry instead of 8).  Duplicate facts are stored once.  Input preparation only: none of the
method's arithmetic lives here.
"""
from dataclasses import dataclass, field

import numpy as np


@dataclass
class TripleTensor:
    n: int
    m: int
    csr_rowptr: np.ndarray      # int64 [m, n+1], offsets local to the slice
    csr_col: np.ndarray         # int32 [nnz]
    csr_slice_off: np.ndarray   # int64 [m+1]
    csc_colptr: np.ndarray      # int64 [m, n+1]
    csc_row: np.ndarray         # int32 [nnz]
    csc_slice_off: np.ndarray   # int64 [m+1]
    entities: list = field(default_factory=list)     # name of entity i
    relations: list = field(default_factory=list)    # name of relation t
    binary: bool = True
    csr_val = None
    csc_val = None

    @property
    def nnz(self):
        return int(self.csr_slice_off[-1])


def from_index_triples(subj, rel, obj, n=None, m=None, entities=None, relations=None):
    """The same tensor from integer arrays (subject id, relation id, object id), one entry per fact."""
    subj = np.asarray(subj, dtype=np.int64)
    rel = np.asarray(rel, dtype=np.int64)
    obj = np.asarray(obj, dtype=np.int64)
    if not (subj.shape == rel.shape == obj.shape and subj.ndim == 1):
        raise ValueError("subject, relation and object arrays must be one-dimensional and of equal length")
    if subj.size and (subj.min() < 0 or obj.min() < 0 or rel.min() < 0):
        raise ValueError("negative index")
    n = int(max(subj.max(initial=-1), obj.max(initial=-1)) + 1) if n is None else int(n)
    m = int(rel.max(initial=-1) + 1) if m is None else int(m)
    if n < 1 or m < 1:
        raise ValueError("no entities or no relations")
    if subj.size and (max(subj.max(), obj.max()) >= n or rel.max() >= m):
        raise ValueError("index out of range")
    if n * n * m >= 2 ** 62:
        raise ValueError("tensor too large for 64-bit coordinate keys")
    key = np.unique((rel * n + subj) * n + obj)                 # slice-major, then row-major; duplicates dropped
    t, i, j = key // (n * n), (key // n) % n, key % n
    off = np.zeros(m + 1, dtype=np.int64)
    off[1:] = np.cumsum(np.bincount(t, minlength=m))
    csr_rowptr = np.zeros((m, n + 1), dtype=np.int64)
    csc_colptr = np.zeros((m, n + 1), dtype=np.int64)
    csc_row = np.empty(key.size, dtype=np.int32)
    for s in range(m):
        lo, hi = int(off[s]), int(off[s + 1])
        csr_rowptr[s, 1:] = np.cumsum(np.bincount(i[lo:hi], minlength=n))
        csc_colptr[s, 1:] = np.cumsum(np.bincount(j[lo:hi], minlength=n))
        order = np.lexsort((i[lo:hi], j[lo:hi]))                # column-major order inside the slice
        csc_row[lo:hi] = i[lo:hi][order]
    return TripleTensor(n, m, csr_rowptr, j.astype(np.int32), off, csc_colptr, csc_row, off.copy(),
                        list(entities) if entities is not None else [str(v) for v in range(n)],
                        list(relations) if relations is not None else [str(v) for v in range(m)])


def load_triples(path):
    """Read a triple file (see the module docstring) -> TripleTensor."""
    ent, rel_ids = {}, {}
    s_idx, r_idx, o_idx = [], [], []
    with open(path, "r", encoding="utf-8") as f:
        for lineno, line in enumerate(f, 1):
            line = line.rstrip("\r\n")
            if not line.strip() or line.lstrip().startswith("#"):
                continue
            parts = [p.strip() for p in line.split("\t")] if "\t" in line else line.split()
            if len(parts) != 3 or not all(parts):
                raise ValueError(f"{path}:{lineno}: expected 'subject relation object', got {line!r}")
            s, r, o = parts
            s_idx.append(ent.setdefault(s, len(ent)))
            o_idx.append(ent.setdefault(o, len(ent)))
            r_idx.append(rel_ids.setdefault(r, len(rel_ids)))
    if not s_idx:
        raise ValueError(f"{path}: no triples")
    return from_index_triples(s_idx, r_idx, o_idx, len(ent), len(rel_ids), list(ent), list(rel_ids))
