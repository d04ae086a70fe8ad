"""Pins for the oracle's random stream: Philox4x32-10 and the perturbation / initialisation maps.

The RESCAL paper fixes no stream (Alg. 4 says "uniformRandom"), so what can be pinned is (a) the
generator against its published known-answer vectors and a second implementation, and (b) the
properties Alg. 4 and the resampling section state: Delta in [1-delta, 1+delta], mean 1, zeros stay
zero, same value for every storage format and every call.
"""
import os

import numpy as np
import pytest

from oracle import perturb, philox

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def test_known_answers_scalar_and_vector():
    for ctr, key, out in _kat():
        assert list(philox.philox4x32_10_scalar(ctr, key)) == out
        v = philox.philox4x32_10(*[np.array([c]) for c in ctr], key[0], key[1])
        assert [int(x[0]) for x in v] == out


def test_two_implementations_agree():
    rng = np.random.default_rng(1)
    c = rng.integers(0, 2**32, size=(4, 257), dtype=np.uint64)
    k0, k1 = 0x12345678, 0x9ABCDEF0
    v = philox.philox4x32_10(c[0], c[1], c[2], c[3], k0, k1)
    for idx in range(c.shape[1]):
        s = philox.philox4x32_10_scalar([int(c[w, idx]) for w in range(4)], (k0, k1))
        assert tuple(int(v[w][idx]) for w in range(4)) == s


def test_delta_range_mean_variance():
    n, delta = 512, 0.03
    ii, jj = np.arange(n)[:, None], np.arange(n)[None, :]
    for member in (0, 5, 7, 8, 19):
        d = perturb.delta_field(7, member, 2, ii, jj, n, delta)
        assert d.dtype == np.float32
        assert d.min() > 1 - delta and d.max() < 1 + delta            # Alg. 4: Delta in [1-d, 1+d]
        assert abs(d.astype(np.float64).mean() - 1.0) < 4 * delta / np.sqrt(3 * n * n)   # mean 1
        assert abs(d.astype(np.float64).var() / (delta**2 / 3) - 1.0) < 0.02
    # the 16-bit lattice is symmetric: h and 65535-h give 1+x and 1-x before rounding
    h = np.arange(65536, dtype=np.float64)
    s = (2 * h - 65535) / 65536
    assert np.all(s + s[::-1] == 0) and not np.any(s == 0)


def test_members_are_distinct_and_decorrelated():
    n = 256
    ii, jj = np.arange(n)[:, None], np.arange(n)[None, :]
    fields = [perturb.delta_field(3, q, 0, ii, jj, n, 0.03).astype(np.float64).ravel() - 1 for q in range(20)]
    C = np.corrcoef(np.stack(fields))
    off = C - np.eye(20)
    assert np.abs(off).max() < 0.03
    # slices and seeds give different fields too
    a = perturb.delta_field(3, 0, 0, ii, jj, n, 0.03)
    assert not np.array_equal(a, perturb.delta_field(3, 0, 1, ii, jj, n, 0.03))
    assert not np.array_equal(a, perturb.delta_field(4, 0, 0, ii, jj, n, 0.03))
    assert np.array_equal(a, perturb.delta_field(3, 0, 0, ii, jj, n, 0.03))       # pure function


def _round_to_fp32(fr):
    """Correctly rounded (nearest, ties to even) fp32 value of a positive rational, as a rational: integer
    arithmetic only, independent of numpy's and the oracle's floating point."""
    from fractions import Fraction
    if fr == 0:
        return Fraction(0)
    e = fr.numerator.bit_length() - fr.denominator.bit_length() - 24
    while fr / Fraction(2) ** e >= 2 ** 24:
        e += 1
    while fr / Fraction(2) ** e < 2 ** 23:
        e -= 1
    assert e >= -149                                   # normal range only
    scaled = fr / Fraction(2) ** e
    q = scaled.numerator // scaled.denominator
    rem = scaled - q
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and q % 2 == 1):
        q += 1
    return Fraction(q) * Fraction(2) ** e


def test_member_to_half_word_mapping_and_arithmetic():
    """Member q uses 16-bit half (q & 7) of block (q >> 3), checked against the scalar generator, and the perturbed
    value is fl32(fl32(x a) h + fl32(x c)) with a = delta 2^-15, c = fl32(1 - 65535 delta 2^-16): every rounding
    redone in rational arithmetic.  The result is x (1 + delta (2h - 65535) / 65536) (Alg. 4) to 3 * 2^-24."""
    from fractions import Fraction
    n, seed, t, delta = 37, (0xDEADBEEF << 32) | 0x01234567, 3, np.float32(0.03)
    d = Fraction(float(delta))
    a = d / 2 ** 15
    assert _round_to_fp32(a) == a
    c = _round_to_fp32(1 - 65535 * d / 2 ** 16)
    rng = np.random.default_rng(4)
    for (i, j) in [(0, 0), (5, 36), (36, 1)]:
        e = i * n + j
        for q in range(24):
            w = philox.philox4x32_10_scalar((e & 0xFFFFFFFF, e >> 32, t, q >> 3), (0x01234567, 0xDEADBEEF))
            r = q & 7
            h = (w[r >> 1] >> 16) if (r & 1) else (w[r >> 1] & 0xFFFF)
            for x in (np.float32(1.0), np.float32(rng.random()), np.float32(rng.random() * 1e-3),
                      np.float32(3.0e4 * rng.random())):
                fx = Fraction(float(x))
                want = _round_to_fp32(_round_to_fp32(fx * a) * h + _round_to_fp32(fx * c))
                got = perturb.perturb_coo(np.array([i]), np.array([j]), np.array([x]), t, n, seed, q, delta)[0]
                assert got.dtype == np.float32 and Fraction(float(got)) == want, (i, j, q, x)
                exact = fx * (1 + d * Fraction(2 * h - 65535, 65536))
                assert abs(want - exact) <= 3 * Fraction(1, 2 ** 24) * exact
            # Delta itself is the perturbed value of 1
            assert perturb.delta_field(seed, q, t, np.array([i]), np.array([j]), n, delta)[0] == \
                perturb.perturb_coo(np.array([i]), np.array([j]), np.array([1.0]), t, n, seed, q, delta)[0]


def test_sparse_pattern_and_format_independence():
    rng = np.random.default_rng(0)
    n = 50
    X = (rng.random((2, n, n)) * (rng.random((2, n, n)) < 0.1)).astype(np.float32)
    Xq = perturb.perturb_dense(X, 11, 3, 0.03)
    assert np.array_equal(Xq == 0, X == 0)                            # zeros stay zero
    assert np.all(np.abs(Xq[X > 0] / X[X > 0] - 1) < 0.0301)
    for t in range(2):
        r, c = np.nonzero(X[t])
        v = perturb.perturb_coo(r, c, X[t][r, c], t, n, 11, 3, 0.03)
        assert np.array_equal(v, Xq[t][r, c])                          # row-major order
        o = np.lexsort((r, c))
        v2 = perturb.perturb_coo(r[o], c[o], X[t][r[o], c[o]], t, n, 11, 3, 0.03)
        assert np.array_equal(v2, Xq[t][r[o], c[o]])                   # column-major order
    assert np.array_equal(perturb.perturb_dense(X, 11, 3, 0.0), X)


def test_init_open_unit_interval_and_exact():
    A = perturb.init_A(5, 2, 1000, 7)
    R = perturb.init_R(5, 2, 3, 7)
    for Z in (A, R):
        assert Z.dtype == np.float32 and Z.min() > 0 and Z.max() < 1
        assert np.all((Z.astype(np.float64) * 2**24) % 2 == 1)         # odd multiples of 2^-24: exact
    assert abs(A.mean() - 0.5) < 0.02
    assert not np.array_equal(A, perturb.init_A(5, 3, 1000, 7))        # different start per member
    assert not np.array_equal(A[:, :5], perturb.init_A(5, 2, 1000, 5))


def test_init_A_rows_is_a_slice_of_init_A():
    from oracle import perturb
    A = perturb.init_A(11, 3, 500, 7)
    rows = np.array([0, 17, 499, 3, 3])
    assert np.array_equal(perturb.init_A_rows(11, 3, rows, 7), A[rows])
