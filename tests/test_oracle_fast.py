"""Pins for the compiled twin of the oracle's perturbation (oracle/fast.py, oracle/csrc/perturb_fast.c).

The NumPy oracle is the definition; the C routines exist because the definition takes hours on a 16384 x 16384 x 32
tensor.  They are pinned to something other than themselves: the generator to the published known-answer vectors
(tests/golden/philox4x32_10_kat.txt) and to the NumPy implementation word for word, the perturbed values bit for bit
to perturb.perturb_dense / perturb.perturb_coo (which are themselves pinned in test_oracle_philox.py: every rounding
redone in rational arithmetic), over members of every half-word, several amplitudes, values from denormal products
to 3e37, row blocks that start inside a slice and linear indices beyond 2^32.
"""
import os

import numpy as np

from oracle import fast, perturb, philox

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_generator_known_answers_and_numpy_agreement():
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        got = fast.philox_blocks(np.array([v[0:4]], dtype=np.uint32), v[4], v[5])
        assert [int(x) for x in got[0]] == v[6:10]
    rng = np.random.default_rng(5)
    c = rng.integers(0, 2**32, size=(1000, 4), dtype=np.uint64)
    want = np.stack(philox.philox4x32_10(c[:, 0], c[:, 1], c[:, 2], c[:, 3], 0xDEADBEEF, 0x01234567), axis=1)
    assert np.array_equal(fast.philox_blocks(c.astype(np.uint32), 0xDEADBEEF, 0x01234567), want)


def test_dense_values_bit_for_bit():
    rng = np.random.default_rng(0)
    n, m = 96, 3
    X = rng.random((m, n, n)).astype(np.float32)
    X[1] *= np.float32(3.0e4)
    X[2, 0, :8] = [0.0, 1e-30, 1.0, 2.5e-7, 65504.0, 3.4e37, 1e-37, 7.0]
    for seed, delta in ((0, 0.03), (0x1234567890ABCDEF, 0.25), (99, 0.0123456789), (7, 0.001)):
        for member in (0, 1, 6, 7, 8, 13, 19, 63):
            want = perturb.perturb_dense(X, seed, member, delta)
            for t in range(m):
                got = fast.perturb_dense_slice(X[t], t, seed, member, delta)
                assert np.array_equal(got.view(np.uint32), want[t].view(np.uint32)), (seed, delta, member, t)
            # a block of rows that starts inside the slice
            got = fast.perturb_dense_slice(X[1, 40:71], 1, seed, member, delta, i0=40)
            assert np.array_equal(got.view(np.uint32), want[1, 40:71].view(np.uint32))
    assert np.array_equal(fast.perturb_dense_slice(X[0], 0, 1, 2, 0.0), X[0])


def test_coordinate_values_bit_for_bit_also_beyond_32_bit_indices():
    rng = np.random.default_rng(1)
    n = 10_000_000                                 # i * n + j needs 47 bits
    rows = rng.integers(0, n, 5000)
    cols = rng.integers(0, n, 5000)
    rows[:3], cols[:3] = [0, n - 1, n - 1], [0, n - 1, 0]
    vals = (rng.random(5000) + 1e-3).astype(np.float32)
    for member in (0, 3, 9):
        want = perturb.perturb_coo(rows, cols, vals, 2, n, 77, member, 0.03)
        got = fast.perturb_coo(rows, cols, vals, 2, n, 77, member, 0.03)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # dense and coordinate forms agree on the same elements
    X = rng.random((1, 50, 50)).astype(np.float32)
    ii, jj = np.nonzero(X[0] > 0.5)
    assert np.array_equal(fast.perturb_coo(ii, jj, X[0][ii, jj], 0, 50, 3, 5, 0.03),
                          fast.perturb_dense_slice(X[0], 0, 3, 5, 0.03)[ii, jj])


def test_random_start_bit_for_bit():
    for seed, member, n, m, k in ((0, 0, 70, 3, 1), (99, 5, 300, 2, 17), (0x1234567890ABCDEF, 63, 129, 4, 64)):
        assert np.array_equal(fast.init_A(seed, member, n, k), perturb.init_A(seed, member, n, k))
        assert np.array_equal(fast.init_R(seed, member, m, k), perturb.init_R(seed, member, m, k))
