"""Resampling (Alg. 4, "Distributed Resampling") and random initialisation (Alg. 3 step 1).

Test infrastructure only (see package docstring).

The paper perturbs every element (sparse: every stored non-zero) by an independent uniform factor
Delta in [1-delta, 1+delta] whose mean is 1, and draws A and R uniformly at random with a different
seed per ensemble member.  It fixes no random stream, so the stream below is this build's reading;
agreement with any outside implementation is PARITY UNPINNED (only oracle <-> HIP library agreement
and the statistical properties the paper states are testable).

Stream definition.  Philox4x32-10 with key (lo32(seed), hi32(seed)) and a counter made of
  e   = linear element index (uint64), words c0 = lo32(e), c1 = hi32(e)
  c2  = a per-domain integer (slice index t for the perturbation, rank k for the initialisation)
  c3  = (domain << 16) | sub, domain 0 = perturbation, 1 = A init, 2 = R init
Perturbation: e = i*n + j (coordinates, not storage position, so dense / CSR / CSC views agree and
the value does not depend on the iteration or on k), sub = member >> 3; the block's four words are
cut into eight 16-bit halves and member q uses half (q & 7): word (q & 7) >> 1, low half if (q & 7)
is even, else high half.  With h in [0, 65535], a = delta * 2**-15 (exact) and
c = fl32(1 - 65535 * delta * 2**-16) (one rounding):
  X^q   = fl32( fl32(X a) * h + fl32(X c) )      (the outer step is ONE fused multiply-add)
i.e. X * (1 + delta * s) with s = (2h - 65535) / 65536 (symmetric about 0, never 0) to within 1.5
units in the last place of fp32; Delta itself is the perturbed value of 1, fl32(a h + c).  (The
products X a and X c do not depend on the member, which is what the definition is arranged for.)
Initialisation: sub = member, value = ((word0 >> 9) + 0.5) / 2**23 in (0, 1): an odd multiple of
2**-24, hence exact in fp32, never 1, and strictly positive (an exact zero can never leave zero
under multiplicative updates).
"""
import numpy as np

from .philox import philox4x32_10

_DOMAIN_PERTURB = 0
_DOMAIN_INIT_A = 1
_DOMAIN_INIT_R = 2


def _key(seed):
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    return seed & 0xFFFFFFFF, seed >> 32


def _constants(delta):
    """a = delta * 2**-15 and c = fl32(1 - 65535 * delta * 2**-16), both fp32, from the fp32 value of delta."""
    d64 = np.float64(np.float32(delta))
    a = np.float32(d64 * 2.0 ** -15)                       # power-of-two scaling: exact
    prod = 65535.0 * (d64 * 2.0 ** -16)                    # 16 x 24 significant bits: exact in fp64
    total = 1.0 - prod
    if (1.0 - total) != prod:                              # the fp64 difference must be exact too
        raise ValueError("delta too small for the exact-sum construction of the fused multiply-add")
    return a, np.float32(total)                            # the single rounding


def _fma32(x, y, z):
    """fl32(x*y + z) with a single rounding for fp32 arrays x, z and integer-valued y < 2**16.

    x*y is exact in fp64 (24 + 16 significant bits).  The fp64 sum with z is checked to be exact
    (both terms recovered from it without error), so the cast to fp32 is the only rounding."""
    prod = x.astype(np.float64) * y.astype(np.float64)
    z64 = z.astype(np.float64)
    total = prod + z64
    if not (np.array_equal(total - z64, prod) and np.array_equal(total - prod, z64)):
        raise ValueError("operands too far apart for the exact-sum construction of the fused multiply-add")
    return total.astype(np.float32)


def _half_words(seed, member, t, i, j, n):
    """h^member[t, i, j] in [0, 65535] as float32 for broadcastable integer arrays i, j."""
    i = np.asarray(i, dtype=np.uint64)
    j = np.asarray(j, dtype=np.uint64)
    e = i * np.uint64(n) + j
    k0, k1 = _key(seed)
    c3 = (_DOMAIN_PERTURB << 16) | (int(member) >> 3)
    words = philox4x32_10(e & np.uint64(0xFFFFFFFF), e >> np.uint64(32), int(t), c3, k0, k1)
    r = int(member) & 7
    w = words[r >> 1]
    h = (w >> np.uint32(16)) if (r & 1) else (w & np.uint32(0xFFFF))
    return h.astype(np.float32)


def _perturb_values(x, h, delta):
    """fl32(fl32(x a) h + fl32(x c)) elementwise for fp32 x and the half-words h (Alg. 4, second statement)."""
    a, c = _constants(delta)
    x = np.asarray(x, dtype=np.float32)
    return _fma32(x * a, h, x * c)                         # fp32 * fp32 -> fp32, then one fused step


def delta_field(seed, member, t, i, j, n, delta):
    """Delta^member[t, i, j] (fp32) for broadcastable integer arrays i, j (Alg. 4, first statement):
    the perturbed value of 1."""
    h = _half_words(seed, member, t, i, j, n)
    return _perturb_values(np.ones(h.shape, dtype=np.float32), h, delta)


def perturb_dense(X, seed, member, delta):
    """X^q = X (*) Delta^q for a dense tensor X[m, n, n] (fp32) -> fp32 (Alg. 4, second statement)."""
    X = np.asarray(X, dtype=np.float32)
    m, n, _ = X.shape
    if delta == 0:
        return X.copy()
    out = np.empty_like(X)
    ii = np.arange(n, dtype=np.uint64)[:, None]
    jj = np.arange(n, dtype=np.uint64)[None, :]
    for t in range(m):
        out[t] = _perturb_values(X[t], _half_words(seed, member, t, ii, jj, n), delta)
    return out


def perturb_coo(rows, cols, vals, t, n, seed, member, delta):
    """Perturb the stored non-zeros of one sparse slice; zeros are never touched, so the
    sparsity pattern is preserved ("Distributed Resampling", last sentence)."""
    vals = np.asarray(vals, dtype=np.float32)
    if delta == 0:
        return vals.copy()
    return _perturb_values(vals, _half_words(seed, member, t, rows, cols, n), delta)


def _unit_open(word):
    """Map uint32 -> fp32 in (0,1): ((w >> 9) + 0.5) * 2**-23 = (2*(w >> 9) + 1) * 2**-24.

    The numerator is an odd integer below 2**24, so the value is exact in fp32 (no rounding
    anywhere), lies in [2**-24, 1 - 2**-24] and is never 0 or 1.
    """
    v = 2 * (word >> np.uint32(9)).astype(np.int64) + 1
    return (v.astype(np.float64) * 2.0 ** -24).astype(np.float32)


def init_A(seed, member, n, k):
    """A^member of shape [n, k], entries uniform in (0,1) (Alg. 3 step 1: rand(n, k))."""
    k0, k1 = _key(seed)
    e = (np.arange(n, dtype=np.uint64)[:, None] * np.uint64(k) + np.arange(k, dtype=np.uint64)[None, :])
    c3 = (_DOMAIN_INIT_A << 16) | int(member)
    w = philox4x32_10(e & np.uint64(0xFFFFFFFF), e >> np.uint64(32), int(k), c3, k0, k1)[0]
    return _unit_open(w)


def init_A_rows(seed, member, rows, k):
    """The rows `rows` of init_A(seed, member, n, k), without forming the other rows (n does not enter the
    stream: the counter of entry (i, s) is i*k + s)."""
    k0, k1 = _key(seed)
    rows = np.asarray(rows, dtype=np.uint64)
    e = rows[:, None] * np.uint64(k) + np.arange(k, dtype=np.uint64)[None, :]
    c3 = (_DOMAIN_INIT_A << 16) | int(member)
    w = philox4x32_10(e & np.uint64(0xFFFFFFFF), e >> np.uint64(32), int(k), c3, k0, k1)[0]
    return _unit_open(w)


def init_R(seed, member, m, k):
    """R^member of shape [m, k, k], entries uniform in (0,1) (Alg. 3 step 1: rand(m, k, k))."""
    k0, k1 = _key(seed)
    e = np.arange(m * k * k, dtype=np.uint64).reshape(m, k, k)
    c3 = (_DOMAIN_INIT_R << 16) | int(member)
    w = philox4x32_10(e & np.uint64(0xFFFFFFFF), e >> np.uint64(32), int(k), c3, k0, k1)[0]
    return _unit_open(w)
