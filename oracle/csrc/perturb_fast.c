/*
 * Test infrastructure only: a compiled twin of oracle/philox.py and of the perturbed-value formula of
 * oracle/perturb.py, for tensors too large for the NumPy versions (a slice of 16384 x 16384 elements, 5e7 stored
 * non-zeros).  It is NOT a second definition: the tests pin it, word for word and bit for bit, to the NumPy
 * oracle and to the published known-answer vectors of the generator.  It shares nothing with the HIP library.
 *
 * Stream (this build's reading of Alg. 4's "uniformRandom" of arxiv 2202.09512; see oracle/perturb.py):
 *   Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), key (lo32(seed), hi32(seed)),
 *   counter (lo32(e), hi32(e), slice t, member >> 3) with e = i * n + j; member r uses 16-bit half (r & 7) of the
 *   block: word (r & 7) >> 1, low half if (r & 7) is even.  With that half h, a = delta * 2^-15 and
 *   c = fl32(1 - 65535 * delta * 2^-16):     X^r = fl32( fl32(x a) * h + fl32(x c) ),  the outer step one fma.
 *
 * Compile with -ffp-contract=off: the two inner products must be rounded to fp32 before the fused step.
 */
#include <math.h>
#include <stdint.h>

static void philox_block(uint32_t c[4], uint32_t k0, uint32_t k1) {
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
    c[1] = (uint32_t)p1;
    c[3] = (uint32_t)p0;
    c[0] = n0;
    c[2] = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
}

/* count blocks: counters ctr[4 * b .. 4 * b + 3] are replaced by their outputs (for the known-answer test) */
void oracle_philox4x32_10(uint32_t *ctr, int64_t count, uint32_t k0, uint32_t k1) {
  for (int64_t b = 0; b < count; ++b) philox_block(ctr + 4 * b, k0, k1);
}

static inline float perturbed_value(float x, uint64_t e, uint32_t t, int member, uint32_t k0, uint32_t k1, float a,
                                    float c) {
  uint32_t w[4] = {(uint32_t)e, (uint32_t)(e >> 32), t, (uint32_t)(member >> 3)};
  philox_block(w, k0, k1);
  const int r = member & 7;
  const uint32_t word = w[r >> 1];
  const float h = (float)((r & 1) ? (word >> 16) : (word & 0xFFFFu));
  const float xa = x * a;      /* rounded to fp32 */
  const float xc = x * c;      /* rounded to fp32 */
  return fmaf(xa, h, xc);      /* one rounding */
}

/* the constants a and c of the formula from the fp32 value of delta, as oracle/perturb.py forms them */
static void constants(float delta, float *a, float *c) {
  const double d = (double)delta;
  *a = (float)(d * 0x1p-15);                  /* power-of-two scaling: exact */
  *c = (float)(1.0 - 65535.0 * (d * 0x1p-16)); /* product and difference exact in fp64 for the deltas in use: one rounding */
}

/* rows [i0, i0 + rows) of slice t of a dense tensor with n columns: x and out hold rows * n values */
void oracle_perturb_dense_rows(const float *x, float *out, int64_t n, int64_t i0, int64_t rows, int32_t t,
                               uint64_t seed, int32_t member, float delta) {
  float a, c;
  constants(delta, &a, &c);
  const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t j = 0; j < n; ++j) {
      const uint64_t e = (uint64_t)(i0 + i) * (uint64_t)n + (uint64_t)j;
      out[i * n + j] = perturbed_value(x[i * n + j], e, (uint32_t)t, member, k0, k1, a, c);
    }
}

/* nnz stored non-zeros of slice t in coordinate form */
void oracle_perturb_coo(const int64_t *row, const int64_t *col, const float *val, float *out, int64_t nnz, int64_t n,
                        int32_t t, uint64_t seed, int32_t member, float delta) {
  float a, c;
  constants(delta, &a, &c);
  const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma omp parallel for schedule(static)
  for (int64_t p = 0; p < nnz; ++p) {
    const uint64_t e = (uint64_t)row[p] * (uint64_t)n + (uint64_t)col[p];
    out[p] = perturbed_value(val[p], e, (uint32_t)t, member, k0, k1, a, c);
  }
}

/* The random start of Alg. 3's first statement as oracle/perturb.py defines it: element e = 0 .. count-1 of a
 * factor (A: e = i * k + s, R: e = (t * k + a) * k + b) is ((w >> 9) + 0.5) * 2^-23 with w the first output word of
 * the block with counter (lo32(e), hi32(e), k, (domain << 16) | member), domain 1 for A and 2 for R. */
void oracle_init_stream(float *out, int64_t count, uint32_t k, uint32_t domain, uint32_t member, uint64_t seed) {
  const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < count; ++e) {
    uint32_t w[4] = {(uint32_t)e, (uint32_t)((uint64_t)e >> 32), k, (domain << 16) | member};
    philox_block(w, k0, k1);
    out[e] = (float)(2u * (w[0] >> 9) + 1u) * 0x1p-24f;   /* an odd integer below 2^24: exact */
  }
}
