// The n x k x k products of the multiplicative-update iteration on fp32 matrix cores, for factor arrays in
// the dense path's row format [rows][q][kp] with kp a multiple of 16 (arxiv 2202.09512, Alg. 3):
//   gram16     G = A^T A (first statement of the loop) and S_t = A^T (X_t A) (ATXA), batched over members
//              and slices: a contraction over the n rows;
//   a_update16 Num = sum_t (X_t A) R_t^T + (X_t^T A) R_t, Den = A W, A <- A (*) Num (/) (Den + eps)  (Eq. 2,
//              second rule): contractions over the k columns; it also writes the operand-order copy of the
//              new A that the pass over X reads, and accumulates the next iteration's A^T A.
// Both stream their inputs once; the matrix-core time is a small fraction of the memory time.
//
// v_mfma_f32_16x16x4f32: D[16x16] += A[16x4] B[4x16]; lane l supplies A[l%16][l/16] and B[l/16][l%16] and
// holds D[4*(l/16)+r][l%16] in register r.
#include "common.h"
#include "kernels.h"

namespace nnr {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------ Gram over rows
// out[(b1*q + mem)][a][c] = sum_i Y[i][mem][a] * Z_b1[i][mem][c],  a, c < k.   One wave per (b1, mem, row split).
// The contraction index (the row) sits on the MFMA's K dimension: in step r lane l supplies row
// i0 + 4*r + l/16 of both operands, column l%16 of a 16-column block.
template <int NT>
__global__ void __launch_bounds__(256)
    gram16_kernel(const float* __restrict__ Y, const float* __restrict__ Z, int64_t zstride, float* __restrict__ out,
                  int64_t n, int q, int k, int nb1, int nsplit, int64_t rows_per_split) {
  const int kp = NT * 16;
  const int lane = threadIdx.x & 63;
  const int64_t wid = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int split = (int)(wid % nsplit);
  const int mem = (int)((wid / nsplit) % q);
  const int b1 = (int)(wid / ((int64_t)nsplit * q));
  if (b1 >= nb1) return;
  const int l16 = lane & 15, row = lane >> 4;
  const int64_t ld = (int64_t)q * kp;
  const float* Yb = Y + (int64_t)mem * kp + l16;
  const float* Zb = Z + b1 * zstride + (int64_t)mem * kp + l16;
  const int64_t r_begin = split * rows_per_split;
  int64_t r_end = r_begin + rows_per_split;
  if (r_end > n) r_end = n;
  floatx4 acc[NT][NT];
#pragma unroll
  for (int a = 0; a < NT; ++a)
#pragma unroll
    for (int c = 0; c < NT; ++c) acc[a][c] = floatx4{0.f, 0.f, 0.f, 0.f};
  for (int64_t i0 = r_begin; i0 < r_end; i0 += 16) {
    float ya[NT][4], zb[NT][4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t i = i0 + 4 * r + row;
      const bool ok = i < r_end;
      const int64_t ic = ok ? i : r_end - 1;       // clamp the address, mask the value
#pragma unroll
      for (int b = 0; b < NT; ++b) {
        const float yv = Yb[ic * ld + b * 16], zv = Zb[ic * ld + b * 16];
        ya[b][r] = ok ? yv : 0.0f;
        zb[b][r] = ok ? zv : 0.0f;
      }
    }
#pragma unroll
    for (int a = 0; a < NT; ++a)
#pragma unroll
      for (int c = 0; c < NT; ++c)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[a][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(ya[a][r], zb[c][r], acc[a][c], 0, 0, 0);
  }
  float* ob = out + ((int64_t)b1 * q + mem) * k * k;
#pragma unroll
  for (int a = 0; a < NT; ++a)
#pragma unroll
    for (int c = 0; c < NT; ++c)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int ai = a * 16 + 4 * row + r, ci = c * 16 + l16;
        const float v = acc[a][c][r];
        if (ai < k && ci < k && v != 0.0f) unsafeAtomicAdd(&ob[ai * k + ci], v);
      }
}

hipError_t launch_gram16(const float* Y, const float* Z, int64_t zstride, float* out, int nb1, const Dims& d,
                         hipStream_t s) {
  hipError_t e = launch_fill_zero(out, (size_t)nb1 * d.q * d.k * d.k * sizeof(float), s);
  if (e != hipSuccess) return e;
  // enough waves to fill the chip (several per SIMD), at least 256 rows each so that the atomic traffic stays small
  const int64_t units = (int64_t)nb1 * d.q;
  int64_t nsplit = ceil_div(8192, units);
  const int64_t max_split = ceil_div(d.n, 256);
  if (nsplit > max_split) nsplit = max_split;
  if (nsplit < 1) nsplit = 1;
  const int64_t rows_per_split = round_up(ceil_div(d.n, nsplit), 16);
  nsplit = ceil_div(d.n, rows_per_split);
  const int64_t waves = units * nsplit;
  dim3 grid((unsigned)ceil_div(waves, 4));
#define NNR_GRAM16(NTV) \
  hipLaunchKernelGGL(gram16_kernel<NTV>, grid, dim3(256), 0, s, Y, Z, zstride, out, d.n, d.q, d.k, nb1, (int)nsplit, rows_per_split)
  switch (d.kp / 16) {
    case 1: NNR_GRAM16(1); break;
    case 2: NNR_GRAM16(2); break;
    case 3: NNR_GRAM16(3); break;
    case 4: NNR_GRAM16(4); break;
    default: return hipErrorInvalidValue;
  }
#undef NNR_GRAM16
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------ A rule
// One wave per (member, run of 16-row tiles).  For every tile:
//   Num[i][c] = sum_t sum_b P_t[i][b] R_t[c][b] + Q_t[i][b] R_t[b][c]     (X_t A R_t^T + X_t^T A R_t, new R_t)
//   Den[i][c] = sum_b A[i][b] W[b][c]
//   A[i][c]  <- A[i][c] * Num[i][c] / (Den[i][c] + eps)
// The contraction index b sits on the MFMA's K dimension: lane l loads the float4 [i0 + l%16][4*(l/16) .. +3]
// of a row-format tile, which is the left operand of the four steps r.  The right operands come from
// copies of R_t and W in operand order: Rp[..][lane][r] = R_t[c = l%16][b = 4*(l/16) + r] and
// Rq[..][lane][r] = R_t[b][c] per (16 x 16) block pair, zero outside k x k.
// (X_t^T A) R_t equals the paper's X_t^T (A R_t) by associativity; the k x k matrix W collects the denominator's
// core over all slices so that the n-sized product A W is formed once.
template <int NT>
__global__ void __launch_bounds__(256)
    a_update16_kernel(float* __restrict__ A_int, float* __restrict__ A_op, const float* __restrict__ P,
                      const float* __restrict__ Q, int64_t pq_slice_stride, const float* __restrict__ Rp,
                      const float* __restrict__ Rq, const float* __restrict__ W, float* __restrict__ G, Dims d,
                      float eps, int tiles_per_wave, int runs) {
  const int kp = NT * 16, k = d.k, q = d.q;
  const int lane = threadIdx.x & 63;
  const int64_t wid = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int mem = (int)(wid % q);                 // neighbouring waves take neighbouring members of the same rows
  const int64_t run = wid / q;
  if (run >= runs) return;
  const int l16 = lane & 15, row = lane >> 4;
  const int64_t ld = (int64_t)q * kp;
  const int64_t n_tiles = d.n_pad / 16;
  const float4* Rp4 = reinterpret_cast<const float4*>(Rp) + (int64_t)mem * d.m * NT * NT * 64 + lane;
  const float4* Rq4 = reinterpret_cast<const float4*>(Rq) + (int64_t)mem * d.m * NT * NT * 64 + lane;
  // W in operand order: Wop[b-block][c-block][r] = W[16*bb + 4*row + r][16*cb + l16]
  float4 wop[NT][NT];
  {
    const float* Wq = W + (int64_t)mem * k * k;
#pragma unroll
    for (int bb = 0; bb < NT; ++bb)
#pragma unroll
      for (int cb = 0; cb < NT; ++cb) {
        float w4[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int b = bb * 16 + 4 * row + r, c = cb * 16 + l16;
          w4[r] = (b < k && c < k) ? Wq[b * k + c] : 0.0f;
        }
        wop[bb][cb] = float4{w4[0], w4[1], w4[2], w4[3]};
      }
  }
  floatx4 gacc[NT][NT];
#pragma unroll
  for (int a = 0; a < NT; ++a)
#pragma unroll
    for (int c = 0; c < NT; ++c) gacc[a][c] = floatx4{0.f, 0.f, 0.f, 0.f};

  for (int tw = 0; tw < tiles_per_wave; ++tw) {
    const int64_t tile = run * tiles_per_wave + tw;
    if (tile >= n_tiles) break;
    const int64_t i0 = tile * 16;
    if (i0 >= d.n) {                              // padding rows of A stay zero; so does their operand copy
      continue;
    }
    const int64_t irow = i0 + l16;                // the row whose float4 pieces this lane loads
    const bool row_ok = irow < d.n;
    const int64_t irc = row_ok ? irow : d.n - 1;
    floatx4 num[NT], den[NT];
#pragma unroll
    for (int c = 0; c < NT; ++c) {
      num[c] = floatx4{0.f, 0.f, 0.f, 0.f};
      den[c] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    for (int t = 0; t < d.m; ++t) {
      const float* Pt = P + (int64_t)t * pq_slice_stride + irc * ld + (int64_t)mem * kp + 4 * row;
      const float* Qt = Q + (int64_t)t * pq_slice_stride + irc * ld + (int64_t)mem * kp + 4 * row;
#pragma unroll
      for (int bb = 0; bb < NT; ++bb) {
        float4 p4 = *reinterpret_cast<const float4*>(Pt + bb * 16);
        float4 q4 = *reinterpret_cast<const float4*>(Qt + bb * 16);
        if (!row_ok) p4 = q4 = float4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cb = 0; cb < NT; ++cb) {
          const float4 rp = Rp4[((int64_t)t * NT * NT + bb * NT + cb) * 64];
          const float4 rq = Rq4[((int64_t)t * NT * NT + bb * NT + cb) * 64];
          num[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(p4.x, rp.x, num[cb], 0, 0, 0);
          num[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(p4.y, rp.y, num[cb], 0, 0, 0);
          num[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(p4.z, rp.z, num[cb], 0, 0, 0);
          num[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(p4.w, rp.w, num[cb], 0, 0, 0);
          num[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(q4.x, rq.x, num[cb], 0, 0, 0);
          num[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(q4.y, rq.y, num[cb], 0, 0, 0);
          num[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(q4.z, rq.z, num[cb], 0, 0, 0);
          num[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(q4.w, rq.w, num[cb], 0, 0, 0);
        }
      }
    }
    // A W
    float* Arow = A_int + irc * ld + (int64_t)mem * kp + 4 * row;
#pragma unroll
    for (int bb = 0; bb < NT; ++bb) {
      float4 a4 = *reinterpret_cast<const float4*>(Arow + bb * 16);
      if (!row_ok) a4 = float4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int cb = 0; cb < NT; ++cb) {
        den[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.x, wop[bb][cb].x, den[cb], 0, 0, 0);
        den[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.y, wop[bb][cb].y, den[cb], 0, 0, 0);
        den[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.z, wop[bb][cb].z, den[cb], 0, 0, 0);
        den[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.w, wop[bb][cb].w, den[cb], 0, 0, 0);
      }
    }
    // element-wise rule in accumulator order: register r of lane l is element [i0 + 4*(l/16) + r][16*cb + l%16]
    float anew[NT][4];
#pragma unroll
    for (int cb = 0; cb < NT; ++cb) {
      const int c = cb * 16 + l16;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int64_t i = i0 + 4 * row + r;
        const bool ok = i < d.n && c < k;
        float* ap = A_int + (ok ? i : i0) * ld + (int64_t)mem * kp + (ok ? c : 0);
        const float aold = *ap;
        const float v = ok ? aold * num[cb][r] / (den[cb][r] + eps) : 0.0f;
        anew[cb][r] = v;
        if (ok) *ap = v;
      }
      if (A_op)
        reinterpret_cast<float4*>(A_op)[((tile * q + mem) * NT + cb) * 64 + lane] =
            float4{anew[cb][0], anew[cb][1], anew[cb][2], anew[cb][3]};
    }
    // next iteration's A^T A: the new tile is at once the left and the right operand (rows on the K dimension)
#pragma unroll
    for (int a = 0; a < NT; ++a)
#pragma unroll
      for (int c = 0; c < NT; ++c)
#pragma unroll
        for (int r = 0; r < 4; ++r) gacc[a][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(anew[a][r], anew[c][r], gacc[a][c], 0, 0, 0);
  }
  float* Gq = G + (int64_t)mem * k * k;
#pragma unroll
  for (int a = 0; a < NT; ++a)
#pragma unroll
    for (int c = 0; c < NT; ++c)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int ai = a * 16 + 4 * row + r, ci = c * 16 + l16;
        const float v = gacc[a][c][r];
        if (ai < k && ci < k && v != 0.0f) unsafeAtomicAdd(&Gq[ai * k + ci], v);
      }
}

hipError_t launch_a_update16(float* A_int, float* A_op, const float* P, const float* Q, int64_t pq_slice_stride,
                             const float* Rp, const float* Rq, const float* W, float* G, const Dims& d, float eps,
                             hipStream_t s) {
  // G receives the new A^T A: clear it first (the R rule, which read the old one, has been enqueued before)
  hipError_t e = launch_fill_zero(G, (size_t)d.q * d.k * d.k * sizeof(float), s);
  if (e != hipSuccess) return e;
  const int64_t n_tiles = d.n_pad / 16;
  // several waves per SIMD; a run of tiles per wave keeps the atomic traffic of A^T A small
  int64_t tiles_per_wave = ceil_div(n_tiles * d.q, 8192);
  if (tiles_per_wave < 1) tiles_per_wave = 1;
  if (tiles_per_wave > 16) tiles_per_wave = 16;
  const int64_t runs = ceil_div(n_tiles, tiles_per_wave);
  const int64_t waves = runs * d.q;
  dim3 grid((unsigned)ceil_div(waves, 4));
#define NNR_AUPD16(NTV)                                                                                           \
  hipLaunchKernelGGL(a_update16_kernel<NTV>, grid, dim3(256), 0, s, A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, \
                     eps, (int)tiles_per_wave, (int)runs)
  switch (d.kp / 16) {
    case 1: NNR_AUPD16(1); break;
    case 2: NNR_AUPD16(2); break;
    case 3: NNR_AUPD16(3); break;
    case 4: NNR_AUPD16(4); break;
    default: return hipErrorInvalidValue;
  }
#undef NNR_AUPD16
  return hipGetLastError();
}

}  // namespace nnr
