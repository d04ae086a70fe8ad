// The n x k x k products of the multiplicative-update iteration on fp32 matrix cores, for factor arrays in
// the dense path's row format [rows][q][kp] with kp a multiple of 16 (arxiv 2202.09512, Alg. 3):
//   gram16     G = A^T A (first statement of the loop) and S_t = A^T (X_t A) (ATXA), batched over members
//              and slices: a contraction over the n rows;
//   a_update16 Num = sum_t (X_t A) R_t^T + (X_t^T A) R_t, Den = A W, A <- A (*) Num (/) (Den + eps)  (Eq. 2,
//              second rule): contractions over the k columns; it also writes the operand-order copy of the
//              new A that the pass over X reads, and accumulates the next iteration's A^T A.
//              (two variants: every slice's R_t resident in LDS, or staged slice by slice).
// Both stream their inputs once.  For k <= 32 the matrix-core time is a small fraction of the memory time; at
// k = 64 the two are of equal size.
//
// v_mfma_f32_16x16x4f32: D[16x16] += A[16x4] B[4x16]; lane l supplies A[l%16][l/16] and B[l/16][l%16] and
// holds D[4*(l/16)+r][l%16] in register r.
#include "common.h"
#include "kernels.h"

namespace nnr {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------ Gram over rows
// out[(b1*q + mem)][a][c] = sum_i Y[i][mem][a] * Z_b1[i][mem][c],  a, c < k.   One wave per (batch of TB values
// of b1, mem, row split): the rows of Y are loaded once for the TB products of the batch (SAME: Z is Y, one
// product, and the rows are loaded once for both operands).
// The contraction index (the row) sits on the MFMA's K dimension: in step r lane l supplies row
// i0 + 4*r + l/16 of both operands.  A lane loads NT neighbouring columns NT*(l%16) .. +NT-1 of its row in one
// piece, so "block" u of the MFMA tiling is the set of columns {NT*j + u}: any labelling of the columns does,
// as long as the result is written back where it belongs.
template <int NT>
struct VecN {
  float v[NT];
};
template <int NT>
__device__ __forceinline__ VecN<NT> load_vec(const float* p) {
  VecN<NT> o;
  if constexpr (NT == 4) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    o.v[0] = t.x; o.v[1] = t.y; o.v[2] = t.z; o.v[3] = t.w;
  } else if constexpr (NT == 2) {
    const float2 t = *reinterpret_cast<const float2*>(p);
    o.v[0] = t.x; o.v[1] = t.y;
  } else {
#pragma unroll
    for (int u = 0; u < NT; ++u) o.v[u] = p[u];
  }
  return o;
}

template <int NT, int TB, bool SAME, bool MASKED>
__global__ void __launch_bounds__(256)
    gram16_kernel(const float* __restrict__ Y, const float* __restrict__ Z, int64_t zstride, float* __restrict__ out,
                  int64_t n, int q, int k, int nb1, int nsplit, int64_t rows_per_split,
                  const uint32_t* __restrict__ zmask, int64_t mask_words, float* __restrict__ part) {
  constexpr int kp = NT * 16;
  const int lane = threadIdx.x & 63;
  const int64_t wid = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int split = (int)(wid % nsplit);
  const int mem = (int)((wid / nsplit) % q);
  const int bat = (int)(wid / ((int64_t)nsplit * q));
  const int nbatch = (nb1 + TB - 1) / TB;
  if (bat >= nbatch) return;                       // uniform over the workgroup (the barriers below); the grid is exact
  const int b1_0 = bat * TB;
  const int l16 = lane & 15, row = lane >> 4;
  const int64_t ld = (int64_t)q * kp;
  const float* Yb = Y + (int64_t)mem * kp + NT * l16;
  const float* Zb = Z + (int64_t)mem * kp + NT * l16;
  const int64_t r_begin = split * rows_per_split;
  int64_t r_end = r_begin + rows_per_split;
  if (r_end > n) r_end = n;
  floatx4 acc[TB][NT][NT];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb)
#pragma unroll
    for (int a = 0; a < NT; ++a)
#pragma unroll
      for (int c = 0; c < NT; ++c) acc[tb][a][c] = floatx4{0.f, 0.f, 0.f, 0.f};
  // zmask (optional): bit i of batch entry b says whether row i of Z_b holds anything; rows that do not are zero and
  // are not loaded, and a row of Y that no entry of the batch needs is not loaded either.  The 16 rows of a step lie
  // in one mask word per entry (steps start at multiples of 16); the words are wave-uniform and are fetched one step
  // ahead, so that no load waits for them.
  static_assert(!(SAME && MASKED), "masks describe Z only");
  uint32_t wnext[TB];
  auto mask_fetch = [&](int64_t i0) {
    if constexpr (MASKED) {
      const int64_t w = __builtin_amdgcn_readfirstlane((int)(i0 >> 5));
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        const int b = b1_0 + tb < nb1 ? b1_0 + tb : nb1 - 1;
        wnext[tb] = zmask[(int64_t)b * mask_words + w];
      }
    }
  };
  if (r_begin < r_end) mask_fetch(r_begin);
  for (int64_t i0 = r_begin; i0 < r_end; i0 += 16) {
    VecN<NT> ya[4];
    bool ok[4];
    int64_t ic[4];
    uint32_t present[4];                           // bit tb: row r of batch entry tb is there
    if constexpr (MASKED) {
      uint32_t wcur[TB];
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) wcur[tb] = wnext[tb] >> (i0 & 31);
      if (i0 + 16 < r_end) mask_fetch(i0 + 16);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        present[r] = 0;
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
          if (b1_0 + tb < nb1) present[r] |= ((wcur[tb] >> (4 * r + row)) & 1u) << tb;
      }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t i = i0 + 4 * r + row;
      ok[r] = i < r_end;
      ic[r] = ok[r] ? i : r_end - 1;               // clamp the address, mask the value
      if constexpr (MASKED) {
        if (!ok[r]) present[r] = 0;
        if (present[r]) ya[r] = load_vec<NT>(Yb + ic[r] * ld);
        else
#pragma unroll
          for (int u = 0; u < NT; ++u) ya[r].v[u] = 0.0f;
      } else {
        present[r] = ~0u;
        ya[r] = load_vec<NT>(Yb + ic[r] * ld);
      }
    }
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      if (b1_0 + tb < nb1) {                       // wave-uniform
        VecN<NT> zb[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if constexpr (SAME) zb[r] = ya[r];
          else if (!MASKED || ((present[r] >> tb) & 1u)) zb[r] = load_vec<NT>(Zb + (int64_t)(b1_0 + tb) * zstride + ic[r] * ld);
          else
#pragma unroll
            for (int u = 0; u < NT; ++u) zb[r].v[u] = 0.0f;
        }
#pragma unroll
        for (int a = 0; a < NT; ++a)
#pragma unroll
          for (int c = 0; c < NT; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r)
              acc[tb][a][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(ok[r] ? ya[r].v[a] : 0.0f, zb[r].v[c], acc[tb][a][c],
                                                                   0, 0, 0);
      }
    }
  }
  // The four waves of the workgroup hold row ranges of the same product(s): their accumulators are summed
  // through LDS, 16 registers at a time, and every wave adds a quarter of the sums to the result.
  __shared__ float red[4][16][64];
  constexpr int NR = TB * NT * NT * 4;
  const int wave = threadIdx.x >> 6;
#pragma unroll
  for (int f0 = 0; f0 < NR; f0 += 16) {
    if (f0 > 0) __syncthreads();
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int f = f0 + j;
      if (f < NR) red[wave][j][lane] = acc[f / (NT * NT * 4)][(f / (NT * 4)) % NT][(f / 4) % NT][f % 4];
    }
    __syncthreads();
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int j = 4 * jj + wave, f = f0 + j;      // register j of this round is summed by wave j % 4
      if (f >= NR) continue;
      const float v = (red[0][j][lane] + red[1][j][lane]) + (red[2][j][lane] + red[3][j][lane]);
      const int tb = f / (NT * NT * 4), a = (f / (NT * 4)) % NT, c = (f / 4) % NT, r = f % 4;
      const int ai = NT * (4 * row + r) + a, ci = NT * l16 + c;
      if (b1_0 + tb < nb1 && ai < k && ci < k) {
        const int64_t e = ((int64_t)(b1_0 + tb) * q + mem) * k * k + ai * k + ci;
        // reproducible mode: the workgroup's share goes to its own copy (workgroups of one product: split / 4)
        if (part) part[(int64_t)(split >> 2) * nb1 * q * k * k + e] = v;
        else if (v != 0.0f) unsafeAtomicAdd(&out[e], v);
      }
    }
  }
}

template <int NT, int TB>
static hipError_t launch_gram16_t(const float* Y, const float* Z, int64_t zstride, float* out, int nb1, const Dims& d,
                                  hipStream_t s, const uint32_t* zmask, float* part, size_t part_floats) {
  const int64_t mask_words = ceil_div(d.n, 32);
  // enough waves to fill the chip (several per SIMD), at least 256 rows each so that the atomic traffic stays
  // small; the 4 waves of a workgroup are neighbouring row ranges of one product (batch)
  const int64_t units = (int64_t)ceil_div(nb1, TB) * d.q;
  int64_t nsplit = ceil_div(8192, units);
  const int64_t max_split = ceil_div(d.n, 256);
  if (nsplit > max_split) nsplit = max_split;
  nsplit = round_up(nsplit < 1 ? 1 : nsplit, 4);
  const int64_t product_floats = (int64_t)nb1 * d.q * d.k * d.k;
  if (part) {                                      // as many workgroups per product as the buffer of shares holds
    const int64_t fit = (int64_t)(part_floats / (size_t)product_floats);
    if (fit < 1) return hipErrorInvalidValue;
    if (nsplit / 4 > fit) nsplit = 4 * fit;
  }
  const int64_t rows_per_split = round_up(ceil_div(d.n, nsplit), 16);   // ranges past the last row stay empty
  const int64_t blocks = units * nsplit / 4;
  if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  if (Y == Z && nb1 == 1)
    hipLaunchKernelGGL((gram16_kernel<NT, 1, true, false>), dim3((unsigned)blocks), dim3(256), 0, s, Y, Z, zstride, out, d.n,
                       d.q, d.k, nb1, (int)nsplit, rows_per_split, nullptr, mask_words, part);
  else if (zmask)
    hipLaunchKernelGGL((gram16_kernel<NT, TB, false, true>), dim3((unsigned)blocks), dim3(256), 0, s, Y, Z, zstride, out, d.n,
                       d.q, d.k, nb1, (int)nsplit, rows_per_split, zmask, mask_words, part);
  else
    hipLaunchKernelGGL((gram16_kernel<NT, TB, false, false>), dim3((unsigned)blocks), dim3(256), 0, s, Y, Z, zstride, out, d.n,
                       d.q, d.k, nb1, (int)nsplit, rows_per_split, nullptr, mask_words, part);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && part) e = launch_reduce_parts(out, part, product_floats, nsplit / 4, product_floats, 0, s);
  return e;
}

hipError_t launch_gram16(const float* Y, const float* Z, int64_t zstride, float* out, int nb1, const Dims& d,
                         hipStream_t s, const uint32_t* zmask, float* det_part, size_t det_part_floats, bool out_cleared) {
  hipError_t e = hipSuccess;
  // the product is added into `out` (reproducible mode: overwritten): cleared here unless the caller has done so
  if (!det_part && !out_cleared) e = launch_fill_zero(out, (size_t)nb1 * d.q * d.k * d.k * sizeof(float), s);
  if (e != hipSuccess) return e;
  // a batch of products per wave when there are several (A^T X_t A over the slices) and the problem is large
  // enough to leave plenty of waves; the accumulators of a batch must fit the register file
  const bool batch = nb1 > 1 && (d.n / 256) * (int64_t)d.q * nb1 >= 32768;
  switch (d.kp / 16) {
    case 1: return batch ? launch_gram16_t<1, 4>(Y, Z, zstride, out, nb1, d, s, zmask, det_part, det_part_floats) : launch_gram16_t<1, 1>(Y, Z, zstride, out, nb1, d, s, zmask, det_part, det_part_floats);
    case 2: return batch ? launch_gram16_t<2, 2>(Y, Z, zstride, out, nb1, d, s, zmask, det_part, det_part_floats) : launch_gram16_t<2, 1>(Y, Z, zstride, out, nb1, d, s, zmask, det_part, det_part_floats);
    // 36 and 64 accumulator registers per product: batches of 2 cost more occupancy than they save, and so does
    // putting the four waves of a workgroup on four products over the same rows (both measured)
    case 3: return launch_gram16_t<3, 1>(Y, Z, zstride, out, nb1, d, s, zmask, det_part, det_part_floats);
    case 4: return launch_gram16_t<4, 1>(Y, Z, zstride, out, nb1, d, s, zmask, det_part, det_part_floats);
    default: return hipErrorInvalidValue;
  }
}

// ------------------------------------------------------------------------------------------ A rule
// A workgroup of 8 waves works on ONE member; every wave takes batches of TT 16-row tiles and loads PF
// 16-column blocks of P and Q per step, one step ahead (wide ranks: a whole slice ahead).  For every tile:
//   Num[i][c] = sum_t sum_b P_t[i][b] R_t[c][b] + Q_t[i][b] R_t[b][c]     (X_t A R_t^T + X_t^T A R_t, new R_t)
//   Den[i][c] = sum_b A[i][b] W[b][c]
//   A[i][c]  <- A[i][c] * Num[i][c] / (Den[i][c] + eps)
// The contraction index b sits on the MFMA's K dimension: lane l loads the float4 [i0 + l%16][4*(l/16) .. +3]
// of a row-format tile, which is the left operand of the four steps r.  The right operands come from
// copies of R_t in operand order, Rp[..][lane][r] = R_t[c = l%16][b = 4*(l/16) + r] and Rq[..][lane][r] =
// R_t[b][c] per (16 x 16) block pair (zero outside k x k); the workgroup stages them in LDS one slice ahead,
// so that the waves read them from there instead of from L2 for every tile.  The denominator runs through the
// same pipeline as one more "slice": left operand A, right operand W (put into operand order while it is
// staged), accumulated apart from the numerator.
// (X_t^T A) R_t equals the paper's X_t^T (A R_t) by associativity; the k x k matrix W collects the denominator's
// core over all slices so that the n-sized product A W is formed once.
constexpr int kAupdWaves = 8;

// WPS: waves per SIMD the register allocation is made for (second launch bound)
template <int NT, int TT, int PF, bool FUSE_G, int WPS>
__global__ void __launch_bounds__(kAupdWaves * 64, WPS)
    a_update16_kernel(float* __restrict__ A_int, float* __restrict__ A_op, const float* __restrict__ P,
                      const float* __restrict__ Q, int64_t pq_slice_stride, const float* __restrict__ Rp,
                      const float* __restrict__ Rq, const float* __restrict__ W, float* __restrict__ G, Dims d,
                      float eps, int batches_per_wave) {
  constexpr int kp = NT * 16;
  constexpr int RB = NT * NT * 64;                 // float4 per operand copy of one slice (Rp or Rq)
  constexpr int STGN = (2 * RB + kAupdWaves * 64 - 1) / (kAupdWaves * 64);  // float4 staged per thread and slice
  extern __shared__ __attribute__((aligned(16))) float lds_raw[];
  float4* rlds = reinterpret_cast<float4*>(lds_raw);   // [2 buffers][Rp | Rq][NT*NT][64]
  const int k = d.k, q = d.q, m = d.m;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int mem = blockIdx.y;
  const int l16 = lane & 15, row = lane >> 4;
  const int64_t ld = (int64_t)q * kp;
  const int64_t n_tiles = (d.n + 15) / 16;         // tiles that hold rows of the matrix
  const float4* Rp4 = reinterpret_cast<const float4*>(Rp) + (int64_t)mem * m * RB;
  const float4* Rq4 = reinterpret_cast<const float4*>(Rq) + (int64_t)mem * m * RB;
  const float* Wq = W + (int64_t)mem * k * k;

  constexpr int GN = FUSE_G ? NT : 1;
  floatx4 gacc[GN][GN];
#pragma unroll
  for (int a = 0; a < GN; ++a)
#pragma unroll
    for (int c = 0; c < GN; ++c) gacc[a][c] = floatx4{0.f, 0.f, 0.f, 0.f};

  // staging of slice t's operands: every thread moves up to STGN float4 (2*RB in all) through registers
  static_assert(STGN <= 4, "staging registers");
  float4 st0, st1, st2, st3;                       // named registers (an array would be placed in scratch memory)
  st0 = st1 = st2 = st3 = float4{0.f, 0.f, 0.f, 0.f};
  auto stage_src = [&](int t, int u) -> const float4* {
    int e = u * (kAupdWaves * 64) + tid;
    if (e > 2 * RB - 1) e = 2 * RB - 1;            // surplus threads repeat the last element
    return e < RB ? Rp4 + (int64_t)t * RB + e : Rq4 + (int64_t)t * RB + (e - RB);
  };
  auto stage_dst = [&](int buf, int u) -> float4* {
    int e = u * (kAupdWaves * 64) + tid;
    if (e > 2 * RB - 1) e = 2 * RB - 1;
    return rlds + buf * 2 * RB + e;
  };
  auto stage_load = [&](int t) {
    st0 = *stage_src(t, 0);
    if constexpr (STGN > 1) st1 = *stage_src(t, 1);
    if constexpr (STGN > 2) st2 = *stage_src(t, 2);
    if constexpr (STGN > 3) st3 = *stage_src(t, 3);
  };
  // the denominator's right operand: W[b = 16*bb + 4*(l/16) + r][c = 16*cb + l%16], the layout of Rq,
  // stored where a slice's Rp goes (the second half of the buffer is not read for it)
  auto w_piece = [&](int u) -> float4 {
    const int e = u * (kAupdWaves * 64) + tid;
    const int ln = e & 63, cb = (e >> 6) % NT, bb = (e >> 6) / NT;
    const int c = cb * 16 + (ln & 15), b = bb * 16 + 4 * (ln >> 4);
    const bool in = e < RB && c < k;
    const float* wp = Wq + b * k + c;
    float4 w;                                      // (no array: it would be placed in scratch memory)
    w.x = in && b + 0 < k ? wp[0] : 0.0f;
    w.y = in && b + 1 < k ? wp[k] : 0.0f;
    w.z = in && b + 2 < k ? wp[2 * k] : 0.0f;
    w.w = in && b + 3 < k ? wp[3 * k] : 0.0f;
    return w;
  };
  auto stage_load_w = [&]() {
    st0 = w_piece(0);
    if constexpr (STGN > 1) st1 = w_piece(1);
    if constexpr (STGN > 2) st2 = w_piece(2);
    if constexpr (STGN > 3) st3 = w_piece(3);
  };
  auto stage_store = [&](int buf) {
    *stage_dst(buf, 0) = st0;
    if constexpr (STGN > 1) *stage_dst(buf, 1) = st1;
    if constexpr (STGN > 2) *stage_dst(buf, 2) = st2;
    if constexpr (STGN > 3) *stage_dst(buf, 3) = st3;
  };

  for (int it = 0; it < batches_per_wave; ++it) {
    // the batches of one workgroup iteration are neighbours: 8 waves x TT tiles of consecutive rows
    const int64_t batch = ((int64_t)blockIdx.x * batches_per_wave + it) * kAupdWaves + wave;
    const int64_t tile0 = batch * TT;
    const bool have = tile0 < n_tiles;             // wave-uniform; waves without tiles still stage and sync
    int64_t irc[TT];
    bool row_ok[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      const int64_t irow = (tile0 + tt) * 16 + l16;  // the row whose float4 pieces this lane loads
      row_ok[tt] = irow < d.n;
      irc[tt] = row_ok[tt] ? irow : d.n - 1;
    }
    floatx4 num[TT][NT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int c = 0; c < NT; ++c) num[tt][c] = floatx4{0.f, 0.f, 0.f, 0.f};

    __syncthreads();                               // the previous batch's last slice has been consumed
    stage_load(0);
    stage_store(0);
    // P and Q pieces of step u = t*(NT/PF) + g (PF neighbouring 16-column blocks per step), one step ahead
    constexpr int SPS = NT / PF;                   // steps per slice
    float4 pn[TT][PF], qn[TT][PF];
    auto pq_fetch = [&](int u) {
      const int t = u / SPS, g = u % SPS;
      // the denominator's step (t == m) reads A itself; its second piece is loaded too, and not used, so that
      // both cases are the same straight-line code
      const float* ps = t < m ? P + (int64_t)t * pq_slice_stride : A_int;
      const float* qs = t < m ? Q + (int64_t)t * pq_slice_stride : A_int;
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) {
        const int64_t off = irc[tt] * ld + (int64_t)mem * kp + g * PF * 16 + 4 * row;
#pragma unroll
        for (int f = 0; f < PF; ++f) {
          pn[tt][f] = *reinterpret_cast<const float4*>(ps + off + f * 16);
          qn[tt][f] = *reinterpret_cast<const float4*>(qs + off + f * 16);
        }
      }
    };
    if (have) pq_fetch(0);
    __syncthreads();
    floatx4 den[TT][NT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int c = 0; c < NT; ++c) den[tt][c] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int t = 0; t <= m; ++t) {                 // t == m: A W
      if (t + 1 < m) stage_load(t + 1);
      if (t + 1 == m) stage_load_w();
      const float4* rb = rlds + (t & 1) * 2 * RB + lane;
      if (have) {
#pragma unroll
        for (int g = 0; g < SPS; ++g) {
          float4 pc[TT][PF], qc[TT][PF];
#pragma unroll
          for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int f = 0; f < PF; ++f) {
              pc[tt][f] = row_ok[tt] ? pn[tt][f] : float4{0.f, 0.f, 0.f, 0.f};
              qc[tt][f] = row_ok[tt] ? qn[tt][f] : float4{0.f, 0.f, 0.f, 0.f};
            }
          if (t * SPS + g + 1 < (m + 1) * SPS) pq_fetch(t * SPS + g + 1);
          if (t < m) {
#pragma unroll
            for (int f = 0; f < PF; ++f) {
              const int bb = g * PF + f;
#pragma unroll
              for (int cb = 0; cb < NT; ++cb) {
                const float4 rp = rb[(bb * NT + cb) * 64];
                const float4 rq = rb[RB + (bb * NT + cb) * 64];
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                  num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].x, rp.x, num[tt][cb], 0, 0, 0);
                  num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].y, rp.y, num[tt][cb], 0, 0, 0);
                  num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].z, rp.z, num[tt][cb], 0, 0, 0);
                  num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].w, rp.w, num[tt][cb], 0, 0, 0);
                  num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(qc[tt][f].x, rq.x, num[tt][cb], 0, 0, 0);
                  num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(qc[tt][f].y, rq.y, num[tt][cb], 0, 0, 0);
                  num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(qc[tt][f].z, rq.z, num[tt][cb], 0, 0, 0);
                  num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(qc[tt][f].w, rq.w, num[tt][cb], 0, 0, 0);
                }
              }
            }
          } else {
#pragma unroll
            for (int f = 0; f < PF; ++f) {
              const int bb = g * PF + f;
#pragma unroll
              for (int cb = 0; cb < NT; ++cb) {
                const float4 w4 = rb[(bb * NT + cb) * 64];
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                  den[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].x, w4.x, den[tt][cb], 0, 0, 0);
                  den[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].y, w4.y, den[tt][cb], 0, 0, 0);
                  den[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].z, w4.z, den[tt][cb], 0, 0, 0);
                  den[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].w, w4.w, den[tt][cb], 0, 0, 0);
                }
              }
            }
          }
        }
      }
      if (t < m) {
        stage_store((t + 1) & 1);                  // the other buffer: read last in slice t - 1, before the barrier
        __syncthreads();
      }
    }
    if (!have) continue;
    // the element-wise rule in accumulator order: register r of lane l is element
    // [i0 + 4*(l/16) + r][16*cb + l%16]
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      const int64_t tile = tile0 + tt, i0 = tile * 16;
      if (tile >= n_tiles) break;
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
          const float v = ok ? aold * num[tt][cb][r] / (den[tt][cb][r] + eps) : 0.0f;
          anew[cb][r] = v;
          if (ok) *ap = v;
        }
        if (A_op)
          reinterpret_cast<float4*>(A_op)[((tile * q + mem) * NT + cb) * 64 + lane] =
              float4{anew[cb][0], anew[cb][1], anew[cb][2], anew[cb][3]};
      }
      // next iteration's A^T A: the new tile is at once the left and the right operand (rows on the K dimension)
      if constexpr (FUSE_G) {
#pragma unroll
        for (int a = 0; a < NT; ++a)
#pragma unroll
          for (int c = 0; c < NT; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r)
              gacc[a][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(anew[a][r], anew[c][r], gacc[a][c], 0, 0, 0);
      }
    }
  }
  if constexpr (!FUSE_G) return;
  if (!G) return;                                  // (reproducible mode: a Gram pass with ordered sums follows instead)
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

// The same rule when the operands of ALL slices of a member (and W) fit in LDS together: the workgroup stages
// them once, and from then on its waves run independently, with no barrier: each takes a unit of TT 16-row
// tiles at a time and keeps the loads of P, Q (and A, for the denominator) one step ahead, across units too.
template <int NT, int TT, int PF, int WAVES, bool FUSE_G, bool MASKED>
__global__ void __launch_bounds__(WAVES * 64)
    a_update16_resident_kernel(float* __restrict__ A_int, float* __restrict__ A_op, const float* __restrict__ P,
                               const float* __restrict__ Q, int64_t pq_slice_stride, const float* __restrict__ Rp,
                               const float* __restrict__ Rq, const float* __restrict__ W, float* __restrict__ G,
                               Dims d, float eps, int units_per_wave, const uint32_t* __restrict__ pmask,
                               const uint32_t* __restrict__ qmask, int64_t mask_words, int64_t nblocks,
                               int members_together) {
  constexpr int kp = NT * 16;
  constexpr int RB = NT * NT * 64;                 // float4 per operand copy of one slice (Rp or Rq)
  constexpr int SPS = NT / PF;                     // steps per slice: PF neighbouring 16-column blocks per step
  extern __shared__ __attribute__((aligned(16))) float lds_raw[];
  float4* rlds = reinterpret_cast<float4*>(lds_raw);   // [m][Rp | Rq][NT*NT][64], then W [NT*NT][64]
  const int k = d.k, q = d.q, m = d.m;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Workgroups go to the 8 XCDs round-robin.  The workgroups of one range of rows (one per member) follow each other on
  // ONE XCD: a member's piece of a row is kp * 4 bytes of the row's q * kp * 4, so for narrow ranks the members' pieces
  // share cache lines, which the second member then finds in that XCD's L2.
  // (When a member's piece is whole lines, kp = 32 or 64, there is nothing to share and member after member is the
  // better order by a few per cent: members_together == 0.)
  const int64_t nb8 = (nblocks + 7) & ~(int64_t)7, slot = blockIdx.x >> 3;
  const int mem = members_together ? (int)(slot % q) : (int)(blockIdx.x / nb8);
  const int64_t bx = members_together ? (slot / q) * 8 + (blockIdx.x & 7) : blockIdx.x % nb8;   // the range of rows
  if (bx >= nblocks) return;                                   // (uniform over the workgroup, before any barrier)
  const int l16 = lane & 15, row = lane >> 4;
  const int64_t ld = (int64_t)q * kp;
  const int64_t n_tiles = (d.n + 15) / 16;
  {
    const float4* Rp4 = reinterpret_cast<const float4*>(Rp) + (int64_t)mem * m * RB;
    const float4* Rq4 = reinterpret_cast<const float4*>(Rq) + (int64_t)mem * m * RB;
    const float* Wq = W + (int64_t)mem * k * k;
    for (int e = tid; e < m * 2 * RB; e += WAVES * 64) {
      const int t = e / (2 * RB), r = e % (2 * RB);
      rlds[e] = r < RB ? Rp4[(int64_t)t * RB + r] : Rq4[(int64_t)t * RB + r - RB];
    }
    // W[b = 16*bb + 4*(l/16) + r][c = 16*cb + l%16]: the layout of Rq
    for (int e = tid; e < RB; e += WAVES * 64) {
      const int ln = e & 63, cb = (e >> 6) % NT, bb = (e >> 6) / NT;
      const int c = cb * 16 + (ln & 15), b = bb * 16 + 4 * (ln >> 4);
      const float* wp = Wq + b * k + c;
      float4 w;
      w.x = c < k && b + 0 < k ? wp[0] : 0.0f;
      w.y = c < k && b + 1 < k ? wp[k] : 0.0f;
      w.z = c < k && b + 2 < k ? wp[2 * k] : 0.0f;
      w.w = c < k && b + 3 < k ? wp[3 * k] : 0.0f;
      rlds[m * 2 * RB + e] = w;
    }
  }
  __syncthreads();                                 // the only barrier

  constexpr int GN = FUSE_G ? NT : 1;
  floatx4 gacc[GN][GN];
#pragma unroll
  for (int a = 0; a < GN; ++a)
#pragma unroll
    for (int c = 0; c < GN; ++c) gacc[a][c] = floatx4{0.f, 0.f, 0.f, 0.f};

  // the units of one workgroup iteration are neighbours
  const int64_t unit_first = bx * units_per_wave * WAVES + wave;
  const int64_t n_units = (n_tiles + TT - 1) / TT;
  const int nsteps = (m + 1) * SPS;                // step u = t*SPS + g; t == m: the denominator, with A as P
  float4 pn[TT][PF], qn[TT][PF];
  // Presence masks (sparse tensors): rows of X_t A / X_t^T A without any stored entry of X_t behind them are zero and
  // are not loaded.  The 16 rows of a unit lie in one mask word per slice and product; lane t holds the word of slice
  // t's X_t A, lane 32 + t that of its X_t^T A, loaded a whole unit ahead, and a step reads its two words with a lane
  // broadcast, so that no load of P or Q waits for a mask.  (Units of more than one tile, or more than 32 slices: no masks.)
  static_assert(!MASKED || TT == 1, "masks need units of one tile");
  uint32_t mcur = ~0u, mnxt = ~0u;                 // this unit's words, the next unit's
  auto mask_load = [&](int64_t unit) -> uint32_t {
    if constexpr (!MASKED) return ~0u;
    const int t = lane & 31;
    const uint32_t* src = (lane < 32) ? pmask : qmask;
    if (t >= m || !src) return ~0u;
    return src[(int64_t)t * mask_words + ((unit * 16) >> 5)];
  };
  auto fetch = [&](int64_t unit, int u, uint32_t mv) {
    const int t = u / SPS, g = u % SPS;
    // the denominator's step (t == m) reads A itself and needs no second piece
    const float* ps = t < m ? P + (int64_t)t * pq_slice_stride : A_int;
    const float* qs = t < m ? Q + (int64_t)t * pq_slice_stride : A_int;
    uint32_t wp = ~0u, wq = t < m ? ~0u : 0u;
    if constexpr (MASKED) {
      if (t < m) {
        wp = __builtin_amdgcn_readlane(mv, t & 31);
        wq = __builtin_amdgcn_readlane(mv, 32 + (t & 31));
      }
    }
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      int64_t irow = (unit * TT + tt) * 16 + l16;  // the row whose float4 pieces this lane loads
      if (irow > d.n - 1) irow = d.n - 1;          // rows past the end: a copy of the last row, never written back
      const int64_t off = irow * ld + (int64_t)mem * kp + g * PF * 16 + 4 * row;
      if constexpr (MASKED) {
        const bool hp = (wp >> (irow & 31)) & 1u;
        const bool hq = (wq >> (irow & 31)) & 1u;
#pragma unroll
        for (int f = 0; f < PF; ++f) {
          pn[tt][f] = hp ? *reinterpret_cast<const float4*>(ps + off + f * 16) : float4{0.f, 0.f, 0.f, 0.f};
          qn[tt][f] = hq ? *reinterpret_cast<const float4*>(qs + off + f * 16) : float4{0.f, 0.f, 0.f, 0.f};
        }
      } else {
#pragma unroll
        for (int f = 0; f < PF; ++f) {
          pn[tt][f] = *reinterpret_cast<const float4*>(ps + off + f * 16);
          qn[tt][f] = *reinterpret_cast<const float4*>(qs + off + f * 16);   // (t == m: loaded, not used)
        }
      }
    }
  };
  if (unit_first < n_units) {
    mcur = mask_load(unit_first);
    fetch(unit_first, 0, mcur);
  }
  for (int it = 0; it < units_per_wave; ++it) {
    const int64_t unit = unit_first + (int64_t)it * WAVES;
    if (unit >= n_units) break;
    const bool has_next = it + 1 < units_per_wave && unit + WAVES < n_units;
    if (has_next) mnxt = mask_load(unit + WAVES);  // a whole unit ahead of its first use
    floatx4 num[TT][NT], den[TT][NT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int c = 0; c < NT; ++c) {
        num[tt][c] = floatx4{0.f, 0.f, 0.f, 0.f};
        den[tt][c] = floatx4{0.f, 0.f, 0.f, 0.f};
      }
    for (int t = 0; t <= m; ++t) {
      const float4* rb = rlds + t * 2 * RB + lane;
#pragma unroll
      for (int g = 0; g < SPS; ++g) {
        // this step's pieces; a row of the result depends on the same row of P and Q only, so that rows past
        // the end need no masking
        float4 pc[TT][PF], qc[TT][PF];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
          for (int f = 0; f < PF; ++f) {
            pc[tt][f] = pn[tt][f];
            qc[tt][f] = qn[tt][f];
          }
        const int un = t * SPS + g + 1;
        if (un < nsteps) fetch(unit, un, mcur);
        else if (has_next) fetch(unit + WAVES, 0, mnxt);
        if (t < m) {
#pragma unroll
          for (int f = 0; f < PF; ++f) {
            const int bb = g * PF + f;
#pragma unroll
            for (int cb = 0; cb < NT; ++cb) {
              const float4 rp = rb[(bb * NT + cb) * 64];
              const float4 rq = rb[RB + (bb * NT + cb) * 64];
#pragma unroll
              for (int tt = 0; tt < TT; ++tt) {
                num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].x, rp.x, num[tt][cb], 0, 0, 0);
                num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].y, rp.y, num[tt][cb], 0, 0, 0);
                num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].z, rp.z, num[tt][cb], 0, 0, 0);
                num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].w, rp.w, num[tt][cb], 0, 0, 0);
                num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(qc[tt][f].x, rq.x, num[tt][cb], 0, 0, 0);
                num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(qc[tt][f].y, rq.y, num[tt][cb], 0, 0, 0);
                num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(qc[tt][f].z, rq.z, num[tt][cb], 0, 0, 0);
                num[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(qc[tt][f].w, rq.w, num[tt][cb], 0, 0, 0);
              }
            }
          }
        } else {
#pragma unroll
          for (int f = 0; f < PF; ++f) {
            const int bb = g * PF + f;
#pragma unroll
            for (int cb = 0; cb < NT; ++cb) {
              const float4 w4 = rb[(bb * NT + cb) * 64];
#pragma unroll
              for (int tt = 0; tt < TT; ++tt) {
                den[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].x, w4.x, den[tt][cb], 0, 0, 0);
                den[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].y, w4.y, den[tt][cb], 0, 0, 0);
                den[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].z, w4.z, den[tt][cb], 0, 0, 0);
                den[tt][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(pc[tt][f].w, w4.w, den[tt][cb], 0, 0, 0);
              }
            }
          }
        }
      }
    }
    // the element-wise rule in accumulator order: register r of lane l is element [i0 + 4*(l/16) + r][16*cb + l%16]
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      const int64_t tile = unit * TT + tt, i0 = tile * 16;
      if (tile >= n_tiles) break;
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
          const float v = ok ? aold * num[tt][cb][r] / (den[tt][cb][r] + eps) : 0.0f;
          anew[cb][r] = v;
          if (ok) *ap = v;
        }
        if (A_op)
          reinterpret_cast<float4*>(A_op)[((tile * q + mem) * NT + cb) * 64 + lane] =
              float4{anew[cb][0], anew[cb][1], anew[cb][2], anew[cb][3]};
      }
      // next iteration's A^T A: the new tile is at once the left and the right operand (rows on the K dimension)
      if constexpr (FUSE_G) {
#pragma unroll
        for (int a = 0; a < NT; ++a)
#pragma unroll
          for (int c = 0; c < NT; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r)
              gacc[a][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(anew[a][r], anew[c][r], gacc[a][c], 0, 0, 0);
      }
    }
    mcur = mnxt;
  }
  if constexpr (!FUSE_G) return;
  if (!G) return;                                  // (reproducible mode: a Gram pass with ordered sums follows instead)
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

constexpr size_t kAupdLdsMax = 156 * 1024;        // of the 160 KB a workgroup may have (rank 48 with 8 slices: 153 KB)

template <int NT, int TT, int PF, int WAVES, bool FUSE_G, bool MASKED>
static hipError_t launch_a_update16_resident_m(float* A_int, float* A_op, const float* P, const float* Q,
                                             int64_t pq_slice_stride, const float* Rp, const float* Rq, const float* W,
                                             float* G, const Dims& d, float eps, hipStream_t s, const uint32_t* pmask,
                                             const uint32_t* qmask) {
  const size_t lds = (size_t)(2 * d.m + 1) * NT * NT * 64 * sizeof(float4);
  if (lds > kAupdLdsMax) return hipErrorInvalidValue;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)a_update16_resident_kernel<NT, TT, PF, WAVES, FUSE_G, MASKED>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kAupdLdsMax);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int64_t n_tiles = (d.n + 15) / 16;
  // about a thousand workgroups per launch when there is that much work; the staging is then paid once for many
  // tiles, and the atomic traffic of A^T A stays small
  const int64_t n_units = ceil_div(n_tiles, TT);
  int64_t per_wave = ceil_div(n_units * d.q, (int64_t)WAVES * 1024);
  if (per_wave < 1) per_wave = 1;
  if (per_wave > 256) per_wave = 256;
  const int64_t blocks = ceil_div(n_units, per_wave * WAVES);
  if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  const int64_t grid_x = 8 * ceil_div(blocks, 8) * d.q;          // see the kernel: (row range, member) -> workgroup number
  if (grid_x > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  dim3 grid((unsigned)grid_x);
  hipLaunchKernelGGL((a_update16_resident_kernel<NT, TT, PF, WAVES, FUSE_G, MASKED>), grid, dim3(WAVES * 64), lds, s, A_int,
                     A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, eps, (int)per_wave, pmask, qmask, ceil_div(d.n, 32), blocks,
                     (NT * 64) % 128 != 0 && d.q > 1 ? 1 : 0);
  return hipGetLastError();
}

// with masks (a sparse tensor of at most 32 slices: one lane per slice and product holds a mask word) or without
template <int NT, int TT, int PF, int WAVES, bool FUSE_G>
static hipError_t launch_a_update16_resident(float* A_int, float* A_op, const float* P, const float* Q,
                                             int64_t pq_slice_stride, const float* Rp, const float* Rq, const float* W,
                                             float* G, const Dims& d, float eps, hipStream_t s, const uint32_t* pmask,
                                             const uint32_t* qmask) {
  if (pmask && d.m <= 32)
    return launch_a_update16_resident_m<NT, TT, PF, WAVES, FUSE_G, true>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d,
                                                                         eps, s, pmask, qmask);
  return launch_a_update16_resident_m<NT, TT, PF, WAVES, FUSE_G, false>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d,
                                                                        eps, s, nullptr, nullptr);
}

template <int NT, int TT, int PF, bool FUSE_G, int WPS = 2>
static hipError_t launch_a_update16_t(float* A_int, float* A_op, const float* P, const float* Q, int64_t pq_slice_stride,
                                      const float* Rp, const float* Rq, const float* W, float* G, const Dims& d,
                                      float eps, hipStream_t s) {
  constexpr size_t lds = (size_t)2 * 2 * NT * NT * 64 * sizeof(float4);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)a_update16_kernel<NT, TT, PF, FUSE_G, WPS>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int64_t n_tiles = (d.n + 15) / 16;
  const int64_t batches = ceil_div(n_tiles, TT);                 // one per wave and workgroup iteration
  // several workgroups per CU and member; more batches per wave keep the atomic traffic of A^T A small
  int64_t per_wave = ceil_div(batches * d.q, (int64_t)kAupdWaves * 2048);
  if (per_wave < 1) per_wave = 1;
  if (per_wave > 32) per_wave = 32;
  const int64_t blocks = ceil_div(batches, per_wave * kAupdWaves);
  if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  dim3 grid((unsigned)blocks, (unsigned)d.q);
  hipLaunchKernelGGL((a_update16_kernel<NT, TT, PF, FUSE_G, WPS>), grid, dim3(kAupdWaves * 64), lds, s, A_int, A_op, P, Q,
                     pq_slice_stride, Rp, Rq, W, G, d, eps, (int)per_wave);
  return hipGetLastError();
}

hipError_t launch_a_update16(float* A_int, float* A_op, const float* P, const float* Q, int64_t pq_slice_stride,
                             const float* Rp, const float* Rq, const float* W, float* G_out, const Dims& d, float eps,
                             hipStream_t s, const uint32_t* pmask, const uint32_t* qmask, float* det_part,
                             size_t det_part_floats) {
  // G receives the new A^T A: clear it first (the R rule, which read the old one, has been enqueued before)
  hipError_t e = launch_fill_zero(G_out, (size_t)d.q * d.k * d.k * sizeof(float), s);
  if (e != hipSuccess) return e;
  // reproducible mode: the rule's kernels do not accumulate A^T A (atomic additions); a Gram pass does, in order
  float* G = det_part ? nullptr : G_out;
  const bool gram_pass_always = det_part != nullptr;
  const int nt = d.kp / 16;
  const size_t lds_all = (size_t)(2 * d.m + 1) * nt * nt * 64 * sizeof(float4);
  bool fused_g = false;                            // the kernel that ran has accumulated A^T A itself
  if (lds_all <= kAupdLdsMax) {
    // every slice's operands in LDS at once; 16 waves where only one workgroup fits a compute unit
    const bool big = lds_all > 64 * 1024;
#define NNR_RES(NT, PF, FG)                                                                                            \
  (big ? launch_a_update16_resident<NT, 1, PF, 16, FG>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, eps, s, pmask, qmask)     \
       : launch_a_update16_resident<NT, 1, PF, 8, FG>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, eps, s, pmask, qmask))
    switch (nt) {
      case 1: e = NNR_RES(1, 1, true); fused_g = true; break;
      case 2: e = NNR_RES(2, 2, true); fused_g = true; break;
      case 3:   // 12 waves: the 16-wave variant does not fit 128 registers without spilling
        e = big ? launch_a_update16_resident<3, 1, 3, 12, false>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, eps, s, pmask, qmask)
                : launch_a_update16_resident<3, 1, 3, 8, false>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, eps, s, pmask, qmask);
        break;
      case 4:   // whole slices ahead and 12 waves: more bytes in flight than 16 waves of half slices
        e = big ? launch_a_update16_resident<4, 1, 4, 12, false>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, eps, s, pmask, qmask)
                : launch_a_update16_resident<4, 1, 2, 8, false>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, eps, s, pmask, qmask);
        break;
      default: return hipErrorInvalidValue;
    }
#undef NNR_RES
  } else {
    // many slices: their operands are staged slice by slice
    // small problems: one tile per wave, so that there are enough waves to fill the chip
    const bool small = ((d.n + 15) / 16) * (int64_t)d.q < 16384;
    switch (nt) {
      case 1:
        e = small ? launch_a_update16_t<1, 1, 1, true>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, eps, s)
                  : launch_a_update16_t<1, 4, 1, true>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, eps, s);
        fused_g = true;
        break;
      case 2:
        e = small ? launch_a_update16_t<2, 1, 2, true>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, eps, s)
                  : launch_a_update16_t<2, 4, 1, true>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, eps, s);
        fused_g = true;
        break;
      // wide ranks: the k x k accumulators of A^T A no longer fit beside the numerators; a Gram pass follows
      case 3:
        e = launch_a_update16_t<3, 1, 3, false>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, eps, s);
        break;
      case 4:
        e = launch_a_update16_t<4, 1, 2, false, 4>(A_int, A_op, P, Q, pq_slice_stride, Rp, Rq, W, G, d, eps, s);
        break;
      default: return hipErrorInvalidValue;
    }
  }
  if (e != hipSuccess) return e;
  if (fused_g && !gram_pass_always) return hipSuccess;
  // wide ranks (and the reproducible mode): the Gram pass is a launch of its own
  return launch_gram16(A_int, A_int, 0, G_out, 1, d, s, nullptr, det_part, det_part_floats);
}

}  // namespace nnr
