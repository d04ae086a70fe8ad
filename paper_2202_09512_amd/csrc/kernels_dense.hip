// Dense pass over X: for every slice t and ensemble member r, in ONE read of X_t,
//   P = X^r_t A^r   (Alg. 3: XA)      and      Q = X^r_t^T A^r   (Alg. 3: XTAR before the R_t factor),
// with X^r = X (*) Delta^r generated on the fly (Alg. 4) from a counter-based random stream, so the
// perturbed tensors are never stored and X is read once for all members of a group.
//
// Mapping to CDNA4.  The contraction runs on fp32 matrix cores, v_mfma_f32_16x16x4f32
// (D[16x16] += A[16x4] B[4x16]; lane l supplies A[l%16][l/16] and B[l/16][l%16], and holds
// D[4*(l/16)+r][l%16] in register r).  The perturbed X tile is the MFMA's left operand, built in
// registers by the lane that loaded the element; the factor rows are the right operand.  A workgroup
// of 8 waves owns a panel of 8*JB*16 columns and walks down a chunk of rows, 16 at a time:
//   - Q accumulators (columns of the wave's own 16*JB columns) stay in registers for the whole chunk;
//   - P accumulators (the 16 rows of the step) are summed over the 8 waves through LDS every step
//     and added to P in memory (other panels add to the same rows).
// One Philox block yields eight 16-bit draws, one per member of the group, so the generator's
// integer work is shared by up to 8 members.
#include "common.h"
#include "kernels.h"

namespace nnr {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 8;  // two waves per SIMD, so that one wave's generator work overlaps the other's MFMAs

// Load the "row" orientation of one 16 x 16 tile: lane (l16, row) gets X[i0 + l16][j0 + 4*row + r], r = 0..3.
// full: the tile lies inside the chunk and the matrix, rows are 16-byte aligned (one vector load, no mask).
__device__ __forceinline__ void load_tile(float (&x)[4], const float* __restrict__ xtile, bool full, int n32,
                                          int rows_left, int cols_left, int l16, int row) {
  if (full) {
    const float4 v = *reinterpret_cast<const float4*>(xtile + (l16 * n32 + 4 * row));
    x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
  } else {
    // clamp the address into the valid part of the tile, then mask: no divergent branches
    const int ic = l16 < rows_left ? l16 : rows_left - 1;
    const bool rok = l16 < rows_left;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int j = 4 * row + r;
      const int jc = j < cols_left ? j : cols_left - 1;
      const float v = xtile[ic * n32 + jc];
      x[r] = (rok && j < cols_left) ? v : 0.0f;
    }
  }
}

constexpr int kTLD = 20;  // row pitch (floats) of the 16 x 16 transposition tile in LDS: conflict-free reads

// Dynamic LDS layout (floats):
//   [0, 2*BQ)                         right operands of the Q products for the current / next step, shared by all
//                                     waves: bq[buf][(qq*NT+nt)][lane][4]  (one 16-byte read per product group)
//   [2*BQ + wave*WBUF, ... + WBUF)    per wave: transposition tiles [QB][16][kTLD]; after the step's products the
//                                     same space stages the wave's P accumulators [QB*NT*4][64]
template <int NT, int QB, int JB, bool PERTURB>
__global__ void __launch_bounds__(kWaves * 64)
    dense_stream_kernel(const float* __restrict__ X, const float* __restrict__ A_int, float* __restrict__ P,
                        float* __restrict__ Q, int64_t n, int q, int kp, int qfirst, int ngroups,
                        int64_t rows_per_chunk, uint32_t k0, uint32_t k1, float dscaled, int vec_ok) {
  constexpr int TJ = kWaves * JB * 16;
  constexpr int NG = QB * NT;                       // product groups (member, 16-column block)
  constexpr int NACC = NG * 4;                      // P accumulator registers per lane
  constexpr int TBUF = QB * 16 * kTLD;              // floats of transposition space per wave
  constexpr int PBUF = NACC * 64;                   // floats of P staging per wave
  constexpr int WBUF = TBUF > PBUF ? TBUF : PBUF;
  constexpr int BQ = NG * 64 * 4;                   // floats of one Q-operand buffer
  extern __shared__ __attribute__((aligned(16))) float lds[];
  float* bqbuf = lds;
  float* wbase = lds + 2 * BQ;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, row = lane >> 4;
  const int t = blockIdx.z / ngroups, grp = blockIdx.z % ngroups;
  // Members [q0, q0 + QB) share one Philox block (QB divides 8 and q0 is a multiple of QB).  Members
  // at or beyond q (a rounded-up tail group) are computed on finite padding and never written.
  const int q0 = qfirst + grp * QB;
  const int qb = (q - q0) < QB ? (q - q0) : QB;
  const uint32_t sub = (uint32_t)(q0 >> 3);         // Philox block index of this member group
  const int hoff = QB == 8 ? 0 : (q0 & 7);          // first 16-bit half used by the group
  const int64_t jw0 = (int64_t)blockIdx.x * TJ + (int64_t)wave * JB * 16;
  const int64_t i_begin = (int64_t)blockIdx.y * rows_per_chunk;
  int64_t i_end = i_begin + rows_per_chunk;
  if (i_end > n) i_end = n;
  const float* Xt = X + (int64_t)t * n * n;
  float* Pt = P + (int64_t)t * n * q * kp;
  float* Qt = Q + (int64_t)t * n * q * kp;
  const int arow = q * kp;                          // floats per entity row of A_int
  const int n32 = (int)n;
  float* tbuf = wbase + wave * WBUF;
  const bool active = jw0 < n;                      // wave-uniform: the wave owns at least one column

  // right operands of the P products: rows j of A for the wave's own columns, kept for the whole chunk
  float bP[JB][4][QB][NT];
#pragma unroll
  for (int jb = 0; jb < JB; ++jb) {
    const int64_t j0 = jw0 + jb * 16;               // padding rows of A exist and are zero
    const float* base = A_int + (j0 < n ? j0 : 0) * arow + q0 * kp + (4 * row * arow + l16);
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int qq = 0; qq < QB; ++qq)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) bP[jb][r][qq][nt] = base[r * arow + qq * kp + nt * 16];
  }

  floatx4 qacc[JB][QB][NT];
#pragma unroll
  for (int jb = 0; jb < JB; ++jb)
#pragma unroll
    for (int qq = 0; qq < QB; ++qq)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) qacc[jb][qq][nt] = floatx4{0.f, 0.f, 0.f, 0.f};

  // Q-operand staging: wave g (< NG) fetches rows i0 + 4*row + r of A for product group g, one float4 per lane
  const bool bq_loader = wave < NG;
  const int bq_src = ((wave / NT) * kp + (wave % NT) * 16) + 4 * row * arow + l16;   // + i0*arow + q0*kp
  float4 bq_next = float4{0.f, 0.f, 0.f, 0.f};
  auto bq_fetch = [&](int64_t i0) {
    if (bq_loader) {
      const float* src = A_int + i0 * arow + q0 * kp + bq_src;
      bq_next = float4{src[0], src[arow], src[2 * arow], src[3 * arow]};
    }
  };
  auto bq_store = [&](int buf) {
    if (bq_loader) *reinterpret_cast<float4*>(bqbuf + buf * BQ + (wave * 64 + lane) * 4) = bq_next;
  };
  // X tiles one step ahead
  float xnext[JB][4];
  auto x_fetch = [&](int64_t i0) {
    const int rows_left = (int)(i_end - i0 < 16 ? i_end - i0 : 16);
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
      const int64_t j0 = jw0 + jb * 16;
      const bool in = j0 < n;
      const int cols_left = in ? (int)(n - j0 < 16 ? n - j0 : 16) : 1;
      const float* xtile = Xt + i0 * n + (in ? j0 : 0);
      load_tile(xnext[jb], xtile, vec_ok && rows_left == 16 && cols_left == 16, n32, rows_left, cols_left, l16, row);
      if (!in) xnext[jb][0] = xnext[jb][1] = xnext[jb][2] = xnext[jb][3] = 0.0f;
    }
  };
  if (i_begin < i_end) {
    x_fetch(i_begin);
    bq_fetch(i_begin);
    bq_store(0);
  }
  __syncthreads();

  int step = 0;
  for (int64_t i0 = i_begin; i0 < i_end; i0 += 16, ++step) {
    float xcur[JB][4];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
      for (int r = 0; r < 4; ++r) xcur[jb][r] = xnext[jb][r];
    const bool more = i0 + 16 < i_end;
    if (more) {
      x_fetch(i0 + 16);
      bq_fetch(i0 + 16);
    }
    const float* bq = bqbuf + (step & 1) * BQ + lane * 4;

    floatx4 pacc[QB][NT];
#pragma unroll
    for (int qq = 0; qq < QB; ++qq)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) pacc[qq][nt] = floatx4{0.f, 0.f, 0.f, 0.f};

    if (active) {
#pragma unroll
      for (int jb = 0; jb < JB; ++jb) {
        const int64_t j0 = jw0 + jb * 16;
        // ---- the generator: one Philox block per element serves all QB members
        u32x4 w[4];
        if (PERTURB) {
          const uint64_t e0 = (uint64_t)(i0 + l16) * (uint64_t)n + (uint64_t)(j0 + 4 * row);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const uint64_t e = e0 + (uint64_t)r;
            w[r] = philox4x32_10((uint32_t)e, (uint32_t)(e >> 32), (uint32_t)t, sub, k0, k1);
          }
        }
        // ---- per member: perturbed tile in "row" orientation -> P products; park it in LDS for the transpose
#pragma unroll
        for (int qq = 0; qq < QB; ++qq) {
          float xq[4];
#pragma unroll
          for (int r = 0; r < 4; ++r)
            xq[r] = PERTURB ? xcur[jb][r] * delta_from_block(w[r], hoff + qq, dscaled) : xcur[jb][r];
          *reinterpret_cast<float4*>(tbuf + (qq * 16 + l16) * kTLD + 4 * row) = float4{xq[0], xq[1], xq[2], xq[3]};
#pragma unroll
          for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              pacc[qq][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(xq[r], bP[jb][r][qq][nt], pacc[qq][nt], 0, 0, 0);
        }
        // ---- "column" orientation read back from LDS: lane (l16, row) gets X^q[i0 + 4*row + r][j0 + l16]
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int qq = 0; qq < QB; ++qq) {
          float xt[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) xt[r] = tbuf[(qq * 16 + 4 * row + r) * kTLD + l16];
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const float4 b = *reinterpret_cast<const float4*>(bq + (qq * NT + nt) * 256);
            qacc[jb][qq][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(xt[0], b.x, qacc[jb][qq][nt], 0, 0, 0);
            qacc[jb][qq][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(xt[1], b.y, qacc[jb][qq][nt], 0, 0, 0);
            qacc[jb][qq][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(xt[2], b.z, qacc[jb][qq][nt], 0, 0, 0);
            qacc[jb][qq][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(xt[3], b.w, qacc[jb][qq][nt], 0, 0, 0);
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
    }
    // ---- sum the step's P over the waves through LDS (plain stores, then a spread-out sum), add to memory
    __syncthreads();  // every wave is done with its transposition tiles and with this step's Q operands
    if (active) {
#pragma unroll
      for (int qq = 0; qq < QB; ++qq)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) tbuf[((qq * NT + nt) * 4 + rr) * 64 + lane] = pacc[qq][nt][rr];
    }
    if (more) bq_store((step + 1) & 1);
    __syncthreads();
    for (int e = tid; e < PBUF; e += kWaves * 64) {
      float v = 0.0f;
#pragma unroll
      for (int wv = 0; wv < kWaves; ++wv) {
        const bool wact = (int64_t)blockIdx.x * TJ + (int64_t)wv * JB * 16 < n;   // uniform
        if (wact) v += wbase[wv * WBUF + e];
      }
      const int idx = e >> 6, ln = e & 63;
      const int rr = idx & 3, nt = (idx >> 2) % NT, qq = idx / (4 * NT);
      const int64_t i = i0 + 4 * (ln >> 4) + rr;
      if (qq < qb && i < i_end && v != 0.0f)
        unsafeAtomicAdd(&Pt[(i * q + q0 + qq) * kp + nt * 16 + (ln & 15)], v);
    }
    __syncthreads();  // the staging space becomes transposition space again
  }
  // ---- flush Q (this wave's columns, summed over the chunk's rows)
#pragma unroll
  for (int jb = 0; jb < JB; ++jb) {
    const int64_t j0 = jw0 + jb * 16;
#pragma unroll
    for (int qq = 0; qq < QB; ++qq)
      if (qq < qb) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            const int64_t j = j0 + 4 * row + rr;
            const float v = qacc[jb][qq][nt][rr];
            if (j < n && v != 0.0f) unsafeAtomicAdd(&Qt[(j * q + q0 + qq) * kp + nt * 16 + l16], v);
          }
      }
  }
}

template <int NT, int QB, int JB>
constexpr size_t stream_lds_bytes() {
  constexpr int NG = QB * NT;
  constexpr int TBUF = QB * 16 * kTLD, PBUF = NG * 4 * 64;
  constexpr int WBUF = TBUF > PBUF ? TBUF : PBUF;
  return (size_t)(2 * NG * 256 + kWaves * WBUF) * sizeof(float);
}

const char* dense_stream_kernel_name() { return "dense_stream_kernel"; }

template <int NT, int QB, int JB>
static hipError_t launch_stream_t(const float* X, const float* A_int, float* P, float* Q, const Dims& d, int qfirst,
                                  int ngroups, uint64_t seed, float delta, hipStream_t s) {
  static_assert(QB * NT <= kWaves, "one wave per product group stages the shared Q operands");
  constexpr int TJ = kWaves * JB * 16;
  constexpr size_t lds = stream_lds_bytes<NT, QB, JB>();
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)dense_stream_kernel<NT, QB, JB, true>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void*)dense_stream_kernel<NT, QB, JB, false>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int64_t n_panels = ceil_div(d.n, TJ);
  // enough workgroups for 256 CUs (one workgroup per CU at a time) with some slack, chunks of at least 128 rows
  const int64_t base = n_panels * d.m * ngroups;
  int64_t n_chunks = ceil_div(1024, base);
  const int64_t max_chunks = ceil_div(d.n, 128);
  if (n_chunks > max_chunks) n_chunks = max_chunks;
  if (n_chunks < 1) n_chunks = 1;
  const int64_t rows_per_chunk = round_up(ceil_div(d.n, n_chunks), 16);
  n_chunks = ceil_div(d.n, rows_per_chunk);
  const int vec_ok = (d.n % 4 == 0) && (((uintptr_t)X & 15) == 0);
  dim3 grid((unsigned)n_panels, (unsigned)n_chunks, (unsigned)(d.m * ngroups));
  if (delta != 0.0f)
    hipLaunchKernelGGL((dense_stream_kernel<NT, QB, JB, true>), grid, dim3(kWaves * 64), lds, s, X, A_int, P, Q, d.n,
                       d.q, d.kp, qfirst, ngroups, rows_per_chunk, (uint32_t)seed, (uint32_t)(seed >> 32),
                       delta * 0x1p-16f, vec_ok);
  else
    hipLaunchKernelGGL((dense_stream_kernel<NT, QB, JB, false>), grid, dim3(kWaves * 64), lds, s, X, A_int, P, Q, d.n,
                       d.q, d.kp, qfirst, ngroups, rows_per_chunk, (uint32_t)seed, (uint32_t)(seed >> 32), 0.0f,
                       vec_ok);
  return hipGetLastError();
}

// Members per group so that (members) x (16-column blocks) = 8 product groups: 8 members for k <= 16,
// 4 for k <= 32, 2 for k <= 64 (3 blocks: 6 groups).
static int group_members(int kp) { return kp <= 16 ? 8 : (kp <= 32 ? 4 : 2); }

DensePlan dense_stream_plan(const Dims& d) {
  const int qbig = group_members(d.kp);
  DensePlan pl;
  pl.full_groups = d.q / qbig;
  pl.full_qb = qbig;
  pl.tail_members = d.q - pl.full_groups * qbig;
  pl.tail_qb = pl.tail_members == 0 ? 0 : 1;
  while (pl.tail_qb < pl.tail_members) pl.tail_qb *= 2;
  return pl;
}

template <int NT, int QB>
static hipError_t launch_tail(const float* X, const float* A_int, float* P, float* Q, const Dims& d, int qf,
                              uint64_t seed, float delta, hipStream_t s) {
  if constexpr (QB * NT <= kWaves)
    return launch_stream_t<NT, QB, 2>(X, A_int, P, Q, d, qf, 1, seed, delta, s);
  else
    return hipErrorInvalidValue;
}

template <int NT>
static hipError_t launch_stream_nt(const float* X, const float* A_int, float* P, float* Q, const Dims& d, int part,
                                   uint64_t seed, float delta, hipStream_t s) {
  constexpr int QBIG = NT == 1 ? 8 : (NT == 2 ? 4 : 2);
  const DensePlan pl = dense_stream_plan(d);
  if (part == 0) {
    if (pl.full_groups == 0) return hipSuccess;
    return launch_stream_t<NT, QBIG, 2>(X, A_int, P, Q, d, 0, pl.full_groups, seed, delta, s);
  }
  const int qf = pl.full_groups * QBIG;
  switch (pl.tail_qb) {
    case 0: return hipSuccess;
    case 1: return launch_tail<NT, 1>(X, A_int, P, Q, d, qf, seed, delta, s);
    case 2: return launch_tail<NT, 2>(X, A_int, P, Q, d, qf, seed, delta, s);
    case 4: return launch_tail<NT, 4>(X, A_int, P, Q, d, qf, seed, delta, s);
    default: return launch_tail<NT, 8>(X, A_int, P, Q, d, qf, seed, delta, s);
  }
}

hipError_t launch_dense_stream(const float* X, const float* A_int, float* P, float* Q, const Dims& d, int part,
                               uint64_t seed, float delta, hipStream_t s) {
  switch (d.kp / 16) {
    case 1: return launch_stream_nt<1>(X, A_int, P, Q, d, part, seed, delta, s);
    case 2: return launch_stream_nt<2>(X, A_int, P, Q, d, part, seed, delta, s);
    case 3: return launch_stream_nt<3>(X, A_int, P, Q, d, part, seed, delta, s);
    case 4: return launch_stream_nt<4>(X, A_int, P, Q, d, part, seed, delta, s);
    default: return hipErrorInvalidValue;
  }
}

// ------------------------------------------------------------------------------------------ Alg. 4 made explicit
__global__ void dense_perturb_kernel(const float* __restrict__ X, float* __restrict__ out, int64_t n, int m,
                                     int member, uint32_t k0, uint32_t k1, float dscaled, int perturb) {
  const int64_t per = n * n;
  const int64_t total = per * m;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int t = (int)(idx / per);
    const uint64_t e = (uint64_t)(idx % per);
    float v = X[idx];
    if (perturb) {
      const u32x4 w = philox4x32_10((uint32_t)e, (uint32_t)(e >> 32), (uint32_t)t, (uint32_t)(member >> 3), k0, k1);
      v *= delta_from_block(w, member & 7, dscaled);
    }
    out[idx] = v;
  }
}

hipError_t launch_dense_perturb(const float* X, float* out, int64_t n, int m, int member, uint64_t seed,
                                float delta, hipStream_t s) {
  int64_t blocks = ceil_div(n * n * m, 256);
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(dense_perturb_kernel, dim3((unsigned)blocks), dim3(256), 0, s, X, out, n, m, member,
                     (uint32_t)seed, (uint32_t)(seed >> 32), delta * 0x1p-16f, delta != 0.0f ? 1 : 0);
  return hipGetLastError();
}

// sum_t ||X^r_t||_F^2 for every member (the constant term of the expanded objective of Eq. 1)
__global__ void __launch_bounds__(256) dense_xnorm_kernel(const float* __restrict__ X, double* __restrict__ xn,
                                                          int64_t n, int m, int q, uint32_t k0, uint32_t k1,
                                                          float dscaled, int perturb) {
  __shared__ double red[4];
  const int64_t per = n * n;
  const int64_t total = per * m;
  for (int b = 0; b < (q + 7) / 8; ++b) {
    double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int qb = (q - 8 * b) < 8 ? (q - 8 * b) : 8;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x) {
      const int t = (int)(idx / per);
      const uint64_t e = (uint64_t)(idx % per);
      const float v = X[idx];
      u32x4 w{0, 0, 0, 0};
      if (perturb) w = philox4x32_10((uint32_t)e, (uint32_t)(e >> 32), (uint32_t)t, (uint32_t)b, k0, k1);
#pragma unroll
      for (int qq = 0; qq < 8; ++qq)
        if (qq < qb) {
          const float xq = perturb ? v * delta_from_block(w, qq, dscaled) : v;
          acc[qq] += (double)xq * (double)xq;
        }
    }
#pragma unroll
    for (int qq = 0; qq < 8; ++qq) {
      if (qq < qb) {  // block-uniform
        double v = acc[qq];
        for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
        __syncthreads();
        if (threadIdx.x == 0) atomicAdd(&xn[8 * b + qq], red[0] + red[1] + red[2] + red[3]);
      }
    }
  }
}

hipError_t launch_dense_xnorm(const float* X, double* xn, int64_t n, int m, int q, uint64_t seed, float delta,
                              hipStream_t s) {
  int64_t blocks = ceil_div(n * n * m, 256 * 8);
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(dense_xnorm_kernel, dim3((unsigned)blocks), dim3(256), 0, s, X, xn, n, m, q, (uint32_t)seed,
                     (uint32_t)(seed >> 32), delta * 0x1p-16f, delta != 0.0f ? 1 : 0);
  return hipGetLastError();
}

}  // namespace nnr
