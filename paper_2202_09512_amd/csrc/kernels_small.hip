// Small kernels of the multiplicative-update iteration: initialisation, generic Gram products, the R rule of
// Eq. 2 (arxiv 2202.09512), layout conversion, medians and the R-only regression loop.
#include "common.h"
#include "kernels.h"

namespace nnr {

// ------------------------------------------------------------------------------------------ fill
__global__ void fill_zero_kernel(uint32_t* p, size_t nwords) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < nwords; i += stride) p[i] = 0u;
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  const size_t nwords = bytes / 4;  // all buffers are multiples of 4 bytes
  int blocks = (int)((nwords + 255) / 256);
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, s, (uint32_t*)p, nwords);
  return hipGetLastError();
}

// blockIdx.y: which buffer
__global__ void fill_zero_multi_kernel(FillList fl) {
  uint32_t* p = (uint32_t*)fl.p[blockIdx.y];
  const size_t nwords = fl.bytes[blockIdx.y] / 4;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < nwords; i += stride) p[i] = 0u;
}

hipError_t launch_fill_zero_multi(const FillList& fl, hipStream_t s) {
  if (fl.count == 0) return hipSuccess;
  size_t most = 0;
  for (int i = 0; i < fl.count; ++i) most = fl.bytes[i] > most ? fl.bytes[i] : most;
  size_t blocks = (most / 4 + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(fill_zero_multi_kernel, dim3((unsigned)blocks, (unsigned)fl.count), dim3(256), 0, s, fl);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------ ordered sums
template <typename T>
__global__ void __launch_bounds__(256) reduce_parts_kernel(T* __restrict__ out, const T* __restrict__ parts, int64_t count,
                                                           int64_t nparts, int64_t stride, int accumulate) {
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += (int64_t)gridDim.x * blockDim.x) {
    T sum = accumulate ? out[e] : T(0);
    for (int64_t p = 0; p < nparts; ++p) sum += parts[p * stride + e];   // always in this order
    out[e] = sum;
  }
}

hipError_t launch_reduce_parts(float* out, const float* parts, int64_t count, int64_t nparts, int64_t stride,
                               int accumulate, hipStream_t s) {
  if (count <= 0) return hipSuccess;
  int64_t blocks = (count + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(reduce_parts_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, s, out, parts, count, nparts, stride,
                     accumulate);
  return hipGetLastError();
}

hipError_t launch_reduce_parts_f64(double* out, const double* parts, int64_t count, int64_t nparts, int64_t stride,
                                   int accumulate, hipStream_t s) {
  if (count <= 0) return hipSuccess;
  int64_t blocks = (count + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(reduce_parts_kernel<double>, dim3((unsigned)blocks), dim3(256), 0, s, out, parts, count, nparts,
                     stride, accumulate);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------ init
// Alg. 3 step 1: A = rand(n, k), R = rand(m, k, k), a different stream per member.
__global__ void init_A_kernel(float* A_int, Dims d, uint32_t k0, uint32_t k1) {
  const int64_t total = d.n_pad * d.q * d.kp;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int c = (int)(idx % d.kp);
    const int r = (int)((idx / d.kp) % d.q);
    const int64_t i = idx / ((int64_t)d.kp * d.q);
    float v = 0.0f;
    if (i < d.n && c < d.k) {
      // the model that column c belongs to: its rank kb and the column's index in it
      const int off = c < d.ksplit ? 0 : d.ksplit, kb = d.ksplit == 0 ? d.k : (c < d.ksplit ? d.ksplit : d.k - d.ksplit);
      const uint64_t e = (uint64_t)i * (uint64_t)kb + (uint64_t)(c - off);
      const u32x4 w = philox4x32_10((uint32_t)e, (uint32_t)(e >> 32), (uint32_t)kb, (1u << 16) | (uint32_t)r, k0, k1);
      v = unit_open(w.x);
    }
    A_int[idx] = v;
  }
}

__global__ void init_R_kernel(float* R, Dims d, uint32_t k0, uint32_t k1) {
  const int64_t per = (int64_t)d.m * d.k * d.k;
  const int64_t total = per * d.q;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int r = (int)(idx / per);
    uint64_t e = (uint64_t)(idx % per);
    int kb = d.k;
    bool inside = true;
    if (d.ksplit > 0) {  // two models: each block is the R of its own rank, the off-diagonal blocks are zero
      const int b = (int)(e % d.k), a = (int)((e / d.k) % d.k), t = (int)(e / ((uint64_t)d.k * d.k));
      const int off = a < d.ksplit ? 0 : d.ksplit;
      kb = a < d.ksplit ? d.ksplit : d.k - d.ksplit;
      inside = (a < d.ksplit) == (b < d.ksplit);
      e = ((uint64_t)t * kb + (uint64_t)(a - off)) * kb + (uint64_t)(b - off);
    }
    const u32x4 w = philox4x32_10((uint32_t)e, (uint32_t)(e >> 32), (uint32_t)kb, (2u << 16) | (uint32_t)r, k0, k1);
    R[idx] = inside ? unit_open(w.x) : 0.0f;
  }
}

static int grid_for(int64_t total, int block = 256, int cap = 16384) {
  int64_t b = (total + block - 1) / block;
  if (b < 1) b = 1;
  if (b > cap) b = cap;
  return (int)b;
}

hipError_t launch_init_factors(float* A_int, float* R, const Dims& d, uint64_t seed, hipStream_t s) {
  const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
  hipLaunchKernelGGL(init_A_kernel, dim3(grid_for(d.n_pad * d.q * d.kp)), dim3(256), 0, s, A_int, d, k0, k1);
  hipLaunchKernelGGL(init_R_kernel, dim3(grid_for((int64_t)d.q * d.m * d.k * d.k)), dim3(256), 0, s, R, d, k0, k1);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------ layout
__global__ void to_internal_kernel(float* E_int, const float* A_api, Dims d) {
  const int64_t total = d.n_pad * d.q * d.kp;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int c = (int)(idx % d.kp);
    const int r = (int)((idx / d.kp) % d.q);
    const int64_t i = idx / ((int64_t)d.kp * d.q);
    E_int[idx] = (i < d.n && c < d.k) ? A_api[((int64_t)r * d.n + i) * d.k + c] : 0.0f;
  }
}

__global__ void copy_kernel(float* dst, const float* src, int64_t total) {
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x)
    dst[idx] = src[idx];
}

hipError_t launch_to_internal(float* E_int, const float* A_api, const Dims& d, hipStream_t s) {
  hipLaunchKernelGGL(to_internal_kernel, dim3(grid_for(d.n_pad * d.q * d.kp)), dim3(256), 0, s, E_int, A_api, d);
  return hipGetLastError();
}

hipError_t launch_import_factors(float* A_int, float* R, const float* A_api, const float* R_api, const Dims& d,
                                 hipStream_t s) {
  hipError_t e = launch_to_internal(A_int, A_api, d, s);
  if (e != hipSuccess) return e;
  const int64_t total = (int64_t)d.q * d.m * d.k * d.k;
  hipLaunchKernelGGL(copy_kernel, dim3(grid_for(total)), dim3(256), 0, s, R, R_api, total);
  return hipGetLastError();
}

// Final normalisation (section "Multiplicative Update Algorithm"): A_:,s / ||A_:,s||, R_t <- D R_t D.
// The squared norms are the diagonal of G = A^T A.  A zero column is left alone.
__device__ __forceinline__ float col_norm(const float* G, int r, int c, int k, int normalised) {
  if (!normalised) return 1.0f;
  const float g = G[((int64_t)r * k + c) * k + c];
  return g > 0.0f ? sqrtf(g) : 1.0f;
}

// The model in columns [off, off + kb) of the internal arrays goes to A_api[q][n][kb], R_api[q][m][kb][kb].
__global__ void export_A_kernel(float* A_api, const float* A_int, const float* G, int normalised, Dims d, int off,
                                int kb) {
  const int64_t total = (int64_t)d.q * d.n * kb;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int c = (int)(idx % kb);
    const int64_t i = (idx / kb) % d.n;
    const int r = (int)(idx / ((int64_t)kb * d.n));
    A_api[idx] = A_int[(i * d.q + r) * d.kp + off + c] / col_norm(G, r, off + c, d.k, normalised);
  }
}

__global__ void export_R_kernel(float* R_api, const float* R, const float* G, int normalised, Dims d, int off,
                                int kb) {
  const int64_t total = (int64_t)d.q * d.m * kb * kb;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int b = (int)(idx % kb);
    const int a = (int)((idx / kb) % kb);
    const int64_t rt = idx / ((int64_t)kb * kb);    // member * m + slice
    const int r = (int)(rt / d.m);
    R_api[idx] = R[(rt * d.k + off + a) * d.k + off + b] * col_norm(G, r, off + a, d.k, normalised) *
                 col_norm(G, r, off + b, d.k, normalised);
  }
}

hipError_t launch_export_factors(float* A_api, float* R_api, const float* A_int, const float* R, const float* G,
                                 int normalised, const Dims& d, hipStream_t s, int col_off, int kb) {
  if (kb < 0) kb = d.k;
  if (A_api)
    hipLaunchKernelGGL(export_A_kernel, dim3(grid_for((int64_t)d.q * d.n * kb)), dim3(256), 0, s, A_api, A_int, G,
                       normalised, d, col_off, kb);
  if (R_api)
    hipLaunchKernelGGL(export_R_kernel, dim3(grid_for((int64_t)d.q * d.m * kb * kb)), dim3(256), 0, s, R_api, R, G,
                       normalised, d, col_off, kb);
  return hipGetLastError();
}

__global__ void from_internal_single_kernel(float* out, const float* M, int ldm, int64_t n, int k) {
  const int64_t total = n * k;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x)
    out[idx] = M[(idx / k) * ldm + (idx % k)];
}

hipError_t launch_from_internal_single(float* A_api_nk, const float* M, int ldm, int64_t n, int k, hipStream_t s) {
  hipLaunchKernelGGL(from_internal_single_kernel, dim3(grid_for(n * k)), dim3(256), 0, s, A_api_nk, M, ldm, n, k);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------ Gram
// out[a][c] += sum over this block's rows of Y[i][a] * Z[i][c] (the "gram_mul" class of the paper's
// timing breakdown: A^T A of Alg. 3's first statement, A^T (X_t A), and the similarity products of
// Alg. 5 and Alg. 6).  A block owns a TW x TW output tile; its 256 threads form 256/(TW/4)^2 groups that
// take interleaved rows, each thread a 4 x 4 register tile; partial tiles are added with atomics.
template <int TW>
__global__ void __launch_bounds__(256) gram_kernel(GramArgs g, int64_t rows_per_block, int nsplit) {
  constexpr int RT = 64;                   // rows staged per step
  constexpr int TG = (TW / 4) * (TW / 4);  // threads per group
  constexpr int NG = 256 / TG;
  __shared__ float Ys[RT][TW + 4];
  __shared__ float Zs[RT][TW + 4];
  const int batch = blockIdx.z / nsplit;
  const int split = blockIdx.z % nsplit;
  const int b1 = batch / g.nb2, b2 = batch % g.nb2;
  const int a0 = blockIdx.x * TW, c0 = blockIdx.y * TW;
  const float* Yb = g.Y + b1 * g.yb1 + b2 * g.yb2;
  const float* Zb = g.Z + b1 * g.zb1 + b2 * g.zb2;
  const int tid = threadIdx.x;
  const int grp = tid / TG, tl = tid % TG;
  const int ta = (tl / (TW / 4)) * 4, tb = (tl % (TW / 4)) * 4;
  float acc[4][4] = {};
  const int64_t r_begin = split * rows_per_block;
  int64_t r_end = r_begin + rows_per_block;
  if (r_end > g.n) r_end = g.n;
  for (int64_t r0 = r_begin; r0 < r_end; r0 += RT) {
    for (int idx = tid; idx < RT * TW; idx += 256) {
      const int rr = idx / TW, cc = idx % TW;
      const int64_t row = r0 + rr;
      const bool ok = row < r_end;
      Ys[rr][cc] = (ok && a0 + cc < g.wa) ? Yb[row * g.ldy + a0 + cc] : 0.0f;
      Zs[rr][cc] = (ok && c0 + cc < g.wb) ? Zb[row * g.ldz + c0 + cc] : 0.0f;
    }
    __syncthreads();
    for (int rr = grp; rr < RT; rr += NG) {
      float y[4], z[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        y[u] = Ys[rr][ta + u];
        z[u] = Zs[rr][tb + u];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[u][v] = fmaf(y[u], z[v], acc[u][v]);
    }
    __syncthreads();
  }
  float* ob = g.out + batch * g.obatch;
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int a = a0 + ta + u, c = c0 + tb + v;
      if (a < g.wa && c < g.wb && acc[u][v] != 0.0f) unsafeAtomicAdd(&ob[(int64_t)a * g.ldo + c], acc[u][v]);
    }
}

hipError_t launch_gram(const GramArgs& g, hipStream_t s) {
  const int nbatch = g.nb1 * g.nb2;
  // zero the whole output range touched
  const size_t obytes = (size_t)((nbatch - 1) * g.obatch + (int64_t)(g.wa - 1) * g.ldo + g.wb) * sizeof(float);
  hipError_t e = launch_fill_zero(g.out, obytes, s);
  if (e != hipSuccess) return e;
  const int w = g.wa > g.wb ? g.wa : g.wb;
  const int TW = w <= 16 ? 16 : (w <= 32 ? 32 : 64);
  const int tiles = (int)(ceil_div(g.wa, TW) * ceil_div(g.wb, TW));
  // enough blocks to fill the chip, but at least 512 rows each to keep the atomic traffic small
  const int64_t want_split = ceil_div(2048, (int64_t)tiles * nbatch);
  int64_t rows_per_block = round_up(ceil_div(g.n, want_split), 64);
  if (rows_per_block < 512) rows_per_block = 512;
  const int nsplit = (int)ceil_div(g.n, rows_per_block);
  dim3 grid((unsigned)ceil_div(g.wa, TW), (unsigned)ceil_div(g.wb, TW), (unsigned)(nbatch * nsplit));
  if (TW == 16)
    hipLaunchKernelGGL(gram_kernel<16>, grid, dim3(256), 0, s, g, rows_per_block, nsplit);
  else if (TW == 32)
    hipLaunchKernelGGL(gram_kernel<32>, grid, dim3(256), 0, s, g, rows_per_block, nsplit);
  else
    hipLaunchKernelGGL(gram_kernel<64>, grid, dim3(256), 0, s, g, rows_per_block, nsplit);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------ R rule
// C[a][b] = sum_c L(a,c) * Rt(c,b) over k x k matrices held in LDS with row stride ld.
// tl / tr: read the left / right operand transposed.
__device__ __forceinline__ void kk_matmul(float* C, const float* L, const float* Rm, int k, int ld, bool tl, bool tr) {
  for (int e = threadIdx.x; e < k * k; e += blockDim.x) {
    const int a = e / k, b = e % k;
    float acc = 0.0f;
    for (int c = 0; c < k; ++c) {
      const float l = tl ? L[c * ld + a] : L[a * ld + c];
      const float r = tr ? Rm[b * ld + c] : Rm[c * ld + b];
      acc = fmaf(l, r, acc);
    }
    C[a * ld + b] = acc;
  }
}

__device__ __forceinline__ double block_sum(double v, double* red) {
  // red: 256/64 doubles of LDS
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  double tot = 0.0;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) tot += red[w];
  return tot;
}

// One block per (slice, member).  Eq. 2, first rule (Alg. 3: RATA, DenoR, R[t] update):
//   R_t <- R_t (*) S_t (/) (G R_t G + eps),  S_t = A^T X_t A, G = A^T A.
// Then, with the NEW R_t (Alg. 3: ATAR, ATART and the two n x k x k products, re-associated so that the
// n-sized product is done once per iteration): W += R_t G R_t^T + R_t^T G R_t.
// Optionally the objective terms <S_t, R_t> and <G R_t G, R_t> of the OLD R_t (expansion of Eq. 1).
__global__ void __launch_bounds__(256) r_update_kernel(const float* __restrict__ G, const float* __restrict__ S,
                                                       float* __restrict__ R, float* __restrict__ W,
                                                       double* __restrict__ obj, float* __restrict__ Rp,
                                                       float* __restrict__ Rq, int t0, Dims d, float eps,
                                                       int update, float* __restrict__ Wpart,
                                                       double* __restrict__ objpart) {
  extern __shared__ float lds[];
  __shared__ double red[4];
  const int k = d.k, ld = k + 1, kk = k * ld;
  float* Gs = lds;
  float* Rs = lds + kk;
  float* T1 = lds + 2 * kk;
  float* T2 = lds + 3 * kk;
  const int t = t0 + blockIdx.x, r = blockIdx.y;
  const float* Gq = G + (int64_t)r * k * k;
  const float* St = S + ((int64_t)t * d.q + r) * k * k;
  float* Rt = R + ((int64_t)r * d.m + t) * k * k;
  const int ks = d.ksplit;                       // two models side by side: only the diagonal blocks of G count
  for (int e = threadIdx.x; e < k * k; e += blockDim.x) {
    const int a = e / k, b = e % k;
    const bool inside = ks == 0 || (a < ks) == (b < ks);
    Gs[a * ld + b] = inside ? Gq[e] : 0.0f;
    Rs[a * ld + b] = Rt[e];
  }
  __syncthreads();
  kk_matmul(T1, Rs, Gs, k, ld, false, false);  // R_t G
  __syncthreads();
  kk_matmul(T2, Gs, T1, k, ld, false, false);  // G R_t G
  __syncthreads();
  if (obj) {
    double s1 = 0.0, s2 = 0.0;
    for (int e = threadIdx.x; e < k * k; e += blockDim.x) {
      const int a = e / k, b = e % k;
      const double rv = Rs[a * ld + b];
      s1 += (double)St[e] * rv;
      s2 += (double)T2[a * ld + b] * rv;
    }
    s1 = block_sum(s1, red);
    s2 = block_sum(s2, red);
    if (threadIdx.x == 0) {
      if (objpart) {                               // reproducible mode: this slice's share, summed over the slices later
        objpart[((int64_t)t * d.q + r) * 2 + 0] = s1;
        objpart[((int64_t)t * d.q + r) * 2 + 1] = s2;
      } else {
        atomicAdd(&obj[2 * r + 0], s1);
        atomicAdd(&obj[2 * r + 1], s2);
      }
    }
  }
  if (!update) return;
  __syncthreads();
  for (int e = threadIdx.x; e < k * k; e += blockDim.x) {
    const int a = e / k, b = e % k;
    const bool inside = ks == 0 || (a < ks) == (b < ks);
    const float v = inside ? Rs[a * ld + b] * St[e] / (T2[a * ld + b] + eps) : 0.0f;
    Rs[a * ld + b] = v;
    Rt[e] = v;
  }
  if (!W && !Rp) return;
  __syncthreads();
  if (Rp) {  // the new R_t in MFMA operand order, for the A rule on matrix cores
    const int nt = d.kp / 16;
    const int64_t base = ((int64_t)r * d.m + t) * nt * nt * 256;
    for (int e = threadIdx.x; e < nt * nt * 256; e += blockDim.x) {
      const int rr = e & 3, ln = (e >> 2) & 63, cb = (e >> 8) % nt, bb = (e >> 8) / nt;
      const int b = bb * 16 + 4 * (ln >> 4) + rr, c = cb * 16 + (ln & 15);
      const bool ok = b < k && c < k;
      Rp[base + e] = ok ? Rs[c * ld + b] : 0.0f;
      Rq[base + e] = ok ? Rs[b * ld + c] : 0.0f;
    }
  }
  if (!W) return;
  kk_matmul(T1, Gs, Rs, k, ld, false, true);   // V  = G R^T
  kk_matmul(T2, Gs, Rs, k, ld, false, false);  // V2 = G R
  __syncthreads();
  float* Wq = W + (int64_t)r * k * k;
  for (int e = threadIdx.x; e < k * k; e += blockDim.x) {
    const int a = e / k, b = e % k;
    float acc = 0.0f;
    for (int c = 0; c < k; ++c) {
      acc = fmaf(Rs[a * ld + c], T1[c * ld + b], acc);  // (R G R^T)[a][b]
      acc = fmaf(Rs[c * ld + a], T2[c * ld + b], acc);  // (R^T G R)[a][b]
    }
    if (Wpart) Wpart[((int64_t)t * d.q + r) * k * k + e] = acc;   // reproducible mode, as above
    else unsafeAtomicAdd(&Wq[e], acc);
  }
}

hipError_t launch_r_update(const float* G, const float* S, float* R, float* W, double* obj, float* Rp, float* Rq,
                           int t0, int tc, const Dims& d, float eps, int update, hipStream_t s, float* Wpart,
                           double* objpart) {
  const size_t lds = (size_t)4 * d.k * (d.k + 1) * sizeof(float);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)r_update_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       4 * 64 * 65 * (int)sizeof(float));
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(r_update_kernel, dim3(tc, d.q), dim3(256), lds, s, G, S, R, W, obj, Rp, Rq, t0, d, eps, update,
                     W ? Wpart : nullptr, obj ? objpart : nullptr);
  hipError_t e = hipGetLastError();
  // the slices' shares in the order of the slices (the caller has cleared W and obj)
  if (e == hipSuccess && W && Wpart && update)
    e = launch_reduce_parts(W, Wpart + (int64_t)t0 * d.q * d.k * d.k, (int64_t)d.q * d.k * d.k, tc, (int64_t)d.q * d.k * d.k, 1, s);
  if (e == hipSuccess && obj && objpart)
    e = launch_reduce_parts_f64(obj, objpart + (int64_t)t0 * d.q * 2, (int64_t)d.q * 2, tc, (int64_t)d.q * 2, 1, s);
  return e;
}

// ------------------------------------------------------------------------------------------ median
// Alg. 5 (medians statement) / Alg. 1 (median statement): element-wise median over the members of the
// column-aligned ensemble; for an even member count the mean of the two middle values.
__global__ void median_kernel(float* M, int ldm, const float* E_int, const int32_t* perm, Dims d) {
  const int64_t total = d.n * d.k;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int sidx = (int)(idx % d.k);
    const int64_t i = idx / d.k;
    float v[NNRESCAL_MAX_Q_INTERNAL];
    for (int r = 0; r < d.q; ++r) {
      const float x = E_int[(i * d.q + r) * d.kp + perm[r * d.k + sidx]];
      int p = r;
      while (p > 0 && v[p - 1] > x) {
        v[p] = v[p - 1];
        --p;
      }
      v[p] = x;
    }
    const float med = (d.q & 1) ? v[d.q / 2] : 0.5f * (v[d.q / 2 - 1] + v[d.q / 2]);
    M[i * ldm + sidx] = med;
  }
}

hipError_t launch_median(float* M, int ldm, const float* E_int, const int32_t* perm_dev, const Dims& d,
                         hipStream_t s) {
  hipLaunchKernelGGL(median_kernel, dim3(grid_for(d.n * d.k, 128)), dim3(128), 0, s, M, ldm, E_int, perm_dev, d);
  return hipGetLastError();
}

__global__ void copy_member_kernel(float* M, int ldm, const float* E_int, int member, Dims d) {
  const int64_t total = d.n * d.k;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int c = (int)(idx % d.k);
    const int64_t i = idx / d.k;
    M[i * ldm + c] = E_int[(i * d.q + member) * d.kp + c];
  }
}

hipError_t launch_copy_member(float* M, int ldm, const float* E_int, int member, const Dims& d, hipStream_t s) {
  hipLaunchKernelGGL(copy_member_kernel, dim3(grid_for(d.n * d.k)), dim3(256), 0, s, M, ldm, E_int, member, d);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------ regression
// Model-selection step 3 ("regression of X_t on the median A, slice by slice", done as R-only updates of
// Eq. 2): with A fixed, S_t = A^T X_t A and G = A^T A are constants and every iteration is k x k work.
// One block per slice, the whole loop inside the kernel.
__global__ void __launch_bounds__(256) regress_kernel(float* __restrict__ R, const float* __restrict__ G,
                                                      const float* __restrict__ S, int k, int iters, float eps) {
  extern __shared__ float lds[];
  const int ld = k + 1, kk = k * ld;
  float* Gs = lds;
  float* Rs = lds + kk;
  float* T1 = lds + 2 * kk;
  float* T2 = lds + 3 * kk;
  const int t = blockIdx.x;
  float* Rt = R + (int64_t)t * k * k;
  const float* St = S + (int64_t)t * k * k;
  for (int e = threadIdx.x; e < k * k; e += blockDim.x) {
    Gs[(e / k) * ld + (e % k)] = G[e];
    Rs[(e / k) * ld + (e % k)] = Rt[e];
  }
  __syncthreads();
  for (int it = 0; it < iters; ++it) {
    kk_matmul(T1, Rs, Gs, k, ld, false, false);
    __syncthreads();
    kk_matmul(T2, Gs, T1, k, ld, false, false);
    __syncthreads();
    for (int e = threadIdx.x; e < k * k; e += blockDim.x) {
      const int a = e / k, b = e % k;
      Rs[a * ld + b] = Rs[a * ld + b] * St[e] / (T2[a * ld + b] + eps);
    }
    __syncthreads();
  }
  for (int e = threadIdx.x; e < k * k; e += blockDim.x) Rt[e] = Rs[(e / k) * ld + (e % k)];
}

hipError_t launch_regress(float* R, const float* G, const float* S, int m, int k, int iters, float eps,
                          hipStream_t s) {
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)regress_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       4 * 64 * 65 * (int)sizeof(float));
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const size_t lds = (size_t)4 * k * (k + 1) * sizeof(float);
  hipLaunchKernelGGL(regress_kernel, dim3(m), dim3(256), lds, s, R, G, S, k, iters, eps);
  return hipGetLastError();
}

}  // namespace nnr
