// Tensors that fit one compute unit's LDS (arxiv 2202.09512, Alg. 3 / Eq. 2 for the small end of the paper's
// synthetic sweep): one workgroup per ensemble member keeps its perturbed tensor X^r (Alg. 4, built once per
// launch), A^r and R^r in LDS and runs ALL the requested iterations in one launch.  At these sizes an iteration
// of the general path is ten kernel launches of a few microseconds each: launch latency, not arithmetic.
//
// Same statements as the general path (the n-sized products re-associated the same way), each batched over the
// slices (the R updates of different slices are independent once G is known), so that an iteration costs seven
// barriers:
//   G = A^T A;  P_t = X_t A, Q_t = X_t^T A;  S_t = A^T P_t;  R_t <- R_t (*) S_t (/) (G R_t G + eps);
//   Num = sum_t P_t R_t^T + Q_t R_t;  W = sum_t R_t G R_t^T + R_t^T G R_t;  A <- A (*) Num (/) (A W + eps).
#include "common.h"
#include "kernels.h"

namespace nnr {

constexpr int kTinyThreads = 256;
constexpr int kTinyMaxN = 64;                        // the A rule stages its new elements in registers

// out[a*cols + b] = sum_{c < len} term(a, b, c).  Four independent partial sums per element keep several LDS
// reads in flight (these loops are bound by LDS latency, not by arithmetic).
template <typename F>
__device__ __forceinline__ void sum_terms(float* out, int rows, int cols, int len, F term) {
  for (int e = threadIdx.x; e < rows * cols; e += kTinyThreads) {
    const int a = e / cols, b = e % cols;
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    int c = 0;
    for (; c + 4 <= len; c += 4) {
      s0 += term(a, b, c);
      s1 += term(a, b, c + 1);
      s2 += term(a, b, c + 2);
      s3 += term(a, b, c + 3);
    }
    for (; c < len; ++c) s0 += term(a, b, c);
    out[e] = (s0 + s1) + (s2 + s3);
  }
}

__global__ void __launch_bounds__(kTinyThreads)
    tiny_fit_kernel(const float* __restrict__ X, float* __restrict__ A_int, float* __restrict__ R, Dims d, int iters,
                    float eps, uint32_t k0, uint32_t k1, float dscaled, int perturb) {
  extern __shared__ float lds[];
  const int n = (int)d.n, m = d.m, k = d.k, q = d.q, kp = d.kp, kk = k * k;
  const int r = blockIdx.x;                          // ensemble member
  const int ldx = n + 1;                             // row pitch of a slice: column walks stay conflict-free
  float* Xs = lds;                                   // [m][n][ldx]
  float* As = Xs + (size_t)m * n * ldx;              // [n][k]
  float* Pa = As + n * k;                            // [m][n][k]: X_t A
  float* Qa = Pa + (size_t)m * n * k;                // [m][n][k]: X_t^T A
  float* Num = Qa + (size_t)m * n * k;               // [n][k]
  float* Rs = Num + n * k;                           // [m][k][k]
  float* Sa = Rs + m * kk;                           // [m][k][k]: A^T X_t A
  float* T1 = Sa + m * kk;                           // [m][k][k]
  float* T2 = T1 + m * kk;                           // [m][k][k]
  float* Gs = T2 + m * kk;                           // [k][k]
  float* Ws = Gs + kk;                               // [k][k]

  // ---- the member's perturbed tensor (one Philox block per element; this member's 16-bit half of it)
  for (int e = threadIdx.x; e < m * n * n; e += kTinyThreads) {
    const int t = e / (n * n), i = (e / n) % n, j = e % n;
    float v = X[e];
    if (perturb) {
      const uint64_t c = (uint64_t)i * (uint64_t)n + (uint64_t)j;
      const u32x4 w = philox4x32_10((uint32_t)c, (uint32_t)(c >> 32), (uint32_t)t, (uint32_t)(r >> 3), k0, k1);
      v = perturbed(v, w, r & 7, dscaled);
    }
    Xs[((size_t)t * n + i) * ldx + j] = v;
  }
  for (int e = threadIdx.x; e < n * k; e += kTinyThreads) As[e] = A_int[((int64_t)(e / k) * q + r) * kp + e % k];
  for (int e = threadIdx.x; e < m * kk; e += kTinyThreads) Rs[e] = R[(int64_t)r * m * kk + e];
  __syncthreads();

  for (int it = 0; it < iters; ++it) {
    // G[a][b] = sum_i A[i][a] A[i][b];  P[(t,i)][c] = sum_j X_t[i][j] A[j][c];  Q[(t,j)][c] = sum_i X_t[i][j] A[i][c]
    sum_terms(Gs, k, k, n, [&](int a, int b, int i) { return As[i * k + a] * As[i * k + b]; });
    sum_terms(Pa, m * n, k, n, [&](int ti, int c, int j) { return Xs[(size_t)ti * ldx + j] * As[j * k + c]; });
    sum_terms(Qa, m * n, k, n,
              [&](int tj, int c, int i) { return Xs[((size_t)(tj / n) * n + i) * ldx + tj % n] * As[i * k + c]; });
    __syncthreads();
    // S[(t,a)][b] = sum_i A[i][a] P_t[i][b];  T1[(t,a)][b] = sum_c R_t[a][c] G[c][b]
    sum_terms(Sa, m * k, k, n, [&](int ta, int b, int i) { return As[i * k + ta % k] * Pa[((ta / k) * n + i) * k + b]; });
    sum_terms(T1, m * k, k, k, [&](int ta, int b, int c) { return Rs[ta * k + c] * Gs[c * k + b]; });
    __syncthreads();
    // T2[(t,a)][b] = sum_c G[a][c] T1_t[c][b] = (G R_t G)[a][b]
    sum_terms(T2, m * k, k, k, [&](int ta, int b, int c) { return Gs[(ta % k) * k + c] * T1[((ta / k) * k + c) * k + b]; });
    __syncthreads();
    for (int e = threadIdx.x; e < m * kk; e += kTinyThreads) Rs[e] = Rs[e] * Sa[e] / (T2[e] + eps);
    __syncthreads();
    // with the new R_t: T1_t = G R_t^T, T2_t = G R_t;
    // Num[i][c] = sum_{(t,b)} P_t[i][b] R_t[c][b] + Q_t[i][b] R_t[b][c]
    sum_terms(T1, m * k, k, k, [&](int ta, int b, int c) { return Gs[(ta % k) * k + c] * Rs[((ta / k) * k + b) * k + c]; });
    sum_terms(T2, m * k, k, k, [&](int ta, int b, int c) { return Gs[(ta % k) * k + c] * Rs[((ta / k) * k + c) * k + b]; });
    sum_terms(Num, n, k, m * k, [&](int i, int c, int tb) {
      const int t = tb / k, b = tb % k;
      return Pa[(t * n + i) * k + b] * Rs[(t * k + c) * k + b] + Qa[(t * n + i) * k + b] * Rs[(t * k + b) * k + c];
    });
    __syncthreads();
    // W[a][b] = sum_{(t,c)} R_t[a][c] (G R_t^T)[c][b] + R_t[c][a] (G R_t)[c][b]
    sum_terms(Ws, k, k, m * k, [&](int a, int b, int tc) {
      const int t = tc / k, c = tc % k;
      return Rs[(t * k + a) * k + c] * T1[(t * k + c) * k + b] + Rs[(t * k + c) * k + a] * T2[(t * k + c) * k + b];
    });
    __syncthreads();
    // A <- A (*) Num (/) (A W + eps): every thread forms its own elements from the old A first
    float newa[(kTinyMaxN * NNRESCAL_MAX_K_INTERNAL + kTinyThreads - 1) / kTinyThreads];
    int cnt = 0;
    for (int e = threadIdx.x; e < n * k; e += kTinyThreads, ++cnt) {
      const int i = e / k, c = e % k;
      float den = 0.0f;
      for (int b = 0; b < k; ++b) den = fmaf(As[i * k + b], Ws[b * k + c], den);
      newa[cnt] = As[e] * Num[e] / (den + eps);
    }
    __syncthreads();
    cnt = 0;
    for (int e = threadIdx.x; e < n * k; e += kTinyThreads, ++cnt) As[e] = newa[cnt];
    __syncthreads();
  }
  for (int e = threadIdx.x; e < n * k; e += kTinyThreads) A_int[((int64_t)(e / k) * q + r) * kp + e % k] = As[e];
  for (int e = threadIdx.x; e < m * kk; e += kTinyThreads) R[(int64_t)r * m * kk + e] = Rs[e];
}

static size_t tiny_fit_lds_bytes(const Dims& d) {
  const size_t n = (size_t)d.n, m = d.m, k = d.k;
  return (m * n * (n + 1) + 2 * n * k + 2 * m * n * k + 4 * m * k * k + 2 * k * k) * sizeof(float);
}

// everything within 150 KB of LDS
bool tiny_fit_applies(const Dims& d) { return d.n <= kTinyMaxN && tiny_fit_lds_bytes(d) <= 150 * 1024; }

hipError_t launch_tiny_fit(const float* X, float* A_int, float* R, const Dims& d, int iters, float eps, uint64_t seed,
                           float delta, hipStream_t s) {
  if (!tiny_fit_applies(d)) return hipErrorInvalidValue;
  const size_t lds = tiny_fit_lds_bytes(d);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)tiny_fit_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(tiny_fit_kernel, dim3((unsigned)d.q), dim3(kTinyThreads), lds, s, X, A_int, R, d, iters, eps,
                     (uint32_t)seed, (uint32_t)(seed >> 32), delta * 0x1p-16f, delta != 0.0f ? 1 : 0);
  return hipGetLastError();
}

}  // namespace nnr
