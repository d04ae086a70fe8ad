// The SVD-based start of the multiplicative updates (arxiv 2202.09512, section "Experiments", algorithmic
// parameters, option 2): NNDSVD (Boutsidis and Gallopoulos 2008) of M = [X_1 .. X_m  X_1^T .. X_m^T], of which
// the left factor becomes A; R_t then takes R-only updates of Eq. 2 from the random R of Alg. 3 step 1.
//
// The k leading left singular vectors of M are the k leading eigenvectors of
//   B = M M^T = sum_t X_t X_t^T + X_t^T X_t,
// found by subspace iteration with a Rayleigh-Ritz step per round, for all q members at once (member r works on
// its own perturbed tensor X^r, generated on the fly by the same passes over X that the updates use):
//   P_t = X_t U, Q_t = X_t^T U                       one pass over X (the kernels of the iteration)
//   T   = U^T B U = sum_t P_t^T P_t + Q_t^T Q_t      k x k, eigen-decomposed on the host: T = V L V^T
//   Y   = B U = sum_t X_t Q_t + X_t^T P_t            a second pass, with P_t and Q_t as the right operands
//   U  <- orth(Y V L^-1)                             Cholesky QR of a well-conditioned matrix (columns ~ unit)
// The right singular vectors are never formed: v_j = M^T u_j / s_j is the stack of the columns j of Q_t and P_t
// over s_j, and NNDSVD needs only the norms of its positive and negative parts.
#include <cmath>
#include <vector>

#include "api_internal.h"

namespace nnr {

static int grid_for(int64_t total, int block = 256, int cap = 16384) {
  int64_t b = (total + block - 1) / block;
  if (b < 1) b = 1;
  if (b > cap) b = cap;
  return (int)b;
}

// ------------------------------------------------------------------------------------------ kernels
// dst[i][r][c] = sum_b src[i][r][b] * Mat[r][b][c] for c < k (zero for k <= c < kp), rows i < rows; in place allowed.
// One wave per (row, member) at a time: lane c holds column c of the row, the others arrive by lane broadcast.
__global__ void __launch_bounds__(256) right_mul_kernel(float* dst, const float* src, const float* __restrict__ Mat,
                                                        int64_t rows, int q, int k, int kp) {
  __shared__ float ms[NNRESCAL_MAX_K_INTERNAL * NNRESCAL_MAX_K_INTERNAL];
  const int r = blockIdx.y;
  for (int e = threadIdx.x; e < k * k; e += blockDim.x) ms[e] = Mat[(int64_t)r * k * k + e];
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * 4;
  for (int64_t i = wave; i < rows; i += nwaves) {
    const int64_t base = (i * q + r) * kp;
    const float y = lane < k ? src[base + lane] : 0.0f;
    float acc = 0.0f;
    for (int b = 0; b < k; ++b) {
      const float yb = __shfl(y, b);
      if (lane < k) acc = fmaf(yb, ms[b * k + lane], acc);
    }
    if (lane < kp) dst[base + lane] = lane < k ? acc : 0.0f;
  }
}

static hipError_t launch_right_mul(float* dst, const float* src, const float* Mat, int64_t rows, const Dims& d,
                                   hipStream_t s) {
  int64_t bx = ceil_div(rows, 4 * 16);
  if (bx > 4096) bx = 4096;
  if (bx < 1) bx = 1;
  hipLaunchKernelGGL(right_mul_kernel, dim3((unsigned)bx, (unsigned)d.q), dim3(256), 0, s, dst, src, Mat, rows, d.q, d.k,
                     d.kp);
  return hipGetLastError();
}

__global__ void add_kernel(float* __restrict__ y, const float* __restrict__ t, int64_t total) {
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x)
    y[idx] += t[idx];
}

// out[r][c][0..3] += sum_i max(x,0)^2, sum_i max(-x,0)^2, sum_i max(x,0), sum_i max(-x,0) over x = src[i][r][c]
__global__ void __launch_bounds__(256) posneg_kernel(const float* __restrict__ src, double* out, int64_t rows, int q, int k,
                                                     int kp) {
  const int r = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * 4;
  double sp = 0.0, sn = 0.0, lp = 0.0, ln = 0.0;
  if (lane < k) {
    for (int64_t i = wave; i < rows; i += nwaves) {
      const float x = src[(i * q + r) * kp + lane];
      const double p = x > 0.0f ? (double)x : 0.0, n = x < 0.0f ? -(double)x : 0.0;
      sp += p * p;
      sn += n * n;
      lp += p;
      ln += n;
    }
    double* o = out + ((int64_t)r * k + lane) * 4;
    atomicAdd(o + 0, sp);
    atomicAdd(o + 1, sn);
    atomicAdd(o + 2, lp);
    atomicAdd(o + 3, ln);
  }
}

static hipError_t launch_posneg(const float* src, double* out, int64_t rows, const Dims& d, hipStream_t s) {
  int64_t bx = ceil_div(rows, 4 * 64);
  if (bx > 1024) bx = 1024;
  if (bx < 1) bx = 1;
  hipLaunchKernelGGL(posneg_kernel, dim3((unsigned)bx, (unsigned)d.q), dim3(256), 0, s, src, out, rows, d.q, d.k, d.kp);
  return hipGetLastError();
}

// A[i][r][c] <- max(floor[r], coef[r][c] * part(A[i][r][c])) for i < n, c < k; part: mode 0 |x|, 1 max(x,0), 2 max(-x,0)
__global__ void assemble_kernel(float* A, const float* __restrict__ coef, const int* __restrict__ mode,
                                const float* __restrict__ floor_r, Dims d) {
  const int64_t total = d.n * d.q * d.kp;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int c = (int)(idx % d.kp);
    const int r = (int)((idx / d.kp) % d.q);
    if (c >= d.k) continue;
    const float x = A[idx];
    const int md = mode[r * d.k + c];
    const float part = md == 0 ? fabsf(x) : (md == 1 ? fmaxf(x, 0.0f) : fmaxf(-x, 0.0f));
    A[idx] = fmaxf(floor_r[r], coef[r * d.k + c] * part);
  }
}

// ------------------------------------------------------------------------------------------ host linear algebra
// Cyclic Jacobi for a symmetric k x k matrix (fp64): T = V diag(lam) V^T, eigenvalues in decreasing order.
static void jacobi_eig(std::vector<double>& T, int k, std::vector<double>& V, std::vector<double>& lam) {
  V.assign((size_t)k * k, 0.0);
  for (int i = 0; i < k; ++i) V[i * k + i] = 1.0;
  for (int sweep = 0; sweep < 60; ++sweep) {
    double off = 0.0, diag = 0.0;
    for (int i = 0; i < k; ++i)
      for (int j = 0; j < k; ++j) (i == j ? diag : off) += T[i * k + j] * T[i * k + j];
    if (off <= 1e-30 * diag || off == 0.0) break;
    for (int p = 0; p < k - 1; ++p)
      for (int qq = p + 1; qq < k; ++qq) {
        const double apq = T[p * k + qq];
        if (apq == 0.0) continue;
        const double theta = (T[qq * k + qq] - T[p * k + p]) / (2.0 * apq);
        const double t = (theta >= 0 ? 1.0 : -1.0) / (std::fabs(theta) + std::sqrt(theta * theta + 1.0));
        const double c = 1.0 / std::sqrt(t * t + 1.0), s = t * c;
        for (int i = 0; i < k; ++i) {                 // columns p, q of T
          const double a = T[i * k + p], b = T[i * k + qq];
          T[i * k + p] = c * a - s * b;
          T[i * k + qq] = s * a + c * b;
        }
        for (int i = 0; i < k; ++i) {                 // rows p, q of T
          const double a = T[p * k + i], b = T[qq * k + i];
          T[p * k + i] = c * a - s * b;
          T[qq * k + i] = s * a + c * b;
        }
        for (int i = 0; i < k; ++i) {
          const double a = V[i * k + p], b = V[i * k + qq];
          V[i * k + p] = c * a - s * b;
          V[i * k + qq] = s * a + c * b;
        }
      }
  }
  std::vector<int> order(k);
  for (int i = 0; i < k; ++i) order[i] = i;
  for (int i = 0; i < k; ++i)                          // selection sort by decreasing eigenvalue
    for (int j = i + 1; j < k; ++j)
      if (T[order[j] * k + order[j]] > T[order[i] * k + order[i]]) std::swap(order[i], order[j]);
  std::vector<double> Vs((size_t)k * k);
  lam.resize(k);
  for (int c = 0; c < k; ++c) {
    lam[c] = T[order[c] * k + order[c]];
    for (int i = 0; i < k; ++i) Vs[i * k + c] = V[i * k + order[c]];
  }
  V.swap(Vs);
}

// Minv = L^-T for G = L L^T (fp64, lower Cholesky); a non-positive pivot (a direction that B annihilates) is
// replaced by a tiny one, which leaves that column finite and meaningless.
static void chol_inv_t(const std::vector<double>& G, int k, std::vector<double>& Minv) {
  std::vector<double> L((size_t)k * k, 0.0);
  double dmax = 0.0;
  for (int i = 0; i < k; ++i) dmax = std::fmax(dmax, G[i * k + i]);
  for (int j = 0; j < k; ++j) {
    double s = G[j * k + j];
    for (int p = 0; p < j; ++p) s -= L[j * k + p] * L[j * k + p];
    if (!(s > 1e-14 * dmax)) s = 1e-14 * dmax + 1e-300;
    L[j * k + j] = std::sqrt(s);
    for (int i = j + 1; i < k; ++i) {
      double v = G[i * k + j];
      for (int p = 0; p < j; ++p) v -= L[i * k + p] * L[j * k + p];
      L[i * k + j] = v / L[j * k + j];
    }
  }
  // Linv by forward substitution, then transpose
  std::vector<double> Li((size_t)k * k, 0.0);
  for (int c = 0; c < k; ++c) {
    Li[c * k + c] = 1.0 / L[c * k + c];
    for (int i = c + 1; i < k; ++i) {
      double v = 0.0;
      for (int p = c; p < i; ++p) v -= L[i * k + p] * Li[p * k + c];
      Li[i * k + c] = v / L[i * k + i];
    }
  }
  Minv.assign((size_t)k * k, 0.0);
  for (int i = 0; i < k; ++i)
    for (int j = 0; j < k; ++j) Minv[i * k + j] = Li[j * k + i];
}

#define HIPCHK(expr)                                                                        \
  do {                                                                                      \
    hipError_t _e = (expr);                                                                 \
    if (_e != hipSuccess) {                                                                 \
      st = fail(h, NNRESCAL_EDEVICE, std::string(#expr) + ": " + hipGetErrorString(_e)); \
      goto done;                                                                            \
    }                                                                                       \
  } while (0)

nnrescal_status start_nndsvd_impl(nnrescal_handle* h, int svd_iters, int r_iters, float floor_rel, float* sigma_out) {
  const Dims& d = h->d;
  const int k = d.k, q = d.q, m = d.m;
  const bool dense = h->X.format == NNRESCAL_DENSE;
  const size_t row = (size_t)q * d.kp;
  const size_t fbytes = (size_t)d.n_pad * row * sizeof(float);
  const int64_t ps = (int64_t)d.n * q * d.kp;       // one slice of P or Q
  const size_t kk = (size_t)k * k;
  // one slice's operand-order copy, with the spare member slots that a rounded-up tail group reads
  const size_t op_stride = (size_t)d.n_pad * row + 8 * (size_t)d.kp * 16;
  nnrescal_status st = NNRESCAL_OK;
  float *Y = nullptr, *T1 = nullptr, *opP = nullptr, *opQ = nullptr, *gram = nullptr, *mat = nullptr, *coef = nullptr, *floor_d = nullptr;
  int* mode_d = nullptr;
  double* sums = nullptr;
  std::vector<float> hg, hm(q * kk);
  std::vector<double> Tm, V, lam, G, Minv;
  std::vector<std::vector<double>> Vq(q), lamq(q);
  hipStream_t s = h->stream;

  auto alloc = [&](void** p, size_t bytes) {
    *p = dev_alloc(h->p, bytes);
    return *p != nullptr;
  };
  if (!alloc((void**)&Y, fbytes) || !alloc((void**)&T1, fbytes) ||
      (dense && (!alloc((void**)&opP, m * op_stride * sizeof(float)) || !alloc((void**)&opQ, m * op_stride * sizeof(float)))) ||
      !alloc((void**)&gram, (size_t)2 * m * q * kk * sizeof(float)) || !alloc((void**)&mat, q * kk * sizeof(float)) ||
      !alloc((void**)&coef, (size_t)q * k * sizeof(float)) || !alloc((void**)&floor_d, q * sizeof(float)) ||
      !alloc((void**)&mode_d, (size_t)q * k * sizeof(int)) || !alloc((void**)&sums, (size_t)2 * q * k * 4 * sizeof(double))) {
    st = fail(h, NNRESCAL_ENOMEM, "the alloc callback returned NULL");
    goto done;
  }
  {
    // ---- helpers on the handle's stream
    auto upload_mats = [&](const std::vector<float>& src) {
      return hipMemcpyAsync(mat, src.data(), q * kk * sizeof(float), hipMemcpyHostToDevice, s);
    };
    // U <- Ysrc * Minv with Minv from the Cholesky factor of Ysrc^T Ysrc (per member); Ysrc has n_pad rows
    auto chol_qr_into_A = [&](float* Ysrc) -> hipError_t {
      hipError_t e = launch_gram16(Ysrc, Ysrc, 0, gram, 1, d, s);
      if (e != hipSuccess) return e;
      hg.resize(q * kk);
      if ((e = hipMemcpyAsync(hg.data(), gram, q * kk * sizeof(float), hipMemcpyDeviceToHost, s)) != hipSuccess) return e;
      if ((e = hipStreamSynchronize(s)) != hipSuccess) return e;
      for (int r = 0; r < q; ++r) {
        G.assign(hg.begin() + r * kk, hg.begin() + (r + 1) * kk);
        chol_inv_t(G, k, Minv);
        for (size_t e2 = 0; e2 < kk; ++e2) hm[r * kk + e2] = (float)Minv[e2];
      }
      if ((e = upload_mats(hm)) != hipSuccess) return e;
      if ((e = launch_right_mul(h->A, Ysrc, mat, d.n, d, s)) != hipSuccess) return e;
      h->aop_valid = false;
      h->g_valid = false;
      return hipStreamSynchronize(s);               // hm is reused by the next upload
    };
    // P_t, Q_t for all slices from the current h->A; T = sum_t P_t^T P_t + Q_t^T Q_t; eigen-decomposition per member
    auto pass_and_ritz = [&]() -> hipError_t {
      hipError_t e;
      if (dense) {
        if ((e = dense_pass(h)) != hipSuccess) return e;
      } else {
        for (int t = 0; t < m; ++t)
          if ((e = sparse_pass(h, t, true)) != hipSuccess) return e;
      }
      for (int t = 0; t < m; ++t) {
        if ((e = launch_gram16(h->P + t * ps, h->P + t * ps, 0, gram + (size_t)(2 * t) * q * kk, 1, d, s)) != hipSuccess)
          return e;
        if ((e = launch_gram16(h->Q + t * ps, h->Q + t * ps, 0, gram + (size_t)(2 * t + 1) * q * kk, 1, d, s)) !=
            hipSuccess)
          return e;
      }
      hg.resize((size_t)2 * m * q * kk);
      if ((e = hipMemcpyAsync(hg.data(), gram, hg.size() * sizeof(float), hipMemcpyDeviceToHost, s)) != hipSuccess)
        return e;
      if ((e = hipStreamSynchronize(s)) != hipSuccess) return e;
      for (int r = 0; r < q; ++r) {
        Tm.assign(kk, 0.0);
        for (int b = 0; b < 2 * m; ++b)
          for (size_t e2 = 0; e2 < kk; ++e2) Tm[e2] += hg[((size_t)b * q + r) * kk + e2];
        for (int i = 0; i < k; ++i)                 // symmetrise the rounding
          for (int j = i + 1; j < k; ++j) Tm[i * k + j] = Tm[j * k + i] = 0.5 * (Tm[i * k + j] + Tm[j * k + i]);
        jacobi_eig(Tm, k, Vq[r], lamq[r]);
      }
      return hipSuccess;
    };

    // ---- random factors (Alg. 3 step 1): R keeps them, A is orthonormalised as the first basis
    HIPCHK(launch_fill_zero(Y, fbytes, s));
    HIPCHK(launch_fill_zero(T1, fbytes, s));
    if (dense) {
      HIPCHK(launch_fill_zero(opP, m * op_stride * sizeof(float), s));
      HIPCHK(launch_fill_zero(opQ, m * op_stride * sizeof(float), s));
    }
    HIPCHK(launch_init_factors(h->A, h->R, d, h->p.seed, s));
    HIPCHK(hipMemcpyAsync(Y, h->A, fbytes, hipMemcpyDeviceToDevice, s));
    HIPCHK(chol_qr_into_A(Y));

    for (int it = 0; it <= svd_iters; ++it) {
      HIPCHK(pass_and_ritz());
      if (it == svd_iters) break;
      // ---- Y = sum_t X_t Q_t + X_t^T P_t
      HIPCHK(launch_fill_zero(Y, fbytes, s));
      for (int t = 0; t < m; ++t) {
        if (dense) {
          // operand-order copies of Q_t (right operand of X_t .) and P_t (of X_t^T .); the products follow below
          HIPCHK(launch_pack_operand(h->Q + t * ps, opQ + (size_t)t * op_stride, d, s, d.n));
          HIPCHK(launch_pack_operand(h->P + t * ps, opP + (size_t)t * op_stride, d, s, d.n));
        } else {
          const int64_t lo = h->csr_off[t], nnz = h->csr_off[t + 1] - lo;
          const int64_t total = d.n * (int64_t)row;
          HIPCHK(launch_spmm_gather(h->X.csr_rowptr + (int64_t)t * (d.n + 1), h->csr_major + lo, h->X.csr_col + lo,
                                    (h->X.csr_val ? h->X.csr_val + lo : nullptr), nnz, h->Q + t * ps, T1, d, t, 0, 1, h->p.seed, h->p.delta, s));
          hipLaunchKernelGGL(add_kernel, dim3(grid_for(total)), dim3(256), 0, s, Y, T1, total);
          if (h->X.format == NNRESCAL_CSR_CSC) {
            const int64_t lo2 = h->csc_off[t];
            HIPCHK(launch_spmm_gather(h->X.csc_colptr + (int64_t)t * (d.n + 1), h->csc_major + lo2, h->X.csc_row + lo2,
                                      (h->X.csc_val ? h->X.csc_val + lo2 : nullptr), nnz, h->P + t * ps, T1, d, t, 1, 1, h->p.seed, h->p.delta, s));
            hipLaunchKernelGGL(add_kernel, dim3(grid_for(total)), dim3(256), 0, s, Y, T1, total);
          } else {                                 // (the scatter form clears its output first)
            HIPCHK(launch_spmm_scatter(h->csr_major + lo, h->X.csr_col + lo, (h->X.csr_val ? h->X.csr_val + lo : nullptr), nnz, h->P + t * ps, T1, d,
                                       t, h->p.seed, h->p.delta, s));
            hipLaunchKernelGGL(add_kernel, dim3(grid_for(total)), dim3(256), 0, s, Y, T1, total);
          }
          HIPCHK(hipGetLastError());
        }
      }
      if (dense) {
        // one launch over all slices: X_t Q_t and X_t^T P_t, both summed over t into Y (slice stride 0 of the outputs)
        DenseStreamOpts so;
        so.A_opQ = opP;
        so.aop_tstride = (int64_t)op_stride;
        so.out_tstride = 0;
        so.timeout_flag = h->dev_error;
        so.spin_limit = h->p.handover_spin_limit;
        HIPCHK(launch_dense_stream(h->X.dense, opQ, Y, Y, d, 0, h->p.seed, h->p.delta, s, so));
        HIPCHK(launch_dense_stream(h->X.dense, opQ, Y, Y, d, 1, h->p.seed, h->p.delta, s, so));
      }
      // ---- Y <- Y V L^-1 (columns of about unit length), then Cholesky QR into A
      for (int r = 0; r < q; ++r)
        for (int i = 0; i < k; ++i)
          for (int j = 0; j < k; ++j) {
            const double l = lamq[r][j] > 1e-30 * lamq[r][0] ? lamq[r][j] : (lamq[r][0] > 0 ? 1e-30 * lamq[r][0] : 1.0);
            hm[r * kk + i * k + j] = (float)(Vq[r][i * k + j] / l);
          }
      HIPCHK(upload_mats(hm));
      HIPCHK(launch_right_mul(Y, Y, mat, d.n, d, s));
      HIPCHK(hipStreamSynchronize(s));
      HIPCHK(chol_qr_into_A(Y));
    }

    // ---- Ritz vectors: U <- U V, and with them P_t <- P_t V, Q_t <- Q_t V (the products are linear in U)
    for (int r = 0; r < q; ++r)
      for (size_t e2 = 0; e2 < kk; ++e2) hm[r * kk + e2] = (float)Vq[r][e2];
    HIPCHK(upload_mats(hm));
    HIPCHK(launch_right_mul(h->A, h->A, mat, d.n, d, s));
    HIPCHK(launch_fill_zero(sums, (size_t)2 * q * k * 4 * sizeof(double), s));
    HIPCHK(launch_posneg(h->A, sums, d.n, d, s));
    for (int t = 0; t < m; ++t) {
      HIPCHK(launch_right_mul(T1, h->P + t * ps, mat, d.n, d, s));
      HIPCHK(launch_posneg(T1, sums + (size_t)q * k * 4, d.n, d, s));
      HIPCHK(launch_right_mul(T1, h->Q + t * ps, mat, d.n, d, s));
      HIPCHK(launch_posneg(T1, sums + (size_t)q * k * 4, d.n, d, s));
    }
    std::vector<double> hs((size_t)2 * q * k * 4);
    HIPCHK(hipMemcpyAsync(hs.data(), sums, hs.size() * sizeof(double), hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));

    // ---- NNDSVD, left factor: which part of each vector is kept, and its scale; the floor from the mean
    std::vector<float> hcoef((size_t)q * k), hfloor(q);
    std::vector<int> hmode((size_t)q * k);
    for (int r = 0; r < q; ++r) {
      double total = 0.0;
      for (int j = 0; j < k; ++j) {
        const double* u = &hs[((size_t)r * k + j) * 4];
        const double* v = &hs[((size_t)(q + r) * k + j) * 4];
        const double sig = std::sqrt(std::fmax(lamq[r][j], 0.0));
        if (sigma_out) sigma_out[r * k + j] = (float)sig;
        double cf = 0.0, l1 = 0.0;
        int md = 1;
        if (j == 0) {
          md = 0;
          cf = std::sqrt(sig);
          l1 = u[2] + u[3];
        } else if (sig > 0.0) {
          const double nxp = std::sqrt(u[0]), nxn = std::sqrt(u[1]);
          const double nyp = std::sqrt(v[0]) / sig, nyn = std::sqrt(v[1]) / sig;   // v_j = M^T u_j / s_j
          const double mp = nxp * nyp, mn = nxn * nyn;
          if (mp > mn) {
            md = 1;
            cf = std::sqrt(sig * mp) / nxp;
            l1 = u[2];
          } else if (mn > 0.0) {
            md = 2;
            cf = std::sqrt(sig * mn) / nxn;
            l1 = u[3];
          }
        }
        hcoef[r * k + j] = (float)cf;
        hmode[r * k + j] = md;
        total += cf * l1;
      }
      hfloor[r] = (float)(floor_rel * total / ((double)d.n * k));
    }
    HIPCHK(hipMemcpyAsync(coef, hcoef.data(), hcoef.size() * sizeof(float), hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(mode_d, hmode.data(), hmode.size() * sizeof(int), hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(floor_d, hfloor.data(), hfloor.size() * sizeof(float), hipMemcpyHostToDevice, s));
    hipLaunchKernelGGL(assemble_kernel, dim3(grid_for(d.n * (int64_t)row)), dim3(256), 0, s, h->A, coef, mode_d, floor_d, d);
    HIPCHK(hipGetLastError());
    HIPCHK(hipStreamSynchronize(s));                // the host vectors go out of scope
    h->aop_valid = false;
    h->g_valid = false;

    // ---- R: r_iters R-only updates of Eq. 2 with this A (A^T A and A^T X_t A are then constants)
    if (r_iters > 0) {
      HIPCHK(compute_G(h));
      if (dense) {
        HIPCHK(dense_pass(h));
      } else {
        for (int t = 0; t < m; ++t) HIPCHK(sparse_pass(h, t, false));
      }
      HIPCHK(launch_gram16(h->A, h->P, ps, h->S, m, d, s));
      for (int it = 0; it < r_iters; ++it)
        HIPCHK(launch_r_update(h->G, h->S, h->R, nullptr, nullptr, nullptr, nullptr, 0, m, d, h->p.eps_div, 1, s));
    }
    h->iterations = 0;
  }
done:
  if (st != NNRESCAL_OK) (void)hipStreamSynchronize(s);
  void* bufs[] = {Y, T1, opP, opQ, gram, mat, coef, floor_d, mode_d, sums};
  if (st == NNRESCAL_OK && hipStreamSynchronize(s) != hipSuccess) st = fail(h, NNRESCAL_EDEVICE, "synchronising the stream");
  if (st == NNRESCAL_OK) st = device_error_status(h);
  for (void* b : bufs)
    if (b) h->p.dealloc(b, h->p.alloc_ctx);
  return st;
}

}  // namespace nnr
