// Model selection by ensemble stability (arxiv 2202.09512: Alg. 1 "Rescalk", Alg. 5 "customCluster",
// Alg. 6 "clusterStability", section "RESCAL with Automatic Model Selection").
//
// The n-sized work (similarity products, medians, the pass over X for the regression) runs in kernels;
// the k x k and q x k decisions (assignment, silhouettes from the similarity matrix, medians of the
// small cores) run on the host in double precision from the fp32 sums the kernels return.
#include <algorithm>
#include <cmath>
#include <limits>
#include <new>
#include <string>
#include <vector>

#include "api_internal.h"

using namespace nnr;

namespace {

#define HIPCHK0(expr)                                                                             \
  do {                                                                                            \
    hipError_t _e = (expr);                                                                       \
    if (_e != hipSuccess)                                                                         \
      return fail(nullptr, NNRESCAL_EDEVICE, std::string(#expr) + ": " + hipGetErrorString(_e)); \
  } while (0)

// Assignment problem (Alg. 5, LSA statement): permutation pi maximising sum_s sim[s][pi[s]].
// Shortest augmenting paths with row/column potentials on cost = -sim, O(k^3).
std::vector<int> assign_max(const std::vector<double>& sim, int k) {
  const double INF = std::numeric_limits<double>::infinity();
  std::vector<double> u(k + 1, 0.0), v(k + 1, 0.0);
  std::vector<int> match(k + 1, 0), way(k + 1, 0);  // match[col] = row (1-based), 0 = free
  for (int i = 1; i <= k; ++i) {
    match[0] = i;
    int j0 = 0;
    std::vector<double> minv(k + 1, INF);
    std::vector<char> used(k + 1, 0);
    do {
      used[j0] = 1;
      const int i0 = match[j0];
      double delta = INF;
      int j1 = 0;
      for (int j = 1; j <= k; ++j) {
        if (used[j]) continue;
        const double cur = -sim[(size_t)(i0 - 1) * k + (j - 1)] - u[i0] - v[j];
        if (cur < minv[j]) { minv[j] = cur; way[j] = j0; }
        if (minv[j] < delta) { delta = minv[j]; j1 = j; }
      }
      for (int j = 0; j <= k; ++j) {
        if (used[j]) { u[match[j]] += delta; v[j] -= delta; }
        else minv[j] -= delta;
      }
      j0 = j1;
    } while (match[j0] != 0);
    do {
      const int j1 = way[j0];
      match[j0] = match[j1];
      j0 = j1;
    } while (j0);
  }
  std::vector<int> pi(k);
  for (int j = 1; j <= k; ++j) pi[match[j] - 1] = j - 1;
  return pi;
}

double median_of(std::vector<double>& v) {
  std::sort(v.begin(), v.end());
  const size_t q = v.size();
  return (q & 1) ? v[q / 2] : 0.5 * (v[q / 2 - 1] + v[q / 2]);
}

struct DevBuf {
  const nnrescal_params& p;
  void* ptr = nullptr;
  DevBuf(const nnrescal_params& p_, size_t bytes) : p(p_) { ptr = dev_alloc(p, bytes); }
  ~DevBuf() { if (ptr) p.dealloc(ptr, p.alloc_ctx); }
  template <class T> T* as() { return (T*)ptr; }
};

// Alg. 5 + Alg. 6 on a column-normalised or raw ensemble in API layout.
nnrescal_status cluster_impl(const float* A_ens, const float* R_ens, int64_t n, int m, int k, int q,
                             const nnrescal_params* p, int32_t* perm_out, float* A_med, float* R_med, float* s_min,
                             float* s_avg, int32_t* rounds_out) {
  hipStream_t s = (hipStream_t)p->stream;
  Dims d;
  d.n = n; d.n_pad = n; d.m = m; d.k = k; d.q = q; d.kp = (int)round_up(k, 4);
  const int qk = q * d.kp;
  DevBuf E(*p, (size_t)n * qk * sizeof(float));           // ensemble, entity-major [n][q][kp]
  DevBuf M(*p, (size_t)n * d.kp * sizeof(float));         // centroid / median [n][kp]
  DevBuf Gfull(*p, (size_t)qk * qk * sizeof(float));      // all-pairs column products
  DevBuf Gm(*p, (size_t)d.kp * qk * sizeof(float));       // centroid x ensemble products
  DevBuf Gmm(*p, (size_t)d.kp * d.kp * sizeof(float));    // centroid x centroid products
  DevBuf permd(*p, (size_t)q * k * sizeof(int32_t));
  if (!E.ptr || !M.ptr || !Gfull.ptr || !Gm.ptr || !Gmm.ptr || !permd.ptr)
    return fail(nullptr, NNRESCAL_ENOMEM, "the alloc callback returned NULL");
  HIPCHK0(launch_to_internal(E.as<float>(), A_ens, d, s));
  // all-pairs products of the q*k columns: norms on the diagonal, cosine similarities for Alg. 6
  GramArgs gf{E.as<float>(), qk, 0, 0, qk, E.as<float>(), qk, 0, 0, qk, Gfull.as<float>(), 0, qk, n, 1, 1};
  HIPCHK0(launch_gram(gf, s));
  std::vector<float> gfull((size_t)qk * qk);
  HIPCHK0(hipMemcpyAsync(gfull.data(), Gfull.ptr, gfull.size() * sizeof(float), hipMemcpyDeviceToHost, s));
  // centroid = first member (Alg. 5, first statement): identity permutation, median over that one member
  std::vector<int32_t> perm((size_t)q * k), prev;
  for (int r = 0; r < q; ++r)
    for (int c = 0; c < k; ++c) perm[(size_t)r * k + c] = c;
  HIPCHK0(hipMemcpyAsync(permd.ptr, perm.data(), perm.size() * sizeof(int32_t), hipMemcpyHostToDevice, s));
  HIPCHK0(launch_copy_member(M.as<float>(), d.kp, E.as<float>(), 0, d, s));
  HIPCHK0(hipStreamSynchronize(s));
  std::vector<double> cn((size_t)q * k);  // column norms of the ensemble
  for (int r = 0; r < q; ++r)
    for (int c = 0; c < k; ++c) {
      const double g = gfull[(size_t)(r * d.kp + c) * qk + (r * d.kp + c)];
      cn[(size_t)r * k + c] = g > 0 ? std::sqrt(g) : 1.0;
    }
  std::vector<float> gm((size_t)d.kp * qk), gmm((size_t)d.kp * d.kp);
  int rounds = 0;
  const int max_rounds = 50;
  for (rounds = 1; rounds <= max_rounds; ++rounds) {
    GramArgs g1{M.as<float>(), d.kp, 0, 0, k, E.as<float>(), qk, 0, 0, qk, Gm.as<float>(), 0, qk, n, 1, 1};
    HIPCHK0(launch_gram(g1, s));
    GramArgs g2{M.as<float>(), d.kp, 0, 0, k, M.as<float>(), d.kp, 0, 0, k, Gmm.as<float>(), 0, d.kp, n, 1, 1};
    HIPCHK0(launch_gram(g2, s));
    HIPCHK0(hipMemcpyAsync(gm.data(), Gm.ptr, (size_t)k * qk * sizeof(float), hipMemcpyDeviceToHost, s));
    HIPCHK0(hipMemcpyAsync(gmm.data(), Gmm.ptr, (size_t)k * d.kp * sizeof(float), hipMemcpyDeviceToHost, s));
    HIPCHK0(hipStreamSynchronize(s));
    std::vector<double> sim((size_t)k * k);
    for (int r = 0; r < q; ++r) {
      for (int sidx = 0; sidx < k; ++sidx) {
        const double gs = gmm[(size_t)sidx * d.kp + sidx];
        const double mn = gs > 0 ? std::sqrt(gs) : 1.0;
        for (int c = 0; c < k; ++c)
          sim[(size_t)sidx * k + c] = (double)gm[(size_t)sidx * qk + r * d.kp + c] / (mn * cn[(size_t)r * k + c]);
      }
      const std::vector<int> pi = assign_max(sim, k);
      for (int sidx = 0; sidx < k; ++sidx) perm[(size_t)r * k + sidx] = pi[sidx];
    }
    HIPCHK0(hipMemcpyAsync(permd.ptr, perm.data(), perm.size() * sizeof(int32_t), hipMemcpyHostToDevice, s));
    HIPCHK0(launch_median(M.as<float>(), d.kp, E.as<float>(), permd.as<int32_t>(), d, s));
    HIPCHK0(hipStreamSynchronize(s));  // perm (host) is reused next round
    if (!prev.empty() && prev == perm) break;
    prev = perm;
  }
  if (rounds > max_rounds) rounds = max_rounds;
  // ---- Alg. 6: silhouettes on cosine distance; point (r, s) = column perm[r][s] of member r, label s
  double smin = 0.0, savg = 0.0;
  if (q > 1 && k > 1) {
    auto dist = [&](int r1, int s1, int r2, int s2) {
      const int c1 = perm[(size_t)r1 * k + s1], c2 = perm[(size_t)r2 * k + s2];
      const double g = gfull[(size_t)(r1 * d.kp + c1) * qk + (r2 * d.kp + c2)];
      return 1.0 - g / (cn[(size_t)r1 * k + c1] * cn[(size_t)r2 * k + c2]);
    };
    std::vector<double> cl_mean(k, 0.0);
    double tot = 0.0;
    for (int r = 0; r < q; ++r)
      for (int s1 = 0; s1 < k; ++s1) {
        double a = 0.0;
        for (int r2 = 0; r2 < q; ++r2)
          if (r2 != r) a += dist(r, s1, r2, s1);
        a /= (q - 1);
        double b = std::numeric_limits<double>::infinity();
        for (int s2 = 0; s2 < k; ++s2) {
          if (s2 == s1) continue;
          double acc = 0.0;
          for (int r2 = 0; r2 < q; ++r2) acc += dist(r, s1, r2, s2);
          b = std::min(b, acc / q);
        }
        const double den = std::max(a, b);
        const double sil = den == 0.0 ? 0.0 : (b - a) / den;
        cl_mean[s1] += sil / q;
        tot += sil;
      }
    smin = *std::min_element(cl_mean.begin(), cl_mean.end());
    savg = tot / ((double)q * k);
  }
  // ---- outputs
  if (A_med) HIPCHK0(launch_from_internal_single(A_med, M.as<float>(), d.kp, n, k, s));
  if (R_med && R_ens) {
    const size_t per = (size_t)m * k * k;
    std::vector<float> rh((size_t)q * per), rm(per);
    HIPCHK0(hipMemcpyAsync(rh.data(), R_ens, rh.size() * sizeof(float), hipMemcpyDeviceToHost, s));
    HIPCHK0(hipStreamSynchronize(s));
    std::vector<double> tmp(q);
    for (int t = 0; t < m; ++t)
      for (int a = 0; a < k; ++a)
        for (int b = 0; b < k; ++b) {
          for (int r = 0; r < q; ++r) {
            const int ca = perm[(size_t)r * k + a], cb = perm[(size_t)r * k + b];
            tmp[r] = rh[(size_t)r * per + ((size_t)t * k + ca) * k + cb];
          }
          rm[((size_t)t * k + a) * k + b] = (float)median_of(tmp);
        }
    HIPCHK0(hipMemcpyAsync(R_med, rm.data(), per * sizeof(float), hipMemcpyHostToDevice, s));
    HIPCHK0(hipStreamSynchronize(s));
  }
  HIPCHK0(hipStreamSynchronize(s));
  if (perm_out) std::copy(perm.begin(), perm.end(), perm_out);
  if (s_min) *s_min = (float)smin;
  if (s_avg) *s_avg = (float)savg;
  if (rounds_out) *rounds_out = rounds;
  return NNRESCAL_OK;
}

}  // namespace

extern "C" {

nnrescal_status nnrescal_cluster(const float* A_ens, const float* R_ens, int64_t n, int32_t m, int32_t k, int32_t q,
                                 const nnrescal_params* p, int32_t* perm, float* A_med, float* R_med, float* s_min,
                                 float* s_avg, int32_t* rounds) {
  if (!A_ens || !p || !p->alloc || !p->dealloc) return fail(nullptr, NNRESCAL_EINVAL, "A_ens, params and allocator callbacks are required");
  if (n <= 0 || k < 1 || k > NNRESCAL_MAX_K || q < 1 || q > NNRESCAL_MAX_Q || m < 0)
    return fail(nullptr, NNRESCAL_EINVAL, "bad sizes");
  if (R_med && (!R_ens || m < 1)) return fail(nullptr, NNRESCAL_EINVAL, "R_med needs R_ens and m >= 1");
  return cluster_impl(A_ens, R_ens, n, m, k, q, p, perm, A_med, R_med, s_min, s_avg, rounds);
}

nnrescal_status nnrescal_select_k(const nnrescal_tensor* X, const nnrescal_params* p, int32_t k_lo, int32_t k_hi,
                                  int32_t iters, int32_t regress_iters, float* s_min, float* s_avg, float* rel_err,
                                  int32_t* k_opt, float* A_med_or_null, float* R_reg_or_null) {
  std::string why;
  nnrescal_status st = validate_tensor(X, why);
  if (st == NNRESCAL_OK) st = validate_params(X, p, false, why);
  if (st != NNRESCAL_OK) return fail(nullptr, st, why);
  if (k_lo < 1 || k_hi < k_lo || k_hi > NNRESCAL_MAX_K || k_hi > X->n || iters < 0 || regress_iters < 0)
    return fail(nullptr, NNRESCAL_EINVAL, "need 1 <= k_lo <= k_hi <= min(n, NNRESCAL_MAX_K), iters >= 0");
  if (!s_min || !s_avg || !rel_err || !k_opt) return fail(nullptr, NNRESCAL_EINVAL, "output pointers are required");
  if (p->A0) return fail(nullptr, NNRESCAL_EINVAL, "select_k draws its own starts; A0/R0 must be NULL");
  if (p->check_input) {                            // once for the whole sweep, not once per fit
    st = check_input(X, p);
    if (st != NNRESCAL_OK) return st;
  }
  hipStream_t s = (hipStream_t)p->stream;
  const int64_t n = X->n;
  const int m = X->m, q = p->q;
  const int nk = k_hi - k_lo + 1;
  std::vector<float> smin(nk), savg(nk), err(nk);
  // robust factors for every k are kept on the device until k_opt is known
  std::vector<DevBuf*> keepA(nk, nullptr), keepR(nk, nullptr);
  // CSR only: one transposed copy, built here, serves every fit of the sweep
  nnrescal_tensor Xc = *X;
  int64_t* own_colptr = nullptr;
  int32_t* own_row = nullptr;
  float* own_val = nullptr;
  if (X->format == NNRESCAL_CSR && !p->no_csc_build) {
    st = build_csc_copy(X, p, &own_colptr, &own_row, &own_val);
    if (st != NNRESCAL_OK) return st;
    Xc.format = NNRESCAL_CSR_CSC;
    Xc.csc_colptr = own_colptr;
    Xc.csc_row = own_row;
    Xc.csc_val = own_val;
    Xc.csc_slice_off = X->csr_slice_off;
    X = &Xc;
  }
  auto cleanup = [&]() {
    for (auto* b : keepA) delete b;
    for (auto* b : keepR) delete b;
    if (own_colptr) p->dealloc(own_colptr, p->alloc_ctx);
    if (own_row) p->dealloc(own_row, p->alloc_ctx);
    if (own_val) p->dealloc(own_val, p->alloc_ctx);
    own_colptr = nullptr; own_row = nullptr; own_val = nullptr;
  };
  // Alg. 5 / Alg. 6 / medians, then the regression, for the ensemble of one rank (API layout, normalised)
  auto finish_rank = [&](int ki, DevBuf& Aens, DevBuf& Rens) -> nnrescal_status {
    const int k = k_lo + ki;
    nnrescal_status st = cluster_impl(Aens.as<float>(), Rens.as<float>(), n, m, k, q, p, nullptr, keepA[ki]->as<float>(),
                                      keepR[ki]->as<float>(), &smin[ki], &savg[ki], nullptr);
    if (st != NNRESCAL_OK) return st;
    // regression (R-only updates on the unperturbed X with A fixed to the median) and relative error
    std::vector<float> rm((size_t)m * k * k);
    hipError_t e = hipMemcpyAsync(rm.data(), keepR[ki]->ptr, rm.size() * sizeof(float), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail(nullptr, NNRESCAL_EDEVICE, hipGetErrorString(e));
    for (auto& v : rm) v = v < 1e-12f ? 1e-12f : v;
    e = hipMemcpyAsync(keepR[ki]->ptr, rm.data(), rm.size() * sizeof(float), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail(nullptr, NNRESCAL_EDEVICE, hipGetErrorString(e));
    nnrescal_params p1 = *p;
    p1.k = k; p1.q = 1; p1.delta = 0.0f; p1.start = 0; p1.check_input = 0;
    p1.A0 = keepA[ki]->as<float>();
    p1.R0 = keepR[ki]->as<float>();
    nnrescal_handle* h1 = nullptr;
    st = init_impl(&h1, X, &p1);
    if (st != NNRESCAL_OK) return st;
    // G = A^T A and S_t = A^T X_t A for the fixed A (left in h1->G, h1->S by the objective pass)
    st = objective_enqueue(h1);
    if (st == NNRESCAL_OK && regress_iters > 0) {
      e = launch_regress(h1->R, h1->G, h1->S, m, k, regress_iters, p->eps_div, s);
      if (e != hipSuccess) st = fail(nullptr, NNRESCAL_EDEVICE, hipGetErrorString(e));
    }
    double f = 0.0, xn = 0.0;
    if (st == NNRESCAL_OK) st = objective_impl(h1, &f, &xn);
    if (st == NNRESCAL_OK) st = nnrescal_get_factors(h1, nullptr, keepR[ki]->as<float>(), 0);
    (void)hipStreamSynchronize(s);
    destroy_impl(h1);
    if (st != NNRESCAL_OK) return st;
    err[ki] = xn > 0 ? (float)std::sqrt(std::max(f, 0.0) / xn) : 0.0f;
    return NNRESCAL_OK;
  };
  // The pass over X costs the same for every rank of one 16-column block, and a member's perturbed tensor does not
  // depend on the rank: two ranks that fit one block together are fitted side by side in one handle (Dims::ksplit).
  // Going down from k_hi, a rank takes the largest free rank that still fits its own block as partner.
  struct Pack { int k_first, k_second; };        // k_second = 0: alone
  std::vector<Pack> packs;
  {
    const bool tiny = X->format == NNRESCAL_DENSE && n <= 64 && !p->no_fused_small;   // fitted by the single-launch kernel
    const bool may_pack = !p->no_rank_packing && p->start == 0 && !tiny;
    std::vector<bool> used(nk, false);
    for (int ki = nk - 1; ki >= 0; --ki) {
      if (used[ki]) continue;
      used[ki] = true;
      const int k = k_lo + ki;
      int partner = 0;
      if (may_pack) {
        int room = (int)round_up(k, 16) - k;
        if (k + room > n) room = (int)n - k;
        for (int kj = std::min(ki - 1, room - k_lo); kj >= 0; --kj)
          if (!used[kj]) { partner = k_lo + kj; used[kj] = true; break; }
      }
      packs.push_back({k, partner});
    }
  }
  for (const Pack& pack : packs) {
    nnrescal_params pk = *p;
    pk.k = pack.k_first + pack.k_second;
    pk.check_input = 0;
    nnrescal_handle* h = nullptr;
    st = init_impl(&h, X, &pk, pack.k_second ? pack.k_first : 0);
    if (st != NNRESCAL_OK) { cleanup(); return st; }
    st = fit_impl(h, iters);
    const int nmodels = pack.k_second ? 2 : 1;
    DevBuf* ens[2][2] = {{nullptr, nullptr}, {nullptr, nullptr}};
    auto drop = [&]() { for (auto& pr : ens) for (auto*& bfr : pr) { delete bfr; bfr = nullptr; } };
    for (int w = 0; w < nmodels && st == NNRESCAL_OK; ++w) {
      const int k = w == 0 ? pack.k_first : pack.k_second, ki = k - k_lo;
      ens[w][0] = new (std::nothrow) DevBuf(*p, (size_t)q * n * k * sizeof(float));
      ens[w][1] = new (std::nothrow) DevBuf(*p, (size_t)q * m * k * k * sizeof(float));
      keepA[ki] = new (std::nothrow) DevBuf(*p, (size_t)n * k * sizeof(float));
      keepR[ki] = new (std::nothrow) DevBuf(*p, (size_t)m * k * k * sizeof(float));
      if (!ens[w][0] || !ens[w][1] || !ens[w][0]->ptr || !ens[w][1]->ptr || !keepA[ki] || !keepR[ki] || !keepA[ki]->ptr ||
          !keepR[ki]->ptr)
        st = fail(nullptr, NNRESCAL_ENOMEM, "the alloc callback returned NULL");
      if (st == NNRESCAL_OK) st = get_factors_of_model(h, w, ens[w][0]->as<float>(), ens[w][1]->as<float>(), 1);
    }
    (void)hipStreamSynchronize(s);
    if (st == NNRESCAL_OK) st = device_error_status(h);
    destroy_impl(h);
    for (int w = 0; w < nmodels && st == NNRESCAL_OK; ++w)
      st = finish_rank((w == 0 ? pack.k_first : pack.k_second) - k_lo, *ens[w][0], *ens[w][1]);
    drop();
    if (st != NNRESCAL_OK) { cleanup(); return st; }
  }
  // section "Synthetic Data": low error, high minimum silhouette, largest separation between the two
  int best = 0;
  for (int ki = 1; ki < nk; ++ki)
    if (smin[ki] - err[ki] >= smin[best] - err[best]) best = ki;
  const int kb = k_lo + best;
  hipError_t e = hipSuccess;
  if (A_med_or_null)
    e = hipMemcpyAsync(A_med_or_null, keepA[best]->ptr, (size_t)n * kb * sizeof(float), hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess && R_reg_or_null)
    e = hipMemcpyAsync(R_reg_or_null, keepR[best]->ptr, (size_t)m * kb * kb * sizeof(float), hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  cleanup();
  if (e != hipSuccess) return fail(nullptr, NNRESCAL_EDEVICE, hipGetErrorString(e));
  std::copy(smin.begin(), smin.end(), s_min);
  std::copy(savg.begin(), savg.end(), s_avg);
  std::copy(err.begin(), err.end(), rel_err);
  *k_opt = kb;
  return NNRESCAL_OK;
}

}  // extern "C"
