// C ABI of the library (see include/nnrescal.h): handle management and the host-side orchestration of
// one multiplicative-update iteration (Alg. 3 of arxiv 2202.09512 with one process), of the objective
// (Eq. 1) and of the final normalisation.  Model selection (Alg. 1, 5, 6) lives in select.hip.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "api_internal.h"

using namespace nnr;

namespace nnr {
thread_local std::string g_last_error;

nnrescal_status fail(nnrescal_handle* h, nnrescal_status st, const std::string& msg) {
  if (h) h->err = msg;
  g_last_error = msg;
  return st;
}

void* dev_alloc(const nnrescal_params& p, size_t bytes) {
  if (bytes == 0) bytes = 4;
  return p.alloc(bytes, p.alloc_ctx);
}

nnrescal_status validate_tensor(const nnrescal_tensor* X, std::string& why) {
  if (!X) { why = "tensor is NULL"; return NNRESCAL_EINVAL; }
  if (X->n <= 0 || X->m <= 0) { why = "n and m must be positive"; return NNRESCAL_EINVAL; }
  if (X->n > 0x7FFFFFFFLL / 16) { why = "n too large (16*n must fit in 31 bits)"; return NNRESCAL_EINVAL; }
  switch (X->format) {
    case NNRESCAL_DENSE:
      if (!X->dense) { why = "format dense but dense pointer is NULL"; return NNRESCAL_EINVAL; }
      break;
    case NNRESCAL_CSR_CSC:
      if (!X->csc_colptr || !X->csc_row || !X->csc_slice_off) {
        why = "format CSR+CSC but a CSC pointer is NULL";
        return NNRESCAL_EINVAL;
      }
      if ((X->csc_val == nullptr) != (X->csr_val == nullptr)) {
        why = "csr_val and csc_val must both be given, or both be NULL (a binary tensor)";
        return NNRESCAL_EINVAL;
      }
      /* fall through */
    case NNRESCAL_CSR:
      if (!X->csr_rowptr || !X->csr_col || !X->csr_slice_off) {   // csr_val may be NULL: a binary tensor
        why = "sparse format but a CSR pointer is NULL";
        return NNRESCAL_EINVAL;
      }
      for (int t = 0; t < X->m; ++t) {
        if (X->csr_slice_off[t + 1] < X->csr_slice_off[t]) { why = "csr_slice_off must be non-decreasing"; return NNRESCAL_EINVAL; }
        if (X->csr_slice_off[t + 1] - X->csr_slice_off[t] > 0x7FFFFFFFLL * 64) { why = "slice too large"; return NNRESCAL_EINVAL; }
        if (X->format == NNRESCAL_CSR_CSC &&
            X->csc_slice_off[t + 1] - X->csc_slice_off[t] != X->csr_slice_off[t + 1] - X->csr_slice_off[t]) {
          why = "CSR and CSC copies of a slice differ in their number of non-zeros";
          return NNRESCAL_EINVAL;
        }
      }
      break;
    default:
      why = "unknown tensor format";
      return NNRESCAL_EINVAL;
  }
  return NNRESCAL_OK;
}

nnrescal_status validate_params(const nnrescal_tensor* X, const nnrescal_params* p, bool need_k, std::string& why) {
  if (!p) { why = "params is NULL"; return NNRESCAL_EINVAL; }
  if (!p->alloc || !p->dealloc) { why = "alloc and dealloc callbacks are required"; return NNRESCAL_EINVAL; }
  if (need_k && (p->k < 1 || p->k > NNRESCAL_MAX_K || p->k > X->n)) {
    why = "k must satisfy 1 <= k <= min(n, NNRESCAL_MAX_K)";
    return NNRESCAL_EINVAL;
  }
  if (p->q < 1 || p->q > NNRESCAL_MAX_Q) { why = "q must satisfy 1 <= q <= NNRESCAL_MAX_Q"; return NNRESCAL_EINVAL; }
  if (!(p->delta >= 0.0f && p->delta < 1.0f)) { why = "delta must satisfy 0 <= delta < 1"; return NNRESCAL_EINVAL; }
  // eps_div = 0 is not accepted: an entry whose numerator and denominator both vanish (a zero row of X, an R_t that
  // has become zero) would turn into NaN instead of staying 0
  if (!(p->eps_div > 0.0f) || !std::isfinite(p->eps_div)) { why = "eps_div must be finite and > 0"; return NNRESCAL_EINVAL; }
  if (p->gather_form < 0 || p->gather_form > kGatherLines) { why = "gather_form must be 0 or one of the NNRESCAL_GATHER_ constants"; return NNRESCAL_EINVAL; }
  if ((p->A0 == nullptr) != (p->R0 == nullptr)) { why = "A0 and R0 must be given together"; return NNRESCAL_EINVAL; }
  if (p->start != 0 && p->start != 1) { why = "start must be 0 (random) or 1 (SVD-based)"; return NNRESCAL_EINVAL; }
  if (p->start == 1 && (p->A0 || p->start_svd_iters < 1 || p->start_r_iters < 0 || !(p->start_floor_rel >= 0.0f))) {
    why = "the SVD-based start needs A0 = R0 = NULL, start_svd_iters >= 1, start_r_iters >= 0, start_floor_rel >= 0";
    return NNRESCAL_EINVAL;
  }
  return NNRESCAL_OK;
}

// ---- profiling ------------------------------------------------------------------------------------
Prof::Prof(nnrescal_handle* h_, int cls_) : h(h_), cls(cls_), start(nullptr), stop(nullptr) {
  if (h->prof_mode == 0 || (h->prof_mode == 2 && cls != 1 && cls != 2 && cls != 4 && cls != 5)) return;
  if (hipEventCreate(&start) != hipSuccess || hipEventCreate(&stop) != hipSuccess) { start = stop = nullptr; return; }
  (void)hipEventRecord(start, h->stream);
}
Prof::~Prof() {
  if (!start) return;
  (void)hipEventRecord(stop, h->stream);
  h->prof_events.push_back({cls, start, stop});
}

static void drain_profile(nnrescal_handle* h) {
  for (auto& pe : h->prof_events) {
    (void)hipEventSynchronize(pe.stop);
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, pe.start, pe.stop) == hipSuccess) {
      h->prof_ms[pe.cls] += ms;
      h->prof_n[pe.cls] += 1;
    }
    (void)hipEventDestroy(pe.start);
    (void)hipEventDestroy(pe.stop);
  }
  h->prof_events.clear();
}

nnrescal_status device_error_status(nnrescal_handle* h) {
  if (h->dev_error_pinned && *(volatile int32_t*)h->dev_error != 0)
    return fail(h, NNRESCAL_EDEVICE,
                "a bounded wait inside the dense pass over X ran out (hand-over of a tile column between two waves): "
                "the products of that launch are incomplete and the factors are not to be trusted");
  return NNRESCAL_OK;
}

// ---- building blocks of one iteration -------------------------------------------------------------
hipError_t compute_G(nnrescal_handle* h) {
  if (h->g_valid) return hipSuccess;
  Prof pf(h, 0);
  const Dims& d = h->d;
  h->g_valid = true;
  return launch_gram16(h->A, h->A, 0, h->G, 1, d, h->stream, nullptr, h->det_gram, h->det_gram_floats);
}

// S_t = A^T P_t for all m slices
static hipError_t compute_S(nnrescal_handle* h, bool s_cleared = false) {
  Prof pf(h, 0);
  const Dims& d = h->d;
  return launch_gram16(h->A, h->P, (int64_t)d.n * d.q * d.kp, h->S, d.m, d, h->stream, h->use_masks ? h->pmask : nullptr,
                       h->det_gram, h->det_gram_floats, s_cleared);
}

hipError_t dense_pass(nnrescal_handle* h, int only_slice, bool pq_cleared) {
  Dims d = h->d;
  const int64_t ps = (int64_t)d.n * d.q * d.kp;
  const float* X = h->X.dense;
  float *P = h->P, *Q = h->Q;
  DenseStreamOpts so;
  if (only_slice >= 0) {                           // one slice: the same launch on a tensor of one slice
    X += (int64_t)only_slice * d.n * d.n;
    P += (int64_t)only_slice * ps;
    Q += (int64_t)only_slice * ps;
    so.t_first = only_slice;                       // the random stream is keyed by the slice's own index
    d.m = 1;
  }
  const size_t bytes = (size_t)d.m * ps * sizeof(float);
  hipError_t e;
  {
    Prof pf(h, 3);
    if (!pq_cleared) {
      FillList fl;
      fl.add(P, bytes);
      fl.add(Q, bytes);
      if ((e = launch_fill_zero_multi(fl, h->stream)) != hipSuccess) return e;
    }
    if (!h->aop_valid) {
      if ((e = launch_pack_operand(h->A, h->A_op, d, h->stream)) != hipSuccess) return e;
      h->aop_valid = true;
    }
  }
  const DensePlan pl = dense_stream_plan(d);
  so.Ppart = h->det_ppart;                         // reproducible mode: panel sums stored, added up in order below
  so.timeout_flag = h->dev_error;
  so.spin_limit = h->p.handover_spin_limit;
  if (pl.full_groups > 0) {
    Prof pf(h, 1);
    if ((e = launch_dense_stream(X, h->A_op, P, Q, d, 0, h->p.seed, h->p.delta, h->stream, so)) != hipSuccess)
      return e;
  }
  if (pl.tail_members > 0) {
    Prof pf(h, 4);
    e = launch_dense_stream(X, h->A_op, P, Q, d, 1, h->p.seed, h->p.delta, h->stream, so);
  }
  if (e == hipSuccess && h->det_ppart) {
    Prof pf(h, 3);
    e = launch_reduce_parts(P, h->det_ppart, (int64_t)d.m * ps, dense_stream_panels(d), (int64_t)d.m * ps, 0, h->stream);
  }
  return e;
}

// values of a slice: NULL stays NULL (a binary tensor has no value array: every stored entry is 1)
// a sparse tensor with at least this many stored non-zeros is asked which form of the products suits it (init)
constexpr int64_t kGatherTuneMinNnz = (int64_t)1 << 22;

static inline const float* vals_at(const float* base, int64_t lo) { return base ? base + lo : nullptr; }

hipError_t sparse_pass_all(nnrescal_handle* h, bool want_q) {
  const Dims& d = h->d;
  hipError_t e = hipSuccess;
  if (!h->segs_dev) {
    for (int t = 0; t < d.m && e == hipSuccess; ++t) e = sparse_pass(h, t, want_q);
    return e;
  }
  const bool csc = h->X.format == NNRESCAL_CSR_CSC;
  const bool both = want_q && csc;
  bool cleared = true;                             // rows without non-zeros are zero already, in every product of the launch
  for (int t = 0; t < d.m; ++t) cleared = cleared && h->p_rows_cleared[t] && (!both || h->q_rows_cleared[t]);
  {
    Prof pf(h, 2);
    e = launch_spmm_gather_batched(h->segs_dev, both ? 2 * d.m : d.m, both ? h->blocks_pq : h->blocks_p, h->A, d, !cleared,
                                   h->p.seed, h->p.delta, h->stream, h->det_side, h->gather_form);
  }
  if (e != hipSuccess) return e;
  for (int t = 0; t < d.m; ++t) {
    h->p_rows_cleared[t] = true;
    if (both) h->q_rows_cleared[t] = true;
  }
  if (want_q && !csc) {
    const int64_t ps = (int64_t)d.n * d.q * d.kp;
    for (int t = 0; t < d.m && e == hipSuccess; ++t) {
      Prof pf(h, 2);
      const int64_t lo = h->csr_off[t], nnz = h->csr_off[t + 1] - lo;
      e = launch_spmm_scatter(h->csr_major + lo, h->X.csr_col + lo, vals_at(h->X.csr_val, lo), nnz, h->A,
                              h->Q + (int64_t)t * ps, d, t, h->p.seed, h->p.delta, h->stream);
    }
  }
  return e;
}

hipError_t sparse_pass(nnrescal_handle* h, int t, bool want_q) {
  const Dims& d = h->d;
  const int64_t lo = h->csr_off[t], nnz = h->csr_off[t + 1] - lo;
  const int64_t ps = (int64_t)d.n * d.q * d.kp;   // P and Q hold all m slices
  float* Pt = h->P + (int64_t)t * ps;
  float* Qt = h->Q + (int64_t)t * ps;
  hipError_t e;
  {
    Prof pf(h, 2);   // one event pair per product
    e = launch_spmm_gather(h->X.csr_rowptr + (int64_t)t * (d.n + 1), h->csr_major + lo, h->X.csr_col + lo,
                           vals_at(h->X.csr_val, lo), nnz, h->A, Pt, d, t, 0, !h->p_rows_cleared[t], h->p.seed, h->p.delta,
                           h->stream, h->det_side, h->gather_form);
    h->p_rows_cleared[t] = true;                  // the slice's own part of P: its empty rows stay zero from now on
  }
  if (e != hipSuccess || !want_q) return e;
  Prof pf(h, 2);
  if (h->X.format == NNRESCAL_CSR_CSC) {
    const int64_t lo2 = h->csc_off[t];
    e = launch_spmm_gather(h->X.csc_colptr + (int64_t)t * (d.n + 1), h->csc_major + lo2, h->X.csc_row + lo2,
                           vals_at(h->X.csc_val, lo2), nnz, h->A, Qt, d, t, 1, !h->q_rows_cleared[t], h->p.seed, h->p.delta,
                           h->stream, h->det_side, h->gather_form);
    h->q_rows_cleared[t] = true;
    return e;
  }
  return launch_spmm_scatter(h->csr_major + lo, h->X.csr_col + lo, vals_at(h->X.csr_val, lo), nnz, h->A, Qt, d, t, h->p.seed,
                             h->p.delta, h->stream);
}

#define HIPCHK(expr)                                                                        \
  do {                                                                                      \
    hipError_t _e = (expr);                                                                 \
    if (_e != hipSuccess)                                                                   \
      return fail(h, NNRESCAL_EDEVICE, std::string(#expr) + ": " + hipGetErrorString(_e)); \
  } while (0)

// sum_t ||X^q_t||_F^2 per member, once per handle
static nnrescal_status xnorm_enqueue(nnrescal_handle* h) {
  const Dims& d = h->d;
  if (!h->xnorm_valid) {
    HIPCHK(launch_fill_zero(h->xnorm, (size_t)d.q * sizeof(double), h->stream));
    if (h->X.format == NNRESCAL_DENSE) {
      HIPCHK(launch_dense_xnorm(h->X.dense, h->xnorm, d.n, d.m, d.q, h->p.seed, h->p.delta, h->stream, h->det_xnpart));
    } else {
      for (int t = 0; t < d.m; ++t) {
        const int64_t lo = h->csr_off[t], nnz = h->csr_off[t + 1] - lo;
        HIPCHK(launch_sparse_xnorm(h->csr_major + lo, h->X.csr_col + lo, vals_at(h->X.csr_val, lo), nnz, h->xnorm, d.n, t, d.q,
                                   h->p.seed, h->p.delta, h->stream, h->det_xnpart));
      }
    }
    h->xnorm_valid = true;
  }
  return NNRESCAL_OK;
}

nnrescal_status mu_step_impl(nnrescal_handle* h, bool with_objective) {
  const Dims& d = h->d;
  const float eps = h->p.eps_div;
  HIPCHK(compute_G(h));
  const bool dense = h->X.format == NNRESCAL_DENSE;
  const int64_t ps = (int64_t)d.n * d.q * d.kp;
  const bool s_cleared = h->det_gram == nullptr;
  {
    // everything that this iteration's kernels add into, cleared by ONE launch: the denominator core, the objective's
    // terms, on the dense path the two products of the pass over X, and A^T X_t A
    Prof pf(h, 3);
    FillList fl;
    fl.add(h->W, (size_t)d.q * d.k * d.k * sizeof(float));
    if (with_objective) fl.add(h->obj, (size_t)2 * d.q * sizeof(double));
    if (dense) {
      fl.add(h->P, (size_t)d.m * ps * sizeof(float));
      fl.add(h->Q, (size_t)d.m * ps * sizeof(float));
    }
    if (s_cleared) fl.add(h->S, (size_t)d.m * d.q * d.k * d.k * sizeof(float));
    HIPCHK(launch_fill_zero_multi(fl, h->stream));
  }
  if (with_objective) {
    nnrescal_status st = xnorm_enqueue(h);
    if (st != NNRESCAL_OK) return st;
  }
  if (dense) {
    HIPCHK(dense_pass(h, -1, true));
  } else {
    HIPCHK(sparse_pass_all(h, true));
  }
  HIPCHK(compute_S(h, s_cleared));
  {
    Prof pf(h, 3);
    // with h->obj: <S_t, R_t> and <G R_t G, R_t> of the factors before this update, at no extra pass over X
    HIPCHK(launch_r_update(h->G, h->S, h->R, h->W, with_objective ? h->obj : nullptr, h->Rp, h->Rq, 0, d.m, d, eps, 1,
                           h->stream, h->det_wpart, h->det_objpart));
  }
  {
    Prof pf(h, 5);
    // writes the new A (dense path: in both layouts) and its A^T A: G (and A_op) stay valid
    HIPCHK(launch_a_update16(h->A, h->A_op, h->P, h->Q, ps, h->Rp, h->Rq, h->W, h->G, d, eps, h->stream,
                             h->use_masks ? h->pmask : nullptr, h->use_masks ? h->qmask : nullptr, h->det_gram,
                             h->det_gram_floats));
  }
  h->iterations += 1;
  return NNRESCAL_OK;
}

nnrescal_status fit_impl(nnrescal_handle* h, int iters) {
  const Dims& d = h->d;
  if (iters > 0 && h->X.format == NNRESCAL_DENSE && !h->p.no_fused_small && h->prof_mode == 0 && d.ksplit == 0 &&
      tiny_fit_applies(d)) {
    HIPCHK(launch_tiny_fit(h->X.dense, h->A, h->R, d, iters, h->p.eps_div, h->p.seed, h->p.delta, h->stream));
    h->g_valid = false;
    h->aop_valid = false;
    h->iterations += iters;
    return NNRESCAL_OK;
  }
  for (int it = 0; it < iters; ++it) {
    nnrescal_status st = mu_step_impl(h);
    if (st != NNRESCAL_OK) return st;
  }
  return NNRESCAL_OK;
}

// Enqueue: obj[r] = (<S,R>, <G R G, R>) summed over slices for the current factors; xnorm if not cached.
nnrescal_status objective_enqueue(nnrescal_handle* h) {
  const Dims& d = h->d;
  HIPCHK(launch_fill_zero(h->obj, (size_t)2 * d.q * sizeof(double), h->stream));
  HIPCHK(compute_G(h));
  if (h->X.format == NNRESCAL_DENSE) {
    HIPCHK(dense_pass(h));
  } else {
    HIPCHK(sparse_pass_all(h, false));
  }
  HIPCHK(compute_S(h));
  HIPCHK(launch_r_update(h->G, h->S, h->R, nullptr, h->obj, nullptr, nullptr, 0, d.m, d, 0.0f, 0, h->stream, nullptr,
                         h->det_objpart));
  return xnorm_enqueue(h);
}

// Copy the enqueued objective terms to the host (synchronises) and combine them: f = ||X||^2 - 2<S,R> + <GRG,R>.
nnrescal_status read_objective(nnrescal_handle* h, double* objective, double* xnorm_sq_or_null) {
  const Dims& d = h->d;
  if (!h->host_scalars) return fail(h, NNRESCAL_ESTATE, "this handle has no host buffer for scalar results");
  double* o = h->host_scalars;
  double* xn = h->host_scalars + 2 * d.q;
  HIPCHK(hipMemcpyAsync(o, h->obj, (size_t)2 * d.q * sizeof(double), hipMemcpyDeviceToHost, h->stream));
  HIPCHK(hipMemcpyAsync(xn, h->xnorm, (size_t)d.q * sizeof(double), hipMemcpyDeviceToHost, h->stream));
  HIPCHK(hipStreamSynchronize(h->stream));
  if (nnrescal_status st = device_error_status(h); st != NNRESCAL_OK) return st;
  for (int r = 0; r < d.q; ++r) {
    const double f = xn[r] - 2.0 * o[2 * r] + o[2 * r + 1];
    if (!std::isfinite(f)) return fail(h, NNRESCAL_ENONFINITE, "objective is not finite");
    objective[r] = f;
    if (xnorm_sq_or_null) xnorm_sq_or_null[r] = xn[r];
  }
  return NNRESCAL_OK;
}

nnrescal_status objective_impl(nnrescal_handle* h, double* objective, double* xnorm_sq_or_null) {
  nnrescal_status st = objective_enqueue(h);
  if (st != NNRESCAL_OK) return st;
  return read_objective(h, objective, xnorm_sq_or_null);
}

void destroy_impl(nnrescal_handle* h) {
  if (!h) return;
  drain_profile(h);
  void* bufs[] = {h->A, h->A_op, h->Rp, h->Rq, h->R, h->G, h->S, h->W, h->P, h->Q, h->obj, h->xnorm, h->csr_major, h->csc_major,
                  h->own_csc_colptr, h->own_csc_row, h->own_csc_val, h->segs_dev, h->pmask, h->qmask, h->det_ppart, h->det_gram,
                  h->det_wpart, h->det_objpart, h->det_xnpart, h->det_side};
  for (void* b : bufs)
    if (b) h->p.dealloc(b, h->p.alloc_ctx);
  if (h->host_scalars) (void)hipHostFree(h->host_scalars);
  if (h->dev_error_pinned && h->dev_error) (void)hipHostFree(h->dev_error);
  delete h;
}

nnrescal_status build_csc_copy(const nnrescal_tensor* X, const nnrescal_params* p, int64_t** colptr, int32_t** row,
                               float** val) {
  hipStream_t s = (hipStream_t)p->stream;
  const int64_t n = X->n;
  const int m = X->m;
  const int64_t total = X->csr_slice_off[m];
  int64_t max_nnz = 0;
  for (int t = 0; t < m; ++t) max_nnz = std::max(max_nnz, X->csr_slice_off[t + 1] - X->csr_slice_off[t]);
  if (max_nnz >= ((int64_t)1 << 31)) return fail(nullptr, NNRESCAL_EINVAL, "a slice has 2^31 or more non-zeros");
  const size_t tmp_bytes = build_csc_tmp_bytes(max_nnz, n);
  *colptr = (int64_t*)dev_alloc(*p, (size_t)m * (n + 1) * sizeof(int64_t));
  *row = (int32_t*)dev_alloc(*p, (size_t)std::max<int64_t>(total, 1) * sizeof(int32_t));
  const bool binary = X->csr_val == nullptr;       // no value array: none is made for the copy either
  *val = binary ? nullptr : (float*)dev_alloc(*p, (size_t)std::max<int64_t>(total, 1) * sizeof(float));
  int32_t* rows_tmp = (int32_t*)dev_alloc(*p, (size_t)std::max<int64_t>(max_nnz, 1) * sizeof(int32_t));
  void* tmp = dev_alloc(*p, tmp_bytes);
  auto release = [&](bool all) {
    if (rows_tmp) p->dealloc(rows_tmp, p->alloc_ctx);
    if (tmp) p->dealloc(tmp, p->alloc_ctx);
    if (all) {
      if (*colptr) p->dealloc(*colptr, p->alloc_ctx);
      if (*row) p->dealloc(*row, p->alloc_ctx);
      if (*val) p->dealloc(*val, p->alloc_ctx);
      *colptr = nullptr; *row = nullptr; *val = nullptr;
    }
  };
  if (!*colptr || !*row || (!binary && !*val) || !rows_tmp || !tmp) {
    release(true);
    return fail(nullptr, NNRESCAL_ENOMEM, "the alloc callback returned NULL while building the CSC copy "
                                          "(nnrescal_params.no_csc_build = 1 fits from the CSR slices alone)");
  }
  hipError_t e = hipSuccess;
  for (int t = 0; t < m && e == hipSuccess; ++t) {
    const int64_t lo = X->csr_slice_off[t], nnz = X->csr_slice_off[t + 1] - lo;
    e = launch_expand_major(X->csr_rowptr + (int64_t)t * (n + 1), rows_tmp, n, nnz, s);
    if (e == hipSuccess)
      e = build_csc_slice(X->csr_col + lo, rows_tmp, vals_at(X->csr_val, lo), nnz, n, *colptr + (int64_t)t * (n + 1), *row + lo,
                          binary ? nullptr : *val + lo, tmp, tmp_bytes, s);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  release(e != hipSuccess);
  if (e != hipSuccess) return fail(nullptr, NNRESCAL_EDEVICE, std::string("building the CSC copy: ") + hipGetErrorString(e));
  return NNRESCAL_OK;
}

nnrescal_status init_impl(nnrescal_handle** out, const nnrescal_tensor* X, const nnrescal_params* p, int ksplit) {
  if (!out) return fail(nullptr, NNRESCAL_EINVAL, "out is NULL");
  std::string why;
  nnrescal_status st = validate_tensor(X, why);
  if (st == NNRESCAL_OK) st = validate_params(X, p, true, why);
  if (st != NNRESCAL_OK) return fail(nullptr, st, why);
  if (p->check_input) {
    st = check_input(X, p);
    if (st != NNRESCAL_OK) return st;
  }
  nnrescal_handle* h = new (std::nothrow) nnrescal_handle();
  if (!h) return fail(nullptr, NNRESCAL_ENOMEM, "host allocation failed");
  h->X = *X;
  h->p = *p;
  h->stream = (hipStream_t)p->stream;
  const bool dense = X->format == NNRESCAL_DENSE;
  Dims& d = h->d;
  d.n = X->n;
  d.m = X->m;
  d.k = p->k;
  d.q = p->q;
  d.kp = (int)round_up(p->k, 16);
  d.n_pad = round_up(X->n, 256);
  if (ksplit < 0 || ksplit >= p->k || (ksplit > 0 && (p->A0 || p->start != 0))) {
    delete h;
    return fail(nullptr, NNRESCAL_EINVAL, "two models in one handle need 0 < ksplit < k and the random start");
  }
  d.ksplit = ksplit;
  if (!dense) {
    h->p_rows_cleared.assign(X->m, false);
    h->q_rows_cleared.assign(X->m, false);
    h->csr_off.assign(X->csr_slice_off, X->csr_slice_off + X->m + 1);
    h->X.csr_slice_off = h->csr_off.data();
    if (X->format == NNRESCAL_CSR_CSC) {
      h->csc_off.assign(X->csc_slice_off, X->csc_slice_off + X->m + 1);
      h->X.csc_slice_off = h->csc_off.data();
    } else if (!p->no_csc_build) {
      // CSR only: the library makes the transposed copy itself, once, so that X_t^T A is a gather as well
      const nnrescal_status stc = build_csc_copy(&h->X, p, &h->own_csc_colptr, &h->own_csc_row, &h->own_csc_val);
      if (stc != NNRESCAL_OK) {
        const std::string msg = g_last_error;
        destroy_impl(h);
        return fail(nullptr, stc, msg);
      }
      h->X.format = NNRESCAL_CSR_CSC;
      h->X.csc_colptr = h->own_csc_colptr;
      h->X.csc_row = h->own_csc_row;
      h->X.csc_val = h->own_csc_val;
      h->csc_off = h->csr_off;
      h->X.csc_slice_off = h->csc_off.data();
    }
  }
  // pinned host memory: the objective terms are read back through it, and kernels report a wait that ran out in it
  if (hipHostMalloc((void**)&h->host_scalars, (size_t)3 * d.q * sizeof(double), hipHostMallocDefault) != hipSuccess ||
      hipHostMalloc((void**)&h->dev_error, sizeof(int32_t), hipHostMallocDefault) != hipSuccess) {
    (void)hipGetLastError();
    destroy_impl(h);
    return fail(nullptr, NNRESCAL_ENOMEM, "pinned host memory for scalar results could not be allocated");
  }
  h->dev_error_pinned = true;
  *h->dev_error = 0;
  const size_t row = (size_t)d.q * d.kp;
  const size_t kk = (size_t)d.k * d.k;
  struct Req { void** p; size_t bytes; };
  std::vector<Req> reqs = {
      {(void**)&h->A, (size_t)d.n_pad * row * sizeof(float)},
      {(void**)&h->R, (size_t)d.q * d.m * kk * sizeof(float)},
      {(void**)&h->G, (size_t)d.q * kk * sizeof(float)},
      {(void**)&h->S, (size_t)d.m * d.q * kk * sizeof(float)},
      {(void**)&h->W, (size_t)d.q * kk * sizeof(float)},
      {(void**)&h->P, (size_t)d.m * d.n * row * sizeof(float)},
      {(void**)&h->Q, (size_t)d.m * d.n * row * sizeof(float)},
      {(void**)&h->Rp, (size_t)d.q * d.m * d.kp * d.kp * sizeof(float)},
      {(void**)&h->Rq, (size_t)d.q * d.m * d.kp * d.kp * sizeof(float)},
      {(void**)&h->obj, (size_t)2 * d.q * sizeof(double)},
      {(void**)&h->xnorm, (size_t)d.q * sizeof(double)},
  };
  // 8 spare member slots behind the operand copy: a rounded-up tail group reads (and discards) up to 7 members
  // past q in the last tile
  if (dense) reqs.push_back({(void**)&h->A_op, ((size_t)d.n_pad * row + 8 * (size_t)d.kp * 16) * sizeof(float)});
  if (!dense) {
    const bool csc = h->X.format == NNRESCAL_CSR_CSC;
    reqs.push_back({(void**)&h->csr_major, (size_t)h->csr_off[d.m] * sizeof(int32_t)});
    if (csc) reqs.push_back({(void**)&h->csc_major, (size_t)h->csc_off[d.m] * sizeof(int32_t)});
    reqs.push_back({(void**)&h->segs_dev, (size_t)(csc ? 2 : 1) * d.m * sizeof(GatherSeg)});
    reqs.push_back({(void**)&h->pmask, (size_t)d.m * ceil_div(d.n, 32) * sizeof(uint32_t)});
    if (csc) reqs.push_back({(void**)&h->qmask, (size_t)d.m * ceil_div(d.n, 32) * sizeof(uint32_t)});
  }
  if (p->deterministic) {
    if (!dense && h->X.format != NNRESCAL_CSR_CSC) {
      destroy_impl(h);
      return fail(nullptr, NNRESCAL_EINVAL, "the reproducible mode needs a CSC copy of a sparse tensor (not with no_csc_build: "
                                            "X_t^T A from CSR slices alone is a scatter of atomic additions)");
    }
    h->det_gram_floats = ((size_t)2052 + (size_t)d.m * d.q) * kk;
    reqs.push_back({(void**)&h->det_gram, h->det_gram_floats * sizeof(float)});
    reqs.push_back({(void**)&h->det_wpart, (size_t)d.m * d.q * kk * sizeof(float)});
    reqs.push_back({(void**)&h->det_objpart, (size_t)d.m * d.q * 2 * sizeof(double)});
    reqs.push_back({(void**)&h->det_xnpart, (size_t)kXnormMaxBlocks * d.q * sizeof(double)});
    if (dense) {
      reqs.push_back({(void**)&h->det_ppart, (size_t)dense_stream_panels(d) * d.m * d.n * row * sizeof(float)});
    } else {
      int64_t blocks = 0;
      for (int t = 0; t < d.m; ++t) blocks += 2 * spmm_gather_blocks(h->csr_off[t + 1] - h->csr_off[t]);
      reqs.push_back({(void**)&h->det_side, (size_t)std::max<int64_t>(blocks, 1) * 4 * 2 * row * sizeof(float)});
    }
  }
  for (auto& r : reqs) {
    *r.p = dev_alloc(h->p, r.bytes);
    if (!*r.p) {
      destroy_impl(h);
      return fail(nullptr, NNRESCAL_ENOMEM, "the alloc callback returned NULL");
    }
  }
  auto bail = [&](hipError_t e, const char* what) {
    std::string msg = std::string(what) + ": " + hipGetErrorString(e);
    destroy_impl(h);
    return fail(nullptr, NNRESCAL_EDEVICE, msg);
  };
  hipError_t e;
  if (dense && (e = launch_fill_zero(h->A_op + (size_t)d.n_pad * row, 8 * (size_t)d.kp * 16 * sizeof(float), h->stream)) !=
                   hipSuccess)
    return bail(e, "clearing the operand padding");
  if (p->A0)
    e = launch_import_factors(h->A, h->R, p->A0, p->R0, d, h->stream);
  else
    e = launch_init_factors(h->A, h->R, d, p->seed, h->stream);
  if (e != hipSuccess) return bail(e, "initialising the factors");
  if (!dense) {
    for (int t = 0; t < d.m; ++t) {
      const int64_t lo = h->csr_off[t], nnz = h->csr_off[t + 1] - lo;
      if ((e = launch_expand_major(X->csr_rowptr + (int64_t)t * (d.n + 1), h->csr_major + lo, d.n, nnz, h->stream)) !=
          hipSuccess)
        return bail(e, "expanding CSR row pointers");
      if (h->X.format == NNRESCAL_CSR_CSC) {
        const int64_t lo2 = h->csc_off[t];
        if ((e = launch_expand_major(h->X.csc_colptr + (int64_t)t * (d.n + 1), h->csc_major + lo2, d.n, nnz,
                                     h->stream)) != hipSuccess)
          return bail(e, "expanding CSC column pointers");
      }
    }
  }
  if (!dense) {
    // the iteration's products in one launch: segment table and presence masks
    const bool csc = h->X.format == NNRESCAL_CSR_CSC;
    const int64_t ps = (int64_t)d.n * row, mw = ceil_div(d.n, 32);
    int64_t blk = 0;
    for (int f = 0; f < (csc ? 2 : 1); ++f)
      for (int t = 0; t < d.m; ++t) {
        const int64_t lo = f == 0 ? h->csr_off[t] : h->csc_off[t], nnz = h->csr_off[t + 1] - h->csr_off[t];
        GatherSeg sg;
        sg.ptr = (f == 0 ? h->X.csr_rowptr : h->X.csc_colptr) + (int64_t)t * (d.n + 1);
        sg.major = (f == 0 ? h->csr_major : h->csc_major) + lo;
        sg.minor = (f == 0 ? h->X.csr_col : h->X.csc_row) + lo;
        sg.val = vals_at(f == 0 ? h->X.csr_val : h->X.csc_val, lo);
        sg.out = (f == 0 ? h->P : h->Q) + (int64_t)t * ps;
        sg.nnz = nnz;
        sg.blk_first = blk;
        sg.t = t;
        sg.transposed = f;
        h->segs_host.push_back(sg);
        blk += spmm_gather_blocks(nnz);
        if (f == 0 && t == d.m - 1) h->blocks_p = blk;
        if ((e = launch_presence_mask(sg.ptr, (f == 0 ? h->pmask : h->qmask) + (int64_t)t * mw, d.n, h->stream)) != hipSuccess)
          return bail(e, "building the presence masks");
      }
    h->blocks_pq = blk;
    // how many rows exist at all: the masks are used only if they rule out more than a tenth of them (counted on the
    // device into the first word of obj, which nothing else uses yet; one synchronisation at init)
    {
      unsigned long long* cnt = reinterpret_cast<unsigned long long*>(h->obj);
      unsigned long long present = 0;
      if ((e = launch_fill_zero(cnt, sizeof(unsigned long long), h->stream)) != hipSuccess) return bail(e, "counting rows");
      if ((e = launch_popcount(h->pmask, (int64_t)d.m * mw, cnt, h->stream)) != hipSuccess) return bail(e, "counting rows");
      if (csc && (e = launch_popcount(h->qmask, (int64_t)d.m * mw, cnt, h->stream)) != hipSuccess) return bail(e, "counting rows");
      if ((e = hipMemcpyAsync(&present, cnt, sizeof(present), hipMemcpyDeviceToHost, h->stream)) != hipSuccess ||
          (e = hipStreamSynchronize(h->stream)) != hipSuccess)
        return bail(e, "counting rows");
      h->use_masks = (double)present < 0.9 * (double)d.n * d.m * (csc ? 2 : 1);
    }
    // (the table stays alive in the handle: the copy may read it after this call has returned)
    if ((e = hipMemcpyAsync(h->segs_dev, h->segs_host.data(), h->segs_host.size() * sizeof(GatherSeg), hipMemcpyHostToDevice,
                            h->stream)) != hipSuccess)
      return bail(e, "uploading the segment table");
    // The form of the products.  Left to the library, a large tensor is asked: one launch of the products per
    // form (after one that is not timed: it also clears the rows without non-zeros), the faster is kept.
    // The factors are the initial ones and X_t A, X_t^T A are overwritten by the first iteration anyway.
    if (p->gather_form != 0) {
      h->gather_form = spmm_gather_form_ok(p->gather_form, d) ? p->gather_form : kGatherRows;
    } else if (csc && !p->deterministic && h->csr_off[d.m] >= kGatherTuneMinNnz) {
      hipEvent_t ev0 = nullptr, ev1 = nullptr;
      if ((e = hipEventCreate(&ev0)) != hipSuccess || (e = hipEventCreate(&ev1)) != hipSuccess) {
        if (ev0) (void)hipEventDestroy(ev0);
        return bail(e, "creating events");
      }
      float best = 0.0f;
      int best_form = kGatherRows;
      e = sparse_pass_all(h, true);
      for (int form : {kGatherRows, kGatherLines}) {
        if (e != hipSuccess) break;
        if (!spmm_gather_form_ok(form, d)) continue;
        h->gather_form = form;
        float ms = 0.0f;
        if ((e = hipEventRecord(ev0, h->stream)) != hipSuccess || (e = sparse_pass_all(h, true)) != hipSuccess ||
            (e = hipEventRecord(ev1, h->stream)) != hipSuccess || (e = hipEventSynchronize(ev1)) != hipSuccess ||
            (e = hipEventElapsedTime(&ms, ev0, ev1)) != hipSuccess)
          break;
        if (form == kGatherRows || ms < best) {
          best = ms;
          best_form = form;
        }
      }
      (void)hipEventDestroy(ev0);
      (void)hipEventDestroy(ev1);
      if (e != hipSuccess) return bail(e, "timing the forms of the sparse products");
      h->gather_form = best_form;
    }
  }
  if (p->start == 1) {
    const nnrescal_status st1 = start_nndsvd_impl(h, p->start_svd_iters, p->start_r_iters, p->start_floor_rel, nullptr);
    if (st1 != NNRESCAL_OK) {
      const std::string msg = h->err;
      destroy_impl(h);
      return fail(nullptr, st1, msg);
    }
  }
  *out = h;
  return NNRESCAL_OK;
}

}  // namespace nnr

// ---- exported C ABI --------------------------------------------------------------------------------
extern "C" {

nnrescal_status nnrescal_init(nnrescal_handle** out, const nnrescal_tensor* X, const nnrescal_params* p) {
  return init_impl(out, X, p);
}

nnrescal_status nnrescal_mu_step(nnrescal_handle* h) {
  if (!h) return fail(nullptr, NNRESCAL_ESTATE, "handle is NULL");
  if (nnrescal_status st = device_error_status(h); st != NNRESCAL_OK) return st;
  return mu_step_impl(h);
}

nnrescal_status nnrescal_fit(nnrescal_handle* h, int32_t iters, double* objective_or_null) {
  if (!h) return fail(nullptr, NNRESCAL_ESTATE, "handle is NULL");
  if (iters < 0) return fail(h, NNRESCAL_EINVAL, "iters must be >= 0");
  nnrescal_status st = device_error_status(h);
  if (st != NNRESCAL_OK) return st;
  st = fit_impl(h, iters);
  if (st != NNRESCAL_OK) return st;
  if (objective_or_null) return objective_impl(h, objective_or_null, nullptr);
  return NNRESCAL_OK;
}

nnrescal_status nnrescal_fit_until(nnrescal_handle* h, int32_t max_iters, double tau, int32_t check_every,
                                   int32_t* iters_done, double* trace_or_null) {
  if (!h) return fail(nullptr, NNRESCAL_ESTATE, "handle is NULL");
  if (max_iters < 0 || check_every < 1 || !iters_done || !(tau == tau))
    return fail(h, NNRESCAL_EINVAL, "fit_until needs max_iters >= 0, check_every >= 1, a threshold and iters_done");
  if (nnrescal_status st = device_error_status(h); st != NNRESCAL_OK) return st;
  const int q = h->d.q;
  std::vector<double> f(q);
  *iters_done = 0;
  for (int l = 1; l <= max_iters; ++l) {
    const bool check = l % check_every == 0;
    nnrescal_status st = mu_step_impl(h, check);
    if (st != NNRESCAL_OK) return st;
    *iters_done = l;
    if (!check) continue;
    st = read_objective(h, f.data(), nullptr);
    if (st != NNRESCAL_OK) return st;
    double worst = f[0];
    for (int r = 0; r < q; ++r) {
      if (trace_or_null) trace_or_null[(size_t)(l / check_every - 1) * q + r] = f[r];
      if (f[r] > worst) worst = f[r];
    }
    if (worst < tau) break;
  }
  return NNRESCAL_OK;
}

nnrescal_status nnrescal_start_nndsvd(nnrescal_handle* h, int32_t svd_iters, int32_t r_iters, float floor_rel,
                                      float* sigma_or_null) {
  if (!h) return fail(nullptr, NNRESCAL_ESTATE, "handle is NULL");
  if (svd_iters < 1 || r_iters < 0 || !(floor_rel >= 0.0f))
    return fail(h, NNRESCAL_EINVAL, "start_nndsvd needs svd_iters >= 1, r_iters >= 0, floor_rel >= 0");
  return start_nndsvd_impl(h, svd_iters, r_iters, floor_rel, sigma_or_null);
}

nnrescal_status nnrescal_objective(nnrescal_handle* h, double* objective, double* xnorm_sq_or_null) {
  if (!h) return fail(nullptr, NNRESCAL_ESTATE, "handle is NULL");
  if (!objective) return fail(h, NNRESCAL_EINVAL, "objective is NULL");
  return objective_impl(h, objective, xnorm_sq_or_null);
}

nnrescal_status nnrescal_get_factors(nnrescal_handle* h, float* A_out, float* R_out, int32_t normalised) {
  if (!h) return fail(nullptr, NNRESCAL_ESTATE, "handle is NULL");
  if (nnrescal_status st = device_error_status(h); st != NNRESCAL_OK) return st;
  if (normalised) HIPCHK(compute_G(h));
  HIPCHK(launch_export_factors(A_out, R_out, h->A, h->R, h->G, normalised, h->d, h->stream));
  return NNRESCAL_OK;
}

}  // extern "C"

namespace nnr {
// one of the two models of a handle made with ksplit > 0: which = 0 -> columns [0, ksplit), 1 -> [ksplit, k)
nnrescal_status get_factors_of_model(nnrescal_handle* h, int which, float* A_out, float* R_out, int normalised) {
  if (!h) return fail(nullptr, NNRESCAL_ESTATE, "handle is NULL");
  const Dims& d = h->d;
  const int off = which == 0 ? 0 : d.ksplit, kb = d.ksplit == 0 ? d.k : (which == 0 ? d.ksplit : d.k - d.ksplit);
  if (normalised) HIPCHK(compute_G(h));
  HIPCHK(launch_export_factors(A_out, R_out, h->A, h->R, h->G, normalised, d, h->stream, off, kb));
  return NNRESCAL_OK;
}
}  // namespace nnr

extern "C" {

nnrescal_status nnrescal_products(nnrescal_handle* h, int32_t t, float* P_out, float* Q_out) {
  if (!h) return fail(nullptr, NNRESCAL_ESTATE, "handle is NULL");
  const Dims& d = h->d;
  if (t < 0 || t >= d.m) return fail(h, NNRESCAL_EINVAL, "slice index out of range");
  if (h->X.format == NNRESCAL_DENSE)
    HIPCHK(dense_pass(h, t));
  else
    HIPCHK(sparse_pass(h, t, true));
  const int64_t ps = (int64_t)d.n * d.q * d.kp;
  // P and Q use the row format of A: the plain (un-normalised) factor export copies slice t out
  HIPCHK(launch_export_factors(P_out, nullptr, h->P + (int64_t)t * ps, nullptr, nullptr, 0, d, h->stream));
  HIPCHK(launch_export_factors(Q_out, nullptr, h->Q + (int64_t)t * ps, nullptr, nullptr, 0, d, h->stream));
  return NNRESCAL_OK;
}

nnrescal_status nnrescal_set_factors(nnrescal_handle* h, const float* A, const float* R) {
  if (!h) return fail(nullptr, NNRESCAL_ESTATE, "handle is NULL");
  if (!A || !R) return fail(h, NNRESCAL_EINVAL, "A and R are both required");
  HIPCHK(launch_import_factors(h->A, h->R, A, R, h->d, h->stream));
  h->g_valid = h->aop_valid = false;
  return NNRESCAL_OK;
}

nnrescal_status nnrescal_perturb(const nnrescal_tensor* X, int32_t member, float delta, uint64_t seed,
                                 int32_t from_csc, void* stream, float* out) {
  nnrescal_handle* h = nullptr;
  std::string why;
  nnrescal_status st = validate_tensor(X, why);
  if (st != NNRESCAL_OK) return fail(nullptr, st, why);
  if (!out) return fail(nullptr, NNRESCAL_EINVAL, "out is NULL");
  if (member < 0 || member >= NNRESCAL_MAX_Q) return fail(nullptr, NNRESCAL_EINVAL, "member out of range");
  if (!(delta >= 0.0f && delta < 1.0f)) return fail(nullptr, NNRESCAL_EINVAL, "delta must satisfy 0 <= delta < 1");
  hipStream_t s = (hipStream_t)stream;
  if (X->format == NNRESCAL_DENSE) {
    HIPCHK(launch_dense_perturb(X->dense, out, X->n, X->m, member, seed, delta, s));
    return NNRESCAL_OK;
  }
  if (from_csc && X->format != NNRESCAL_CSR_CSC) return fail(nullptr, NNRESCAL_EINVAL, "from_csc needs a CSC copy");
  for (int t = 0; t < X->m; ++t) {
    if (from_csc) {
      const int64_t lo = X->csc_slice_off[t], nnz = X->csc_slice_off[t + 1] - lo;
      HIPCHK(launch_sparse_perturb(X->csc_colptr + (int64_t)t * (X->n + 1), X->csc_row + lo, vals_at(X->csc_val, lo), nnz,
                                   out + lo, X->n, t, 1, member, seed, delta, s));
    } else {
      const int64_t lo = X->csr_slice_off[t], nnz = X->csr_slice_off[t + 1] - lo;
      HIPCHK(launch_sparse_perturb(X->csr_rowptr + (int64_t)t * (X->n + 1), X->csr_col + lo, vals_at(X->csr_val, lo), nnz,
                                   out + lo, X->n, t, 0, member, seed, delta, s));
    }
  }
  return NNRESCAL_OK;
}

void nnrescal_destroy(nnrescal_handle* h) { destroy_impl(h); }

int32_t nnrescal_gather_form(const nnrescal_handle* h) { return h && h->segs_dev ? h->gather_form : 0; }

}  // extern "C"

// ---- one iteration without a handle and without any allocation ---------------------------------------
// Every workspace of the iteration is carved out of this array.  In host code its name is a stand-in, not a device
// address: the address on the current device comes from hipGetSymbolAddress, once per device, and only that pointer
// is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[NNRESCAL_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

void* no_alloc(size_t, void*) { return nullptr; }
void no_dealloc(void*, void*) {}

hipError_t scratch_on_current_device(unsigned char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = (unsigned char*)ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}
}  // namespace

extern "C" {

nnrescal_status nnrescal_mu_step_static(const nnrescal_tensor* X, const nnrescal_params* p, float* A, float* R,
                                        int32_t* status_or_null) {
  std::string why;
  nnrescal_status st = validate_tensor(X, why);
  nnrescal_params pp{};
  if (st == NNRESCAL_OK && !p) { st = NNRESCAL_EINVAL; why = "params is NULL"; }
  if (st == NNRESCAL_OK) {
    pp = *p;
    pp.alloc = no_alloc;               // never called: every buffer below comes from the static array
    pp.dealloc = no_dealloc;
    pp.A0 = pp.R0 = nullptr;
    pp.start = 0;
    st = validate_params(X, &pp, true, why);
  }
  if (st != NNRESCAL_OK) return fail(nullptr, st, why);
  if (!A || !R) return fail(nullptr, NNRESCAL_EINVAL, "A and R are required");
  nnrescal_handle hh;                  // lives on the host stack for the duration of the call
  nnrescal_handle* h = &hh;
  h->X = *X;
  h->p = pp;
  h->stream = (hipStream_t)pp.stream;
  const bool dense = X->format == NNRESCAL_DENSE;
  Dims& d = h->d;
  d.n = X->n;
  d.m = X->m;
  d.k = pp.k;
  d.q = pp.q;
  d.kp = (int)round_up(pp.k, 16);
  d.n_pad = round_up(X->n, 256);
  d.ksplit = 0;
  int64_t nnz = 0;
  if (!dense) {
    h->p_rows_cleared.assign(X->m, false);
    h->q_rows_cleared.assign(X->m, false);
    h->csr_off.assign(X->csr_slice_off, X->csr_slice_off + X->m + 1);
    h->X.csr_slice_off = h->csr_off.data();
    nnz = h->csr_off[X->m];
    if (X->format == NNRESCAL_CSR_CSC) {
      h->csc_off.assign(X->csc_slice_off, X->csc_slice_off + X->m + 1);
      h->X.csc_slice_off = h->csc_off.data();
    }
  }
  // the workspaces of nnrescal_init, one after the other in the static array (256-byte aligned each)
  const size_t row = (size_t)d.q * d.kp, kk = (size_t)d.k * d.k;
  const size_t pad = 8 * (size_t)d.kp * 16;      // spare member slots behind the operand copy (see init_impl)
  struct Req { void** p; size_t bytes; };
  Req reqs[] = {
      {(void**)&h->A, (size_t)d.n_pad * row * sizeof(float)},
      {(void**)&h->R, (size_t)d.q * d.m * kk * sizeof(float)},
      {(void**)&h->G, (size_t)d.q * kk * sizeof(float)},
      {(void**)&h->S, (size_t)d.m * d.q * kk * sizeof(float)},
      {(void**)&h->W, (size_t)d.q * kk * sizeof(float)},
      {(void**)&h->P, (size_t)d.m * d.n * row * sizeof(float)},
      {(void**)&h->Q, (size_t)d.m * d.n * row * sizeof(float)},
      {(void**)&h->Rp, (size_t)d.q * d.m * d.kp * d.kp * sizeof(float)},
      {(void**)&h->Rq, (size_t)d.q * d.m * d.kp * d.kp * sizeof(float)},
      {(void**)&h->A_op, dense ? ((size_t)d.n_pad * row + pad) * sizeof(float) : 0},
      {(void**)&h->csr_major, dense ? 0 : (size_t)nnz * sizeof(int32_t)},
      {(void**)&h->csc_major, X->format == NNRESCAL_CSR_CSC ? (size_t)nnz * sizeof(int32_t) : 0},
  };
  size_t need = 0;
  for (const Req& r : reqs) need += (r.bytes + 255) & ~(size_t)255;
  if (need > (size_t)NNRESCAL_STATIC_SCRATCH_BYTES)
    return fail(nullptr, NNRESCAL_EINVAL,
                "nnrescal_mu_step_static: this problem needs " + std::to_string(need) + " bytes of workspace, the static array holds " +
                    std::to_string((size_t)NNRESCAL_STATIC_SCRATCH_BYTES) + " (use nnrescal_init / nnrescal_mu_step)");
  unsigned char* base = nullptr;
  HIPCHK(scratch_on_current_device(&base));
  size_t off = 0;
  for (const Req& r : reqs) {
    *r.p = r.bytes ? (void*)(base + off) : nullptr;
    off += (r.bytes + 255) & ~(size_t)255;
  }
  h->dev_error = status_or_null;       // a device word of the caller's (or none)
  h->dev_error_pinned = false;
  if (status_or_null) HIPCHK(launch_fill_zero(status_or_null, sizeof(int32_t), h->stream));
  if (dense) HIPCHK(launch_fill_zero(h->A_op + (size_t)d.n_pad * row, pad * sizeof(float), h->stream));
  HIPCHK(launch_import_factors(h->A, h->R, A, R, d, h->stream));
  if (!dense) {
    for (int t = 0; t < d.m; ++t) {
      const int64_t lo = h->csr_off[t], nz = h->csr_off[t + 1] - lo;
      HIPCHK(launch_expand_major(X->csr_rowptr + (int64_t)t * (d.n + 1), h->csr_major + lo, d.n, nz, h->stream));
      if (X->format == NNRESCAL_CSR_CSC)
        HIPCHK(launch_expand_major(X->csc_colptr + (int64_t)t * (d.n + 1), h->csc_major + h->csc_off[t], d.n, nz, h->stream));
    }
  }
  st = mu_step_impl(h);
  if (st != NNRESCAL_OK) return fail(nullptr, st, h->err);
  HIPCHK(launch_export_factors(A, R, h->A, h->R, h->G, 0, d, h->stream));
  return NNRESCAL_OK;
}


const char* nnrescal_last_error(const nnrescal_handle* h_or_null) {
  if (h_or_null) return h_or_null->err.c_str();
  return g_last_error.c_str();
}

nnrescal_status nnrescal_profile(nnrescal_handle* h, int32_t enable, double* ms, int64_t* launches) {
  if (!h) return fail(nullptr, NNRESCAL_ESTATE, "handle is NULL");
  HIPCHK(hipStreamSynchronize(h->stream));
  drain_profile(h);
  if (nnrescal_status st = device_error_status(h); st != NNRESCAL_OK) return st;
  for (int c = 0; c < kProfClasses; ++c) {
    if (ms) ms[c] = h->prof_ms[c];
    if (launches) launches[c] = h->prof_n[c];
  }
  if (enable) {
    for (int c = 0; c < kProfClasses; ++c) { h->prof_ms[c] = 0.0; h->prof_n[c] = 0; }
  }
  h->prof_mode = enable == 2 ? 2 : (enable != 0 ? 1 : 0);
  return NNRESCAL_OK;
}

}  // extern "C"
