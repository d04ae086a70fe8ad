// Internal declarations shared by api.hip and select.hip.
#pragma once
#include <string>
#include <vector>

#include "../../include/nnrescal.h"
#include "common.h"
#include "kernels.h"

constexpr int kProfClasses = 6;  // gram_mul, dense pass (full groups), sparse pass, elementwise, dense pass (tail group), A rule

struct ProfEvent {
  int cls;
  hipEvent_t start, stop;
};

struct nnrescal_handle {
  nnrescal_tensor X{};
  nnrescal_params p{};
  nnr::Dims d{};
  hipStream_t stream = nullptr;
  std::vector<int64_t> csr_off, csc_off;  // host copies of the slice offsets
  std::vector<bool> p_rows_cleared, q_rows_cleared;  // sparse path, per slice: the rows without non-zeros are zero
  float *A = nullptr, *A_op = nullptr, *R = nullptr, *G = nullptr, *S = nullptr, *W = nullptr, *P = nullptr, *Q = nullptr,
        *Rp = nullptr, *Rq = nullptr;
  double *obj = nullptr, *xnorm = nullptr;
  double* host_scalars = nullptr;  // pinned host memory (3 q doubles) for the read-back of the objective terms
  // One word that kernels set when a bounded wait inside them ran out (the dense pass's hand-over of tile columns).
  // Handles made by nnrescal_init keep it in pinned host memory, so that every later call sees it without a copy;
  // the call that allocates nothing points it at a device word of the caller's.
  int32_t* dev_error = nullptr;
  bool dev_error_pinned = false;
  int32_t *csr_major = nullptr, *csc_major = nullptr;
  // sparse path: the products of all slices in one launch.  segs: the m segments X_t A (CSR), then, if there is a CSC
  // copy, the m segments X_t^T A; blocks_p / blocks_pq: workgroups of the first m / of all of them.
  std::vector<nnr::GatherSeg> segs_host;
  nnr::GatherSeg* segs_dev = nullptr;
  int64_t blocks_p = 0, blocks_pq = 0;
  int gather_form = nnr::kGatherRows;   // which form of the gather kernel the batched products use
  // which entity rows of X_t A (pmask) and of X_t^T A (qmask) exist at all: [m][ceil(n/32)] bit words
  uint32_t *pmask = nullptr, *qmask = nullptr;
  bool use_masks = false;  // the kernels that read X_t A and X_t^T A skip the rows the masks rule out (it pays when
                           // more than a tenth of the rows are empty; the masks cost a little otherwise)
  // the CSC copy that the library built itself from a CSR-only tensor (X.csc_* then point here)
  int64_t* own_csc_colptr = nullptr;
  int32_t* own_csc_row = nullptr;
  float* own_csc_val = nullptr;
  // the reproducible mode (nnrescal_params.deterministic): places for sums that are stored in pieces and added up in
  // a fixed order instead of atomically
  float* det_ppart = nullptr;     // dense: [panels][m][n][q][kp], X_t A per 128-column panel
  float* det_gram = nullptr;      // shares of the workgroups of a k x k product over row ranges
  size_t det_gram_floats = 0;
  float* det_wpart = nullptr;     // [m][q][k][k], the denominator core per slice
  double* det_objpart = nullptr;  // [m][q][2], the objective terms per slice
  double* det_xnpart = nullptr;   // [kXnormMaxBlocks][q], block sums of ||X||^2
  float* det_side = nullptr;      // sparse: [chunks][2][q kp], pieces of rows that cross chunk borders
  bool xnorm_valid = false;
  bool g_valid = false;    // G holds A^T A of the current A
  bool aop_valid = false;  // A_op holds the current A (dense path)
  int64_t iterations = 0;
  std::string err;
  int prof_mode = 0;       // 0 off, 1 every kernel class, 2 only the passes over X and the A rule (classes 1, 2, 4, 5)
  double prof_ms[kProfClasses] = {0, 0, 0, 0, 0, 0};
  int64_t prof_n[kProfClasses] = {0, 0, 0, 0, 0, 0};
  std::vector<ProfEvent> prof_events;
};

namespace nnr {

extern thread_local std::string g_last_error;

// RAII: HIP events around the launches of one kernel class on the handle's stream (only when profiling is on)
struct Prof {
  nnrescal_handle* h;
  int cls;
  hipEvent_t start, stop;
  Prof(nnrescal_handle* h, int cls);
  ~Prof();
};

nnrescal_status fail(nnrescal_handle* h, nnrescal_status st, const std::string& msg);
void* dev_alloc(const nnrescal_params& p, size_t bytes);
nnrescal_status validate_tensor(const nnrescal_tensor* X, std::string& why);
nnrescal_status validate_params(const nnrescal_tensor* X, const nnrescal_params* p, bool need_k, std::string& why);
// ksplit > 0: the handle fits TWO models of ranks ksplit and p->k - ksplit side by side (see Dims::ksplit); only
// fit_impl / mu_step_impl and get_factors_of_model are meant for such a handle (no objective, no given start)
nnrescal_status init_impl(nnrescal_handle** out, const nnrescal_tensor* X, const nnrescal_params* p, int ksplit = 0);
nnrescal_status get_factors_of_model(nnrescal_handle* h, int which, float* A_out, float* R_out, int normalised);
// with_objective: also enqueue the objective terms of the factors the iteration STARTS from (they fall out of
// the R rule's operands) into h->obj, and sum_t ||X^q_t||^2 into h->xnorm if it is not there yet
nnrescal_status mu_step_impl(nnrescal_handle* h, bool with_objective = false);
nnrescal_status read_objective(nnrescal_handle* h, double* objective, double* xnorm_sq_or_null);
// `iters` iterations: the single-launch kernel for small tensors where it applies, else mu_step_impl in a loop
nnrescal_status fit_impl(nnrescal_handle* h, int iters);
nnrescal_status objective_enqueue(nnrescal_handle* h);
nnrescal_status objective_impl(nnrescal_handle* h, double* objective, double* xnorm_sq_or_null);
void destroy_impl(nnrescal_handle* h);
// EDEVICE if a kernel of this handle has reported a wait that ran out (the factors are then not to be trusted);
// reliable after a synchronisation of the handle's stream, opportunistic before
nnrescal_status device_error_status(nnrescal_handle* h);
hipError_t compute_G(nnrescal_handle* h);
// the pass over X for the current A: P_t = X^q_t A, Q_t = X^q_t^T A into the handle's P and Q (dense: all slices)
// only_slice >= 0: that slice alone (its part of P and Q)
hipError_t dense_pass(nnrescal_handle* h, int only_slice = -1, bool pq_cleared = false);
hipError_t sparse_pass(nnrescal_handle* h, int t, bool want_q);
// all slices: one launch for every gather product when the handle has its segment table, slice by slice otherwise
hipError_t sparse_pass_all(nnrescal_handle* h, bool want_q);
// CSC copy of the CSR slices of X, built on the device into arrays from the alloc callback (the caller frees them with
// the dealloc callback); synchronises the stream.  ENOMEM if an allocation fails, EINVAL if a slice has 2^31 or more
// non-zeros.
nnrescal_status build_csc_copy(const nnrescal_tensor* X, const nnrescal_params* p, int64_t** colptr, int32_t** row,
                               float** val);
// nnrescal_params.check_input: one pass over X (values finite and >= 0; sparse: pointers consistent, indices in range,
// rows sorted without duplicates); synchronises.  EINVAL / ENONFINITE with a message, ENOMEM, EDEVICE.
nnrescal_status check_input(const nnrescal_tensor* X, const nnrescal_params* p);
nnrescal_status start_nndsvd_impl(nnrescal_handle* h, int svd_iters, int r_iters, float floor_rel, float* sigma_out);

}  // namespace nnr
