/*
 * nnrescal - non-negative RESCAL multiplicative updates with a fused perturbation ensemble,
 * for one AMD MI355X (gfx950).  C ABI; no C++ or framework types cross this boundary.
 *
 * Method: arxiv 2202.09512 ("Distributed non-negative RESCAL with Automatic Model Selection").
 *   X_t ~ A R_t A^T for every relation slice t, A >= 0 (n x k), R_t >= 0 (k x k)        (Eq. 1)
 *   multiplicative updates for R_t and A                                                  (Eq. 2, Alg. 3)
 *   an ensemble of q perturbed tensors X^q = X (*) Delta^q, Delta in [1-delta, 1+delta]   (Alg. 4)
 *   clustering of the q solutions, silhouettes, regression, relative error, choice of k   (Alg. 1, 5, 6)
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the current device; "host" pointers are ordinary
 *     host memory.  Every argument says which.
 *   - X is borrowed: it must stay valid and unchanged while a handle that was created from it is
 *     alive; the library never writes to it.
 *   - All device work is enqueued on the caller's stream.  A call synchronises that stream only
 *     when it returns values to the host (documented per call).
 *   - Factors and workspaces are owned by the handle and obtained only through the caller's
 *     alloc/dealloc callbacks (so that a framework's caching allocator can supply them).
 *   - Every call returns a status; on error, outputs are left untouched and
 *     nnrescal_last_error() describes the problem.  Nothing throws or aborts.
 *   - A handle is not thread-safe.  Handles on different streams are independent.
 *   - Ranks up to NNRESCAL_MAX_K and ensembles up to NNRESCAL_MAX_Q are supported.
 *
 * Two different small constants appear in the paper and must not be confused:
 *   delta    perturbation half-width (Alg. 4; the paper uses 0.005 ... 0.03)
 *   eps_div  guard added to the denominators of Eq. 2 (the paper uses about 1e-16)
 */
#ifndef NNRESCAL_H
#define NNRESCAL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define NNRESCAL_API __attribute__((visibility("default")))
#else
#define NNRESCAL_API
#endif

#define NNRESCAL_MAX_K 64
#define NNRESCAL_MAX_Q 64

typedef struct nnrescal_handle nnrescal_handle; /* opaque, owned by the library */

typedef enum {
  NNRESCAL_OK = 0,
  NNRESCAL_EINVAL = 1,     /* bad argument (see nnrescal_last_error) */
  NNRESCAL_ENOMEM = 2,     /* the alloc callback returned NULL */
  NNRESCAL_EDEVICE = 3,    /* a HIP call failed, or a kernel reported a bounded wait that ran out (see
                              nnrescal_params.handover_spin_limit); the handle's factors are then not to be trusted */
  NNRESCAL_ESTATE = 4,     /* call not valid in the handle's state */
  NNRESCAL_ENONFINITE = 5  /* a requested host result is not finite, or (nnrescal_params.check_input) X holds a NaN
                              or an infinity */
} nnrescal_status;

enum { NNRESCAL_DENSE = 0, NNRESCAL_CSR = 1, NNRESCAL_CSR_CSC = 2 };

/* The input tensor (n x n x m, non-negative).  All pointers are DEVICE pointers, borrowed.
 *   format NNRESCAL_DENSE:   dense[m][n][n], fp32, slice-major, each slice row-major (Alg. 1 states
 *                            X as m x n x n); the other pointers are ignored.
 *   format NNRESCAL_CSR:     per slice t a CSR matrix: csr_rowptr[t*(n+1) .. ] (n+1 int64 offsets that
 *                            are local to the slice), column indices and values of slice t start at
 *                            csr_slice_off[t] (HOST array of m+1 int64) inside csr_col / csr_val.
 *                            Rows sorted by column, no duplicate coordinates, values > 0.
 *                            By default nnrescal_init builds the CSC copy of the slices itself (see
 *                            nnrescal_params.no_csc_build); without it X_t^T A is formed with atomic adds
 *                            on the CSR stream.
 *   format NNRESCAL_CSR_CSC: additionally the same slices in CSC (csc_colptr, csc_row, csc_val,
 *                            csc_slice_off), used for X_t^T A.
 *   Binary tensors (Introduction: X[t][i][j] = 1 iff relation t links entity i to entity j): csr_val = NULL (and
 *   csc_val = NULL in format NNRESCAL_CSR_CSC: both or neither, else NNRESCAL_EINVAL) means that every stored entry
 *   is 1; no value array is read, and the CSC copy that the library builds has none either.
 */
typedef struct {
  int32_t format;
  int64_t n;
  int32_t m;
  const float *dense;
  const int64_t *csr_rowptr;
  const int32_t *csr_col;
  const float *csr_val;
  const int64_t *csr_slice_off; /* HOST, m+1 entries */
  const int64_t *csc_colptr;
  const int32_t *csc_row;
  const float *csc_val;
  const int64_t *csc_slice_off; /* HOST, m+1 entries */
} nnrescal_tensor;

typedef void *(*nnrescal_alloc_fn)(size_t bytes, void *ctx); /* returns DEVICE memory, 256-byte aligned, or NULL */
typedef void (*nnrescal_dealloc_fn)(void *ptr, void *ctx);

typedef struct {
  int32_t k;        /* rank, 1 <= k <= min(n, NNRESCAL_MAX_K) */
  int32_t q;        /* ensemble size r of Alg. 1, 1 <= q <= NNRESCAL_MAX_Q */
  float delta;      /* perturbation half-width of Alg. 4, 0 <= delta < 1; 0 = members see X itself */
  float eps_div;    /* division guard of Eq. 2, > 0 (1e-16f in the paper): with it 0 * 0 / (0 + eps_div) = 0, so
                       entries without any support in X stay 0 instead of becoming NaN */
  uint64_t seed;    /* seed of the counter-based random stream (perturbation and initialisation) */
  void *stream;     /* hipStream_t; NULL = the default stream */
  nnrescal_alloc_fn alloc;
  nnrescal_dealloc_fn dealloc;
  void *alloc_ctx;
  const float *A0;  /* optional DEVICE start A[q][n][k]; NULL = random start (Alg. 3 step 1) */
  const float *R0;  /* optional DEVICE start R[q][m][k][k]; NULL = random start */
  int32_t start;    /* 0: the random start (or A0/R0); 1: the SVD-based start of nnrescal_start_nndsvd, made by
                       nnrescal_init (and by nnrescal_select_k for every fit); A0/R0 must then be NULL */
  int32_t start_svd_iters;  /* with start = 1: the arguments of nnrescal_start_nndsvd */
  int32_t start_r_iters;
  float start_floor_rel;
  int32_t no_fused_small;   /* != 0: never use the single-launch kernel for tensors that fit one compute unit's
                               LDS (nnrescal_fit, nnrescal_select_k); the general kernels run instead */
  int32_t no_csc_build;     /* != 0: a tensor given as NNRESCAL_CSR is used as it is (X_t^T A then scatters with
                               atomic adds: several times slower per iteration).  By default nnrescal_init and
                               nnrescal_select_k build the CSC copy of the slices on the device once, in arrays
                               from the alloc callback (8 bytes per non-zero + 8 (n+1) m; sorted by column, rows
                               ascending inside a column), and run as with NNRESCAL_CSR_CSC */
  int32_t no_rank_packing;  /* != 0: nnrescal_select_k fits every rank in a handle of its own.  By default two
                               ranks whose columns fit one 16-column block together share a handle and with it
                               the passes over X (random start only; the two models stay independent: the same
                               starts and the same update rules, sums taken in another order) */
  int32_t check_input;      /* != 0: nnrescal_init (and nnrescal_select_k) first check X in one pass and synchronise:
                               every value finite (else NNRESCAL_ENONFINITE) and >= 0 (the multiplicative rules keep
                               the factors non-negative only then; else NNRESCAL_EINVAL); for a sparse tensor also
                               the pointer arrays (start at 0, non-decreasing, end at the slice's entry count), the
                               indices (inside [0, n)) and the order inside a row or column (strictly increasing: no
                               coordinate twice), each NNRESCAL_EINVAL.  By default X is trusted. */
  int32_t deterministic;    /* != 0: the reproducible mode.  By default sums that several workgroups share (X_t A over
                               the column panels of a dense slice, X_t^T A over its row chunks, rows of a sparse
                               product that cross chunk borders, the k x k products over row ranges, the denominator
                               core over slices, the objective terms) are finished with atomic additions, in whatever
                               order the hardware takes them: two runs agree to rounding, not bit for bit.  In this
                               mode every such sum is stored in pieces and added up in a fixed order: two runs on the
                               same input give the same bits (nnrescal_mu_step, nnrescal_fit, nnrescal_fit_until,
                               nnrescal_objective, nnrescal_products, and the fits inside nnrescal_select_k).  It costs
                               memory (dense: one copy of X_t A per 128-column panel) and some time, needs a CSC copy
                               for a sparse tensor (given or built: not with no_csc_build), and does not cover
                               nnrescal_start_nndsvd or the clustering step of nnrescal_select_k. */
  int32_t handover_spin_limit; /* 0: the default.  In the dense pass over X a wave takes a column of partial sums
                               over from its neighbouring wave and polls that wave's step count first, at most this
                               many times (default 2^20, about 30 ms; a wait normally ends after microseconds).  A
                               wait that runs out never passes silently: the wave skips that step's share of X_t^T A,
                               the kernel ends normally, and the handle reports NNRESCAL_EDEVICE from then on: at the
                               latest in the first call that synchronises (nnrescal_fit with an objective pointer,
                               nnrescal_fit_until, nnrescal_objective, nnrescal_profile, nnrescal_start_nndsvd,
                               nnrescal_select_k), and in any later call.  A negative value allows no poll at all, so that
                               every wait runs out at once: tests use it to see the error path. */
  int32_t gather_form;      /* sparse tensors with a CSC copy: how a pass over the stored non-zeros fetches the rows of A.
                               NNRESCAL_GATHER_ROWS: all q kp columns of a row at once (up to 256 per pass);
                               NNRESCAL_GATHER_LINES: one 128-byte line (32 columns) of every row per pass.  The results
                               agree to rounding.  Narrow passes ask for fewer distinct bytes at a time, so that more of
                               them are still in a cache when the next non-zero refers to them, and walk the coordinates
                               once per pass; which form is faster depends on how the tensor's non-zeros cluster.
                               0 (the default): nnrescal_init decides.  A tensor with fewer than 2^22 stored non-zeros
                               gets NNRESCAL_GATHER_ROWS; on a larger one the products are launched once per form at
                               init, on the tensor itself with the initial factors, timed with events, and the faster
                               form is kept (nnrescal_gather_form reports it).  The reproducible mode never times (a
                               choice made by a clock is not reproducible): with 0 it uses NNRESCAL_GATHER_ROWS. */
} nnrescal_params;

#define NNRESCAL_GATHER_ROWS 1
#define NNRESCAL_GATHER_LINES 2

/* Alg. 3 step 1: create a fit of all q ensemble members at rank p->k.  Allocates the factors and
 * workspaces and initialises A and R (from A0/R0, else from the random stream: a different start per
 * member).  Asynchronous for a dense tensor; for a sparse one it synchronises (it builds the CSC copy, counts the
 * rows that hold entries and, on large tensors, times the forms of the products: see gather_form; check_input and
 * start = 1 synchronise for any tensor).  Errors: EINVAL (sizes, NULL pointers, format/pointer mismatch, and what
 * check_input finds), ENOMEM, ENONFINITE (check_input), EDEVICE. */
NNRESCAL_API nnrescal_status nnrescal_init(nnrescal_handle **out, const nnrescal_tensor *X, const nnrescal_params *p);

/* One iteration of Alg. 3's outer loop (Eq. 2) for every member: A^T A; for every slice the pass
 * over X_t that forms X^q_t A and X^q_t^T A with the perturbation of Alg. 4 applied on the fly, the
 * R_t update, the accumulation of the A update; then the A update.  Asynchronous.  The call enqueues kernels on the
 * handle's stream and nothing else (no allocation, no memset or copy, no synchronisation), so a caller may capture
 * it into a HIP graph on that stream and replay it; make one iteration outside the capture first (a handle's first
 * iteration also forms A^T A, clears rows that stay empty, and sets kernel attributes). */
NNRESCAL_API nnrescal_status nnrescal_mu_step(nnrescal_handle *h);

/* `iters` iterations.  A dense tensor with n <= 64 whose m slices fit the LDS of one compute unit (150 KB
 * with the factors) is fitted by one launch for all iterations, one workgroup per member, unless
 * nnrescal_params.no_fused_small is set or profiling is on: at that size an iteration of the general
 * kernels is launch latency.  If objective_or_null (HOST, q doubles) is given, the objective of Eq. 1,
 * sum_t ||X^q_t - A R_t A^T||_F^2 of the factors after the last iteration, is evaluated with one
 * more pass over X and the stream is synchronised; otherwise asynchronous. */
NNRESCAL_API nnrescal_status nnrescal_fit(nnrescal_handle *h, int32_t iters, double *objective_or_null);

/* Alg. 3 with the termination rule of section "Distributed RESCAL" (last paragraph): iterate until the
 * reconstruction error of Eq. 1 is below the threshold tau, at most max_iters iterations.  The error is
 * evaluated for the factors at the START of every check_every-th iteration (l = check_every, 2*check_every,
 * ..., counting from 1): those values fall out of the operands of that iteration's R update, so a check
 * costs no pass over X, only a synchronisation.  The iteration of a check is still carried out; if every
 * member's value was below tau it is the last.  iters_done (HOST, required) receives the number of
 * iterations carried out; trace_or_null (HOST, [max_iters / check_every][q] doubles) receives the values
 * of the checks made, in order.  tau <= 0 never stops early.  Synchronises at every check.
 * Errors: EINVAL (max_iters < 0, check_every < 1, tau NaN, iters_done NULL), ENONFINITE. */
NNRESCAL_API nnrescal_status nnrescal_fit_until(nnrescal_handle *h, int32_t max_iters, double tau, int32_t check_every,
                                                int32_t *iters_done, double *trace_or_null);

/* The SVD-based start of section "Experiments" (algorithmic parameters, option 2; named with Alg. 1 and
 * Alg. 3 as the alternative to the random start): replaces the handle's factors, for every member on its own
 * perturbed tensor.  A: left factor of the non-negative double SVD (Boutsidis and Gallopoulos 2008) of the
 * concatenated unfoldings M = [X_1 .. X_m  X_1^T .. X_m^T]: column 0 is sqrt(s_0)|u_0|, column j keeps the
 * positive or the negative part of the singular pair (u_j, v_j), whichever has the larger product of norms,
 * scaled by sqrt(s_j ||u+-|| ||v+-||) / ||u+-||; entries below floor_rel times the mean of that factor are
 * raised to it (a zero never leaves zero under the multiplicative rules).  The leading singular pairs come
 * from svd_iters rounds of subspace iteration with a Rayleigh-Ritz step on M M^T (two passes over X per
 * round).  R: the random R of Alg. 3 step 1, then r_iters R-only updates of Eq. 2 with that A.
 * sigma_or_null (HOST, [q][k] floats) receives the singular values found.  The iteration count of the
 * handle restarts at 0.  Synchronises.  Errors: EINVAL (svd_iters < 1, r_iters < 0, floor_rel < 0), ENOMEM
 * (workspaces are allocated for the duration of the call: two arrays of the size of A, and for a dense tensor
 * 2 m more). */
NNRESCAL_API nnrescal_status nnrescal_start_nndsvd(nnrescal_handle *h, int32_t svd_iters, int32_t r_iters, float floor_rel,
                                                   float *sigma_or_null);

/* Objective of Eq. 1 for the current factors (HOST, q doubles) and, optionally, sum_t ||X^q_t||_F^2
 * (HOST, q doubles or NULL).  Synchronises. */
NNRESCAL_API nnrescal_status nnrescal_objective(nnrescal_handle *h, double *objective, double *xnorm_sq_or_null);

/* Copy the factors out: A_out DEVICE [q][n][k], R_out DEVICE [q][m][k][k] (either may be NULL).
 * normalised != 0 applies the final normalisation of section "Multiplicative Update Algorithm"
 * (unit Euclidean columns of A, inverse scaling in R) to the copy; the handle's own factors stay
 * as they are, so the fit can be continued.  Asynchronous. */
NNRESCAL_API nnrescal_status nnrescal_get_factors(nnrescal_handle *h, float *A_out, float *R_out, int32_t normalised);

/* The two products of the pass over X for the current factors and slice t (Alg. 3: XA, and XTAR before its
 * R_t factor): P_out[r][i][:] = sum_j X^r_t[i][j] A^r[j][:] and Q_out[r][j][:] = sum_i X^r_t[i][j] A^r[i][:],
 * DEVICE [q][n][k] each (either may be NULL).  The fit never needs them outside the library; the call exists
 * so that the dominant kernel can be checked row by row at sizes where a whole iteration cannot be recomputed.
 * Leaves the factors untouched.  Asynchronous.  Errors: EINVAL (t out of range). */
NNRESCAL_API nnrescal_status nnrescal_products(nnrescal_handle *h, int32_t t, float *P_out, float *Q_out);

/* Replace the factors (DEVICE, same layouts as get_factors; both required).  Asynchronous. */
NNRESCAL_API nnrescal_status nnrescal_set_factors(nnrescal_handle *h, const float *A, const float *R);

/* Alg. 4 made explicit: write the values of member `member` of the perturbed tensor,
 * out[...] = X[...] * Delta, DEVICE, in the storage order of X (dense: [m][n][n]; sparse: the order
 * of csr_val, or of csc_val if from_csc != 0).  The fit never materialises this; the call exists so
 * that the random stream can be checked.  Asynchronous on `stream`. */
NNRESCAL_API nnrescal_status nnrescal_perturb(const nnrescal_tensor *X, int32_t member, float delta, uint64_t seed,
                                 int32_t from_csc, void *stream, float *out);

/* Alg. 5 and Alg. 6 on an ensemble of solutions: A_ens DEVICE [q][n][k], R_ens DEVICE [q][m][k][k]
 * or NULL.  Outputs: perm HOST [q][k] (perm[r*k+s] = column of member r placed in cluster s),
 * A_med DEVICE [n][k] (element-wise median of the aligned members) or NULL, R_med DEVICE
 * [m][k][k] (median of the aligned cores) or NULL, s_min / s_avg HOST scalars (minimum over clusters
 * of the mean silhouette, and overall mean silhouette; cosine distance), rounds HOST (clustering
 * rounds used) or NULL.  Needs alloc/dealloc/stream from `p` (k, q taken from the arguments).
 * Synchronises. */
NNRESCAL_API nnrescal_status nnrescal_cluster(const float *A_ens, const float *R_ens, int64_t n, int32_t m, int32_t k,
                                 int32_t q, const nnrescal_params *p, int32_t *perm, float *A_med,
                                 float *R_med, float *s_min, float *s_avg, int32_t *rounds);

/* Alg. 1: for every k in [k_lo, k_hi]: fit the q members for `iters` iterations, normalise, cluster
 * (Alg. 5), silhouettes (Alg. 6), median factors, regression of X on the median A (R-only updates of
 * Eq. 2, regress_iters of them), relative error ||X - A R A^T||_F / ||X||_F.  Outputs (HOST, length
 * k_hi-k_lo+1): s_min, s_avg, rel_err; k_opt HOST: the k with the largest s_min - rel_err (ties: the
 * larger k).  A_med_or_null DEVICE [n][k_opt], R_reg_or_null DEVICE [m][k_opt][k_opt]: the robust
 * factors at k_opt (buffers must hold k_hi columns).  p->k is ignored.  Synchronises. */
NNRESCAL_API nnrescal_status nnrescal_select_k(const nnrescal_tensor *X, const nnrescal_params *p, int32_t k_lo,
                                  int32_t k_hi, int32_t iters, int32_t regress_iters, float *s_min,
                                  float *s_avg, float *rel_err, int32_t *k_opt, float *A_med_or_null,
                                  float *R_reg_or_null);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  One nnrescal_mu_step without a handle and without any allocation: A (DEVICE [q][n][k])
 * and R (DEVICE [q][m][k][k]) hold the factors on entry and the updated factors on return, X and the fields k, q,
 * delta, eps_div, seed, stream, handover_spin_limit of p are as for nnrescal_init (alloc, dealloc, A0, R0, the start
 * fields, check_input, deterministic and gather_form are ignored: sums shared by several workgroups are added
 * atomically, the sparse products take whole rows; a tensor given as NNRESCAL_CSR is used as it is, X_t^T A by atomic adds, no CSC copy is
 * built).  Every workspace of the iteration (the factors in the kernels' layouts, X_t A and X_t^T A of all slices,
 * the k x k matrices, the expanded row indices of a sparse tensor) lies in ONE static device array of
 * NNRESCAL_STATIC_SCRATCH_BYTES that the library holds on every GPU it is loaded on until the process ends.  A
 * problem takes about 4 q kp ((2 m + 2) n + 512) + 8 q m kp^2 bytes of it, kp = k rounded up to a multiple of 16,
 * plus 4 bytes per stored non-zero and format of a sparse tensor; one that takes more is rejected with
 * NNRESCAL_EINVAL before any device work, and the message names both figures.  All calls on one GPU share that array: calls that overlap in time on one
 * GPU (different streams or threads) race; calls on one stream are fine.  Nothing from an earlier call is reused
 * (what must start at zero is cleared by kernels, no memset).  status_or_null (DEVICE int32, may be NULL) is set
 * to 0 by the call and to 1 by a kernel whose bounded wait ran out (see handover_spin_limit): the caller reads it
 * when it next synchronises.  Asynchronous on p->stream; calls no hipMalloc, hipFree, hipHostMalloc or any other
 * allocating routine (its first call on a device looks up the array's address, which allocates nothing).
 * Errors: EINVAL (as nnrescal_init; A or R NULL; scratch need above the maximum), EDEVICE. */
#define NNRESCAL_STATIC_SCRATCH_BYTES (32u << 20)
NNRESCAL_API nnrescal_status nnrescal_mu_step_static(const nnrescal_tensor *X, const nnrescal_params *p, float *A, float *R,
                                                     int32_t *status_or_null);

/* The form of the sparse products that this handle uses (see nnrescal_params.gather_form): one of the
 * NNRESCAL_GATHER_ constants; 0 for a dense tensor, a tensor without a CSC copy, or h == NULL. */
NNRESCAL_API int32_t nnrescal_gather_form(const nnrescal_handle *h);

/* Release everything the handle owns (through dealloc).  NULL is allowed. */
NNRESCAL_API void nnrescal_destroy(nnrescal_handle *h);

/* Message of the last error on this handle, or (h == NULL) of the last error of a call that had no
 * handle, in this thread.  Never NULL. */
NNRESCAL_API const char *nnrescal_last_error(const nnrescal_handle *h_or_null);

/* Time spent per kernel class, measured with HIP events on the handle's stream around every launch
 * while profiling is on.  The call synchronises, returns what was accumulated so far (ms HOST
 * [NNRESCAL_PROF_CLASSES] milliseconds, launches HOST [NNRESCAL_PROF_CLASSES] event pairs; either may be
 * NULL), then switches profiling on (enable != 0: counters are reset) or off; enable == 2 times only the
 * passes over X and the A rule (classes 1, 2, 4 and 5), which perturbs a timed run less.  Classes follow the
 * paper's timing breakdown (section "Scalability"): 0 gram_mul (A^T A, A^T (X_t A)), 1 matrix_mul: the
 * dense pass over X for the groups of 8 members (one event pair = one kernel launch over all slices),
 * 2 matrix_mul_sparse (with a CSC copy one pair per iteration: the launch that clears shared rows and the launch of
 * both products of all slices; without one, a pair for X_t A of all slices and one per slice for the scatter form of
 * X_t^T A), 3 element-wise and k x k update kernels,
 * 4 the dense pass for the tail group of fewer than 8 members (one pair = one launch), 5 the A rule (the
 * n x k x k products of Eq. 2's second rule and the update itself; one pair per iteration, including the A^T A
 * pass that follows it for ranks above 32). */
#define NNRESCAL_PROF_CLASSES 6
NNRESCAL_API nnrescal_status nnrescal_profile(nnrescal_handle *h, int32_t enable, double *ms, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* NNRESCAL_H */
