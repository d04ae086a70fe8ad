// Host-side launchers of the HIP kernels.  Layouts (all fp32 unless noted):
//   A_int  [n_pad][q][kp]   entity-major factor of all members; kp = k rounded up to a multiple of 16;
//                           columns >= k and rows >= n are zero and stay zero
//   A_op   [n_pad/16][q][kp/16][64][4]   the same numbers in MFMA operand order (dense path only), rebuilt
//                           from A_int before every pass over X
//   R      [q][m][k][k]
//   G, W   [q][k][k]        A^T A and the k x k core of the A denominator
//   S      [m][q][k][k]     A^T X_t A
//   P, Q   [m][n][q][kp]    X^q_t A and X^q_t^T A of all slices
//   Rp, Rq [q][m][kp/16][kp/16][64][4]   the new R_t in MFMA operand order (see launch_r_update)
//   obj    double [q][2]    <S,R> and <G R G, R> summed over slices
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nnr {

struct Dims {
  int64_t n, n_pad;
  int32_t m, k, kp, q;
  // > 0: the k columns hold TWO independent models of the same members, columns [0, ksplit) and [ksplit, k):
  // they share the passes over X (a member's perturbed tensor does not depend on the rank); R_t is block-diagonal
  // and the R rule reads A^T A with its off-diagonal blocks masked, which is all that keeps the two apart
  int32_t ksplit = 0;
};

// ---- small kernels (kernels_small.hip)
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);
// several buffers in ONE launch (an iteration clears four or five; at small sizes a launch costs more than the clearing)
struct FillList {
  static constexpr int kMax = 6;
  void* p[kMax];
  size_t bytes[kMax];                              // multiples of 4
  int count = 0;
  void add(void* ptr, size_t nbytes) {
    if (ptr && nbytes && count < kMax) { p[count] = ptr; bytes[count] = nbytes; ++count; }
  }
};
hipError_t launch_fill_zero_multi(const FillList& fl, hipStream_t s);
// Fixed-order sums of partial results (the reproducible mode: partial sums are stored, not added atomically, and
// summed here in the order of their index): out[e] = (accumulate ? out[e] : 0) + parts[0][e] + parts[1][e] + ...,
// parts[p] = parts + p * stride, e < count.
hipError_t launch_reduce_parts(float* out, const float* parts, int64_t count, int64_t nparts, int64_t stride,
                               int accumulate, hipStream_t s);
hipError_t launch_reduce_parts_f64(double* out, const double* parts, int64_t count, int64_t nparts, int64_t stride,
                                   int accumulate, hipStream_t s);
hipError_t launch_init_factors(float* A_int, float* R, const Dims& d, uint64_t seed, hipStream_t s);
hipError_t launch_import_factors(float* A_int, float* R, const float* A_api, const float* R_api, const Dims& d,
                                 hipStream_t s);
// dnorm: [q][k] column norms or nullptr (no normalisation)
// col_off, kb: export the model in columns [col_off, col_off + kb) only (kb < 0: all d.k columns)
hipError_t launch_export_factors(float* A_api, float* R_api, const float* A_int, const float* R, const float* G,
                                 int normalised, const Dims& d, hipStream_t s, int col_off = 0, int kb = -1);
// Batched Gram product with a two-level batch index b = b1 * nb2 + b2:
//   out[b][a*ldo + c] = sum_i Y[i*ldy + b1*yb1 + b2*yb2 + a] * Z[i*ldz + b1*zb1 + b2*zb2 + c],  a < wa, c < wb.
// Zeroes the output first.
struct GramArgs {
  const float* Y; int64_t ldy, yb1, yb2; int wa;
  const float* Z; int64_t ldz, zb1, zb2; int wb;
  float* out; int64_t obatch; int ldo;
  int64_t n; int nb1, nb2;
};
hipError_t launch_gram(const GramArgs& g, hipStream_t s);
// R rule of Eq. 2 for slices [t0, t0+tc) of every member (+ W accumulation, + objective terms).
// Rp, Rq (both or neither): copies of the new R_t in MFMA operand order for launch_a_update16,
//   [q][m][kp/16][kp/16][64][4]: Rp[..][bb][cb][lane][r] = R_t[16*cb + lane%16][16*bb + 4*(lane/16) + r],
//   Rq[..][bb][cb][lane][r] = R_t[16*bb + 4*(lane/16) + r][16*cb + lane%16], zero outside k x k.
// Wpart ([m][q][k][k]) / objpart ([m][q][2] doubles), both optional: the reproducible mode.  Every (slice, member)
// block stores its share of W / of the objective terms there instead of adding it atomically, and the shares are then
// summed over the slices in order.
hipError_t launch_r_update(const float* G, const float* S, float* R, float* W, double* obj, float* Rp, float* Rq,
                           int t0, int tc, const Dims& d, float eps, int update, hipStream_t s, float* Wpart = nullptr,
                           double* objpart = nullptr);
// Element-wise median over members of the aligned ensemble: M[i][s] = median_r E[i][r][perm[r][s]].
hipError_t launch_median(float* M, int ldm, const float* E_int, const int32_t* perm_dev, const Dims& d,
                         hipStream_t s);
// M[i][c] = E[i][member][c] (Alg. 5, first statement: the centroid starts as one member's solution)
hipError_t launch_copy_member(float* M, int ldm, const float* E_int, int member, const Dims& d, hipStream_t s);
// iters R-only updates with constant G [k][k] and S [m][k][k] (regression step of model selection).
hipError_t launch_regress(float* R, const float* G, const float* S, int m, int k, int iters, float eps,
                          hipStream_t s);
// [q][n][k] API layout <-> [n_pad][q][kp] internal layout, A only
hipError_t launch_to_internal(float* E_int, const float* A_api, const Dims& d, hipStream_t s);
hipError_t launch_from_internal_single(float* A_api_nk, const float* M, int ldm, int64_t n, int k, hipStream_t s);

// ---- matrix-core versions for the dense path's row format, kp a multiple of 16 (kernels_update.hip)
// out[(b1*q + mem)][a][c] = sum_i Y[i][mem][a] * Z[b1*zstride + ...][i][mem][c] (a, c < k); zeroes out first.
// zmask (optional, DEVICE, [nb1][ceil(n / 32)] words): bit i of entry b1 says whether row i of Z_b1 holds anything;
// rows that do not must be zero and are not read.
// det_part (optional, DEVICE, det_part_floats floats): the reproducible mode.  The workgroups that share a product
// store their partial results there and a second kernel sums them in order, instead of atomic additions.
hipError_t launch_gram16(const float* Y, const float* Z, int64_t zstride, float* out, int nb1, const Dims& d,
                         hipStream_t s, const uint32_t* zmask = nullptr, float* det_part = nullptr,
                         size_t det_part_floats = 0, bool out_cleared = false);
// The whole A rule over all m slices; also writes the operand-order copy A_op of the new A and G = A^T A of
// the new A (G is cleared first).  Rp, Rq as written by launch_r_update.  det_part (as for launch_gram16): the new
// A^T A is then never accumulated inside the rule's kernel but always by a Gram pass with ordered sums.  pmask, qmask (optional, DEVICE,
// [m][ceil(n / 32)] words): which rows of P_t and Q_t hold anything (the others must be zero and are not read).
hipError_t launch_a_update16(float* A_int, float* A_op, const float* P, const float* Q, int64_t pq_slice_stride,
                             const float* Rp, const float* Rq, const float* W, float* G, const Dims& d, float eps,
                             hipStream_t s, const uint32_t* pmask = nullptr, const uint32_t* qmask = nullptr,
                             float* det_part = nullptr, size_t det_part_floats = 0);

// ---- dense pass over X (kernels_dense.hip)
// A_op[tile][member][block][lane][r] = A_int[16*tile + 4*(lane/16) + r][member][16*block + lane%16]
// n_rows: rows that A_int really holds (default: n_pad); the rest of the copy is zero
hipError_t launch_pack_operand(const float* A_int, float* A_op, const Dims& d, hipStream_t s, int64_t n_rows = -1);
// For every slice t and member r: P[t][i][r][:] = sum_j X[t][i][j] Delta^r[t][i][j] A[j][r][:],
//                                 Q[t][j][r][:] = sum_i X[t][i][j] Delta^r[t][i][j] A[i][r][:].
// P and Q must be zero on entry (partial sums are added atomically); the launcher does not clear them.
// The members are processed in groups that share one Philox block: `full` launches cover the groups of
// 8 members (4 for kp = 32, 2 for kp > 32), `tail` the remaining members rounded up to a power of two.
// part 0 = full groups, part 1 = tail group; a part with no members launches nothing.
struct DensePlan {
  int full_groups, full_qb, tail_members, tail_qb;
};
DensePlan dense_stream_plan(const Dims& d);
int64_t dense_stream_panels(const Dims& d);   // 128-column panels of a slice
struct DenseStreamOpts {
  int t_first = 0;               // slice index that X (and P, Q) start at, for callers that pass a part of the tensor:
                                 // the random stream is keyed by the slice's index in the whole tensor
  const float* A_opQ = nullptr;  // right operand of the second product (X^T .), if it is to differ from the first one's
  int64_t aop_tstride = 0;       // floats between the operand arrays of consecutive slices (0: the same for every slice)
  int64_t out_tstride = -1;      // floats between the slices of P and of Q (default n*q*kp; 0 sums the products over
                                 // the slices)
  int32_t* timeout_flag = nullptr;  // set to 1 (device or pinned host word) when a bounded wait inside the kernel ran
                                 // out: the products are then incomplete and the caller must report an error
  float* Ppart = nullptr;        // the reproducible mode: [panels][the layout of P] partial sums of X_t A, one per
                                 // 128-column panel, stored instead of added atomically (the caller sums them in
                                 // order); every workgroup then takes all rows of its panel, so that X_t^T A is
                                 // stored by its only writer as well
  int spin_limit = 0;            // polls a wave makes while it waits for its neighbour (0: the default, 2^20;
                                 // negative: none, every wait runs out at once)
};
hipError_t launch_dense_stream(const float* X, const float* A_op, float* P, float* Q, const Dims& d, int part,
                               uint64_t seed, float delta, hipStream_t s, const DenseStreamOpts& o = DenseStreamOpts());
hipError_t launch_dense_perturb(const float* X, float* out, int64_t n, int m, int member, uint64_t seed,
                                float delta, hipStream_t s);
// xn[r] += sum (X * Delta^r)^2 over all slices (double [q], zeroed by the caller)
// part (optional, [kXnormMaxBlocks][q] doubles): the reproducible mode, block sums stored and added in order
constexpr int kXnormMaxBlocks = 4096;
hipError_t launch_dense_xnorm(const float* X, double* xn, int64_t n, int m, int q, uint64_t seed, float delta,
                              hipStream_t s, double* part = nullptr);
const char* dense_stream_kernel_name();

// ---- tensors that fit one CU's LDS (kernels_tiny.hip): `iters` whole iterations in one launch, one workgroup per member
bool tiny_fit_applies(const Dims& d);
hipError_t launch_tiny_fit(const float* X, float* A_int, float* R, const Dims& d, int iters, float eps, uint64_t seed,
                           float delta, hipStream_t s);

// ---- sparse pass over X (kernels_sparse.hip)
// major[p] = row (CSR) or column (CSC) of stored non-zero p, expanded once from the pointer array.
hipError_t launch_expand_major(const int64_t* ptr, int32_t* major, int64_t n, int64_t nnz, hipStream_t s);
// ---- the CSC copy of CSR slices, built on the device (transpose.hip)
size_t build_csc_tmp_bytes(int64_t max_nnz, int64_t n);
hipError_t build_csc_slice(const int32_t* csr_col, const int32_t* row_of_entry, const float* val, int64_t nnz, int64_t n,
                           int64_t* colptr_out, int32_t* row_out, float* val_out, void* tmp, size_t tmp_bytes,
                           hipStream_t s);
// One product of one slice for the gather kernel: the slice's n+1 row (column) pointers, its non-zeros in coordinate
// form (major expanded from the pointers, minor, val; val == nullptr: a binary tensor, every stored entry is 1), the
// product's rows [n][q][kp], and, in a launch over several segments, the number of the segment's first workgroup.
struct GatherSeg {
  const int64_t* ptr;
  const int32_t* major;
  const int32_t* minor;
  const float* val;
  float* out;
  int64_t nnz;
  int64_t blk_first;
  int32_t t, transposed;
};
// workgroups that the gather kernel needs for a segment of nnz non-zeros
int64_t spmm_gather_blocks(int64_t nnz);
// All segments in one launch (segs_dev: DEVICE array of nseg entries whose blk_first are the running sums of
// spmm_gather_blocks, total_blocks their sum); clear_empty as below, for every segment.
// side (optional, DEVICE, [4 * total_blocks][2][q * kp] floats): the reproducible mode.  A wavefront stores the partial
// sums of a row that it shares with a neighbouring chunk there (slot 0: a row that continues from the chunk before,
// slot 1: a row that goes on into the next chunk) and a second kernel sums the pieces of every such row in chunk
// order, instead of atomic additions.
// form: how a pass over the non-zeros gathers the factor rows.  kGatherRows: all q * kp columns of a row (in one pass
// up to 256 columns); kGatherLines: one 128-byte line (32 columns) of every row per pass, eight lines per gather
// instruction.  Narrow passes want fewer distinct bytes at a time (more of them stay in the L2s) and walk the
// coordinates more often; which is faster depends on the tensor.  A form that the shape does not admit runs as
// kGatherRows.  Both forms know the reproducible mode's `side` buffer.
enum { kGatherRows = 1, kGatherLines = 2 };
bool spmm_gather_form_ok(int form, const Dims& d);
hipError_t launch_spmm_gather_batched(const GatherSeg* segs_dev, int nseg, int64_t total_blocks, const float* A_int,
                                      const Dims& d, int clear_empty, uint64_t seed, float delta, hipStream_t s,
                                      float* side = nullptr, int form = kGatherRows);
// mask[w] bit b: entity row (column) 32 w + b of the slice holds a stored non-zero (ceil(n / 32) words)
hipError_t launch_presence_mask(const int64_t* ptr, uint32_t* mask, int64_t n, hipStream_t s);
// *count (DEVICE) += set bits of nwords mask words
hipError_t launch_popcount(const uint32_t* mask, int64_t nwords, unsigned long long* count, hipStream_t s);
// One compressed slice in coordinate form (major, minor, val), sorted by major.  CSR: major = row,
// transposed = 0; CSC: major = column, transposed = 1 (only the random stream needs to know).
//   out[major][r][:] = sum over the non-zeros of that major index of val * Delta^r[t][i][j] * A[minor][r][:]
// ptr: the slice's n+1 row (column) pointers.  Rows with non-zeros are (re)written.  clear_empty != 0: rows
// without non-zeros are cleared too; a caller that keeps `out` for this slice alone needs that only once, since
// nothing ever writes those rows.
hipError_t launch_spmm_gather(const int64_t* ptr, const int32_t* major, const int32_t* minor, const float* val,
                              int64_t nnz, const float* A_int, float* out, const Dims& d, int t, int transposed,
                              int clear_empty, uint64_t seed, float delta, hipStream_t s, float* side = nullptr,
                              int form = kGatherRows);
// CSR stream, scatter form: out is cleared, then out[col][r][:] += val * Delta * A[row][r][:] (atomics; used when
// no CSC is given)
hipError_t launch_spmm_scatter(const int32_t* major, const int32_t* minor, const float* val, int64_t nnz,
                               const float* A_int, float* out, const Dims& d, int t, uint64_t seed, float delta,
                               hipStream_t s);
hipError_t launch_sparse_perturb(const int64_t* ptr, const int32_t* idx, const float* val, int64_t nnz, float* out,
                                 int64_t n, int t, int transposed, int member, uint64_t seed, float delta,
                                 hipStream_t s);
// xn[r] += sum (val * Delta^r)^2 over one CSR slice (double [q])
hipError_t launch_sparse_xnorm(const int32_t* major, const int32_t* minor, const float* val, int64_t nnz, double* xn,
                               int64_t n, int t, int q, uint64_t seed, float delta, hipStream_t s, double* part = nullptr);

}  // namespace nnr
