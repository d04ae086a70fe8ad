// Optional check of the input tensor at nnrescal_init (nnrescal_params.check_input): the multiplicative rules of Eq. 2
// (arxiv 2202.09512) keep the factors non-negative only for a non-negative X, and the sparse kernels rely on rows that
// are sorted by column without duplicates.  One pass over the values (and, for a sparse tensor, over the index
// arrays), one word of flags read back.
#include <string>

#include "api_internal.h"

namespace nnr {

enum : int32_t { kBadNonFinite = 1, kBadNegative = 2, kBadPointers = 4, kBadColumn = 8, kBadOrder = 16 };

__global__ void __launch_bounds__(256) check_values_kernel(const float* __restrict__ x, int64_t count,
                                                           int32_t* __restrict__ flags) {
  int32_t f = 0;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < count; p += (int64_t)gridDim.x * blockDim.x) {
    const float v = x[p];
    if (!(v - v == 0.0f)) f |= kBadNonFinite;      // NaN or infinity
    else if (v < 0.0f) f |= kBadNegative;
  }
  if (f) atomicOr(flags, f);
}

// pointers of one slice: ptr[0] = 0, non-decreasing, ptr[n] = nnz
__global__ void __launch_bounds__(256) check_pointers_kernel(const int64_t* __restrict__ ptr, int64_t n, int64_t nnz,
                                                             int32_t* __restrict__ flags) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i > n) return;
  bool bad = false;
  if (i == 0) bad = ptr[0] != 0 || ptr[n] != nnz;
  if (i < n) bad = bad || ptr[i] > ptr[i + 1] || ptr[i] < 0;
  if (bad) atomicOr(flags, (int32_t)kBadPointers);
}

// minor indices of one slice (its pointers have passed check_pointers_kernel): inside [0, n), strictly increasing
// inside a row (column)
__global__ void __launch_bounds__(256) check_indices_kernel(const int64_t* __restrict__ ptr, const int32_t* __restrict__ idx,
                                                            int64_t n, int64_t nnz, int32_t* __restrict__ flags) {
  int32_t f = 0;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += (int64_t)gridDim.x * blockDim.x) {
    const int32_t c = idx[p];
    if (c < 0 || c >= n) f |= kBadColumn;
    if (p > 0 && idx[p - 1] >= c) {                 // allowed only where a new row starts at p
      int64_t lo = 0, hi = n - 1;                   // largest r with ptr[r] <= p
      while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (ptr[mid] <= p) lo = mid; else hi = mid - 1;
      }
      if (ptr[lo] != p) f |= kBadOrder;
    }
  }
  if (f) atomicOr(flags, f);
}

static int grid_of(int64_t count) {
  int64_t b = (count + 255) / 256;
  return (int)(b < 1 ? 1 : (b > 16384 ? 16384 : b));
}

nnrescal_status check_input(const nnrescal_tensor* X, const nnrescal_params* p) {
  hipStream_t s = (hipStream_t)p->stream;
  int32_t* flags = (int32_t*)dev_alloc(*p, sizeof(int32_t));
  if (!flags) return fail(nullptr, NNRESCAL_ENOMEM, "the alloc callback returned NULL");
  int32_t host = 0;
  auto read_back = [&]() -> hipError_t {
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(&host, flags, sizeof(host), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    return e;
  };
  hipError_t e = launch_fill_zero(flags, sizeof(int32_t), s);
  const int64_t n = X->n;
  if (e == hipSuccess) {
    if (X->format == NNRESCAL_DENSE) {
      const int64_t count = (int64_t)X->m * n * n;
      hipLaunchKernelGGL(check_values_kernel, dim3(grid_of(count)), dim3(256), 0, s, X->dense, count, flags);
    } else {
      // the pointers first: the index check walks them
      for (int f = 0; f < (X->format == NNRESCAL_CSR_CSC ? 2 : 1); ++f)
        for (int t = 0; t < X->m; ++t) {
          const int64_t* off = f == 0 ? X->csr_slice_off : X->csc_slice_off;
          hipLaunchKernelGGL(check_pointers_kernel, dim3(grid_of(n + 1)), dim3(256), 0, s,
                             (f == 0 ? X->csr_rowptr : X->csc_colptr) + (int64_t)t * (n + 1), n, off[t + 1] - off[t], flags);
        }
    }
    e = read_back();
  }
  if (e == hipSuccess && host == 0 && X->format != NNRESCAL_DENSE) {
    for (int f = 0; f < (X->format == NNRESCAL_CSR_CSC ? 2 : 1); ++f)
      for (int t = 0; t < X->m; ++t) {
        const int64_t* off = f == 0 ? X->csr_slice_off : X->csc_slice_off;
        const int64_t lo = off[t], nnz = off[t + 1] - lo;
        if (nnz == 0) continue;
        hipLaunchKernelGGL(check_indices_kernel, dim3(grid_of(nnz)), dim3(256), 0, s,
                           (f == 0 ? X->csr_rowptr : X->csc_colptr) + (int64_t)t * (n + 1),
                           (f == 0 ? X->csr_col : X->csc_row) + lo, n, nnz, flags);
        const float* val = f == 0 ? X->csr_val : X->csc_val;
        if (val) hipLaunchKernelGGL(check_values_kernel, dim3(grid_of(nnz)), dim3(256), 0, s, val + lo, nnz, flags);
      }
    e = read_back();
  }
  p->dealloc(flags, p->alloc_ctx);
  if (e != hipSuccess) return fail(nullptr, NNRESCAL_EDEVICE, std::string("checking the input tensor: ") + hipGetErrorString(e));
  if (host & kBadPointers)
    return fail(nullptr, NNRESCAL_EINVAL, "check_input: a slice's row (column) pointers do not start at 0, are not non-decreasing, or do "
                                          "not end at the slice's number of stored entries");
  if (host & kBadColumn) return fail(nullptr, NNRESCAL_EINVAL, "check_input: a stored entry's index lies outside [0, n)");
  if (host & kBadOrder)
    return fail(nullptr, NNRESCAL_EINVAL, "check_input: the stored entries of a row (column) are not sorted, or a coordinate is stored twice");
  if (host & kBadNonFinite) return fail(nullptr, NNRESCAL_ENONFINITE, "check_input: X holds a NaN or an infinity");
  if (host & kBadNegative)
    return fail(nullptr, NNRESCAL_EINVAL, "check_input: X holds a negative entry (the multiplicative rules need X >= 0)");
  return NNRESCAL_OK;
}

}  // namespace nnr
