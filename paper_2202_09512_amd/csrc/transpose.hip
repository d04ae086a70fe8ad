// The CSC copy of CSR slices, built on the device (section "Distributed RESCAL": the sparse tensor is stored slice
// by slice; X_t^T A wants the transposed view).  Without it X_t^T A has to scatter with atomics; with it both products
// are gathers.  A stable sort of the row-major entries by column gives columns ascending and rows ascending inside a
// column, so the copy (and every sum taken along it) is the same in every run.
#include <hipcub/hipcub.hpp>

#include "common.h"
#include "kernels.h"

namespace nnr {

__global__ void __launch_bounds__(256) csc_count_kernel(const int32_t* __restrict__ col, int64_t nnz,
                                                        int32_t* __restrict__ cnt) {
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += (int64_t)gridDim.x * blockDim.x)
    atomicAdd(&cnt[col[p]], 1);
}

__global__ void __launch_bounds__(256) csc_iota_kernel(int32_t* __restrict__ idx, int64_t nnz) {
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += (int64_t)gridDim.x * blockDim.x)
    idx[p] = (int32_t)p;
}

__global__ void __launch_bounds__(256) csc_gather_kernel(const int32_t* __restrict__ perm,
                                                         const int32_t* __restrict__ row_of_entry,
                                                         const float* __restrict__ val, int64_t nnz,
                                                         int32_t* __restrict__ row_out, float* __restrict__ val_out) {
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += (int64_t)gridDim.x * blockDim.x) {
    const int32_t src = perm[p];
    row_out[p] = row_of_entry[src];
    if (val) val_out[p] = val[src];            // a binary tensor has no value array
  }
}

static int key_bits(int64_t n) {
  int b = 1;
  while (((int64_t)1 << b) < n) ++b;
  return b;
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// bytes of scratch for one slice of at most max_nnz entries: counts, the entry numbers, two sort outputs, the
// library's own scratch
size_t build_csc_tmp_bytes(int64_t max_nnz, int64_t n) {
  size_t sort_tmp = 0, scan_tmp = 0;
  (void)hipcub::DeviceRadixSort::SortPairs(nullptr, sort_tmp, (const int32_t*)nullptr, (int32_t*)nullptr,
                                           (const int32_t*)nullptr, (int32_t*)nullptr, (int)max_nnz, 0, key_bits(n));
  (void)hipcub::DeviceScan::ExclusiveSum(nullptr, scan_tmp, (const int32_t*)nullptr, (int64_t*)nullptr, (int)(n + 1));
  const size_t lib = sort_tmp > scan_tmp ? sort_tmp : scan_tmp;
  return align256((size_t)(n + 1) * sizeof(int32_t)) + 3 * align256((size_t)max_nnz * sizeof(int32_t)) + align256(lib);
}

// One slice: csr_col, row_of_entry, val (nnz entries in row-major order, nnz < 2^31) -> colptr_out (n + 1 offsets
// local to the slice), row_out, val_out.  tmp: build_csc_tmp_bytes(>= nnz, n) bytes.  Asynchronous on s.
hipError_t build_csc_slice(const int32_t* csr_col, const int32_t* row_of_entry, const float* val, int64_t nnz, int64_t n,
                           int64_t* colptr_out, int32_t* row_out, float* val_out, void* tmp, size_t tmp_bytes,
                           hipStream_t s) {
  char* base = (char*)tmp;
  int32_t* cnt = (int32_t*)base;
  base += align256((size_t)(n + 1) * sizeof(int32_t));
  int32_t* idx = (int32_t*)base;
  base += align256((size_t)nnz * sizeof(int32_t));
  int32_t* keys_out = (int32_t*)base;
  base += align256((size_t)nnz * sizeof(int32_t));
  int32_t* perm = (int32_t*)base;
  base += align256((size_t)nnz * sizeof(int32_t));
  if (base > (char*)tmp + tmp_bytes) return hipErrorInvalidValue;
  size_t lib_bytes = (size_t)((char*)tmp + tmp_bytes - base);
  hipError_t e = launch_fill_zero(cnt, (size_t)(n + 1) * sizeof(int32_t), s);
  if (e != hipSuccess) return e;
  if (nnz > 0) {
    int64_t blocks = ceil_div(nnz, 256);
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(csc_count_kernel, dim3((unsigned)blocks), dim3(256), 0, s, csr_col, nnz, cnt);
    hipLaunchKernelGGL(csc_iota_kernel, dim3((unsigned)blocks), dim3(256), 0, s, idx, nnz);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  size_t need = 0;
  e = hipcub::DeviceScan::ExclusiveSum(nullptr, need, cnt, colptr_out, (int)(n + 1), s);
  if (e != hipSuccess) return e;
  if (need > lib_bytes) return hipErrorInvalidValue;
  e = hipcub::DeviceScan::ExclusiveSum(base, need, cnt, colptr_out, (int)(n + 1), s);
  if (e != hipSuccess || nnz == 0) return e;
  e = hipcub::DeviceRadixSort::SortPairs(nullptr, need, csr_col, keys_out, idx, perm, (int)nnz, 0, key_bits(n), s);
  if (e != hipSuccess) return e;
  if (need > lib_bytes) return hipErrorInvalidValue;
  e = hipcub::DeviceRadixSort::SortPairs(base, need, csr_col, keys_out, idx, perm, (int)nnz, 0, key_bits(n), s);
  if (e != hipSuccess) return e;
  int64_t blocks = ceil_div(nnz, 256);
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(csc_gather_kernel, dim3((unsigned)blocks), dim3(256), 0, s, perm, row_of_entry, val, nnz, row_out,
                     val_out);
  return hipGetLastError();
}

}  // namespace nnr
