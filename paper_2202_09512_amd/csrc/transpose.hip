// The CSC copy of CSR slices, built on the device (section "Distributed RESCAL": the sparse tensor is stored slice
// by slice; X_t^T A wants the transposed view).  Without it X_t^T A has to scatter with atomics; with it both products
// are gathers.  A stable sort of the row-major entries by column gives columns ascending and rows ascending inside a
// column, so the copy (and every sum taken along it) is the same in every run.
//
// The sort is this library's own: a least-significant-digit radix sort of the entry numbers by column, 8 bits per
// pass.  A pass is three kernels: per-block digit histograms; per digit an exclusive scan over the blocks (one
// workgroup per digit: the table is digit-major, so a digit's counters are contiguous) that also leaves the digit's
// total; and a scatter in which ONE wavefront per block first turns the 256 totals into the digits' start positions,
// then walks its keys in order, 64 at a time, and ranks equal digits inside the 64 by their lane order (a ballot per
// digit bit), which keeps every pass stable.  One-time set-up, not the iteration: three passes over a slice's entries
// for up to 2^24 entities.
#include "common.h"
#include "kernels.h"

namespace nnr {

constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;
constexpr int kSortBlockKeys = 8192;   // keys per block of a pass (one wavefront scatters them: 128 steps of 64;
                                       // 2048 was measured: the same time, a four times larger table)

// table[digit * nblocks + block] = number of keys of the block with that digit
__global__ void __launch_bounds__(256) radix_hist_kernel(const int32_t* __restrict__ keys, int64_t count, int shift,
                                                         uint32_t* __restrict__ table, int64_t nblocks) {
  __shared__ uint32_t hist[kRadix];
  hist[threadIdx.x] = 0;
  __syncthreads();
  const int64_t lo = (int64_t)blockIdx.x * kSortBlockKeys;
  const int64_t hi = lo + kSortBlockKeys < count ? lo + kSortBlockKeys : count;
  for (int64_t p = lo + threadIdx.x; p < hi; p += 256) atomicAdd(&hist[((uint32_t)keys[p] >> shift) & (kRadix - 1)], 1u);
  __syncthreads();
  table[(int64_t)threadIdx.x * nblocks + blockIdx.x] = hist[threadIdx.x];
}

// Row `digit` of the table (one counter per block): exclusive prefix sums in place, the row's sum to totals[digit].
// One workgroup per digit, 256 counters per trip: a scan inside each wavefront, the four wavefronts' sums through LDS.
__global__ void __launch_bounds__(256) scan_rows_kernel(uint32_t* __restrict__ table, int64_t nblocks,
                                                        uint32_t* __restrict__ totals) {
  __shared__ uint32_t wsum[4];
  uint32_t* row = table + (int64_t)blockIdx.x * nblocks;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t carry = 0;                              // sum of the trips before this one
  for (int64_t base = 0; base < nblocks; base += 256) {
    const int64_t i = base + threadIdx.x;
    const uint32_t c = i < nblocks ? row[i] : 0u;
    uint32_t inc = c;                              // inclusive sum over the lanes up to this one
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t up = __shfl_up(inc, off);
      if (lane >= off) inc += up;
    }
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t s = wsum[w];
      if (w < wave) before += s;
      all += s;
    }
    if (i < nblocks) row[i] = carry + before + inc - c;
    carry += all;
    __syncthreads();                               // wsum is written again in the next trip
  }
  if (threadIdx.x == 0) totals[blockIdx.x] = carry;
}

// One wavefront per block: keys (and their payloads) go to their places in order.  vals_in == nullptr: the payload
// of key p is p itself (first pass).
__global__ void __launch_bounds__(64) radix_scatter_kernel(const int32_t* __restrict__ keys_in,
                                                           const int32_t* __restrict__ vals_in, int64_t count, int shift,
                                                           const uint32_t* __restrict__ table,
                                                           const uint32_t* __restrict__ totals, int64_t nblocks,
                                                           int32_t* __restrict__ keys_out, int32_t* __restrict__ vals_out) {
  __shared__ uint32_t next[kRadix];                // where the block's next key of each digit goes
  const int lane = threadIdx.x;
  {
    // a digit's keys start behind all keys of smaller digits; inside the digit, behind those of earlier blocks.
    // Lane l holds digits 4l .. 4l+3.
    uint32_t t[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) t[j] = totals[4 * lane + j];
    const uint32_t mine = t[0] + t[1] + t[2] + t[3];
    uint32_t inc = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t up = __shfl_up(inc, off);
      if (lane >= off) inc += up;
    }
    uint32_t start = inc - mine;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      next[4 * lane + j] = start + table[(int64_t)(4 * lane + j) * nblocks + blockIdx.x];
      start += t[j];
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  const int64_t lo = (int64_t)blockIdx.x * kSortBlockKeys;
  const int64_t hi = lo + kSortBlockKeys < count ? lo + kSortBlockKeys : count;
  const uint64_t below = lane == 0 ? 0ull : (~0ull >> (64 - lane));   // the lanes before this one
  for (int64_t base = lo; base < hi; base += 64) {
    const int64_t p = base + lane;
    const bool have = p < hi;
    const int32_t key = have ? keys_in[p] : 0;
    const int32_t val = have ? (vals_in ? vals_in[p] : (int32_t)p) : 0;
    const uint32_t d = ((uint32_t)key >> shift) & (kRadix - 1);
    // the lanes of this step that hold a key with the same digit
    uint64_t same = __ballot(have);
#pragma unroll
    for (int b = 0; b < kRadixBits; ++b) {
      const uint64_t set = __ballot(have && ((d >> b) & 1u));
      same &= ((d >> b) & 1u) ? set : ~set;
    }
    const uint32_t rank = (uint32_t)__popcll(same & below);
    uint32_t dst = 0;
    if (have) dst = next[d] + rank;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();               // every lane has read its digit's counter
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    if (have && rank == 0) next[d] += (uint32_t)__popcll(same);       // one lane per digit moves it on
    if (have) {
      keys_out[dst] = key;
      vals_out[dst] = val;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  }
}

// colptr[j] = number of sorted keys below j, j = 0 .. n (the sorted columns say where every column starts)
__global__ void __launch_bounds__(256) lower_bounds_kernel(const int32_t* __restrict__ sorted, int64_t count, int64_t n,
                                                           int64_t* __restrict__ colptr) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j > n) return;
  int64_t lo = 0, hi = count;                      // first position whose key is >= j
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (sorted[mid] < j) lo = mid + 1; else hi = mid;
  }
  colptr[j] = lo;
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

// bytes of scratch for one slice of at most max_nnz entries: two pairs of (keys, entry numbers) that the passes
// alternate between, the (digit, block) table and the digits' totals
size_t build_csc_tmp_bytes(int64_t max_nnz, int64_t n) {
  (void)n;
  const int64_t nblocks = ceil_div(max_nnz > 0 ? max_nnz : 1, kSortBlockKeys);
  return 4 * align256((size_t)(max_nnz > 0 ? max_nnz : 1) * sizeof(int32_t)) +
         align256((size_t)kRadix * nblocks * sizeof(uint32_t)) + align256((size_t)kRadix * sizeof(uint32_t));
}

// One slice: csr_col, row_of_entry, val (nnz entries in row-major order, nnz < 2^31; val may be NULL) -> colptr_out
// (n + 1 offsets local to the slice), row_out, val_out.  tmp: build_csc_tmp_bytes(>= nnz, n) bytes.  Asynchronous on s.
hipError_t build_csc_slice(const int32_t* csr_col, const int32_t* row_of_entry, const float* val, int64_t nnz, int64_t n,
                           int64_t* colptr_out, int32_t* row_out, float* val_out, void* tmp, size_t tmp_bytes,
                           hipStream_t s) {
  if (nnz == 0) return launch_fill_zero(colptr_out, (size_t)(n + 1) * sizeof(int64_t), s);
  if (tmp_bytes < build_csc_tmp_bytes(nnz, n)) return hipErrorInvalidValue;
  const size_t arr = align256((size_t)nnz * sizeof(int32_t));
  char* base = (char*)tmp;
  int32_t* keys[2] = {(int32_t*)base, (int32_t*)(base + arr)};
  int32_t* vals[2] = {(int32_t*)(base + 2 * arr), (int32_t*)(base + 3 * arr)};
  uint32_t* table = (uint32_t*)(base + 4 * arr);
  const int64_t nblocks = ceil_div(nnz, kSortBlockKeys);
  if (nblocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  uint32_t* totals = (uint32_t*)((char*)table + align256((size_t)kRadix * nblocks * sizeof(uint32_t)));
  const int passes = (key_bits(n) + kRadixBits - 1) / kRadixBits;
  const int32_t* kin = csr_col;
  const int32_t* vin = nullptr;                    // first pass: the entry numbers themselves
  for (int pass = 0; pass < passes; ++pass) {
    const int shift = pass * kRadixBits, o = pass & 1;
    hipLaunchKernelGGL(radix_hist_kernel, dim3((unsigned)nblocks), dim3(256), 0, s, kin, nnz, shift, table, nblocks);
    hipLaunchKernelGGL(scan_rows_kernel, dim3(kRadix), dim3(256), 0, s, table, nblocks, totals);
    hipLaunchKernelGGL(radix_scatter_kernel, dim3((unsigned)nblocks), dim3(64), 0, s, kin, vin, nnz, shift, table, totals,
                       nblocks, keys[o], vals[o]);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    kin = keys[o];
    vin = vals[o];
  }
  hipLaunchKernelGGL(lower_bounds_kernel, dim3((unsigned)ceil_div(n + 1, 256)), dim3(256), 0, s, kin, nnz, n, colptr_out);
  int64_t blocks = ceil_div(nnz, 256);
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(csc_gather_kernel, dim3((unsigned)blocks), dim3(256), 0, s, vin, row_of_entry, val, nnz, row_out,
                     val_out);
  return hipGetLastError();
}

}  // namespace nnr
