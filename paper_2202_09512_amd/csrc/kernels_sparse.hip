// Sparse pass over X (CSR, optionally CSC): X^r_t A^r and X^r_t^T A^r as sparse-times-dense products
// ("matrix_mul_sparse" in the paper's timing breakdown; Alg. 3 with X stored in CSR, section
// "Distributed RESCAL"), with the perturbation of Alg. 4 applied to the stored non-zeros only and keyed
// by coordinates, so CSR and CSC views of a slice see the same Delta.
//
// Load balance: the non-zeros of a slice are cut into equal chunks, one wavefront per chunk, whatever the
// row lengths (a row holding millions of non-zeros is spread over many wavefronts).  Inside a chunk the
// wavefront walks the non-zeros in order; its 64 lanes span the (member, column) pairs of one entity row
// of the factor, so a gather of A[j] is one coalesced read and the running sum needs no cross-lane
// reduction; the sum is written when the row changes (atomically for the chunk's first and last row,
// which other wavefronts may share).
#include "common.h"
#include "kernels.h"

namespace nnr {

// major index (row for CSR, column for CSC) of non-zero p: largest r with ptr[r] <= p
__device__ __forceinline__ int64_t find_major(const int64_t* __restrict__ ptr, int64_t n, int64_t p) {
  int64_t lo = 0, hi = n - 1;
  while (lo < hi) {
    const int64_t mid = (lo + hi + 1) >> 1;
    if (ptr[mid] <= p) lo = mid; else hi = mid - 1;
  }
  return lo;
}

__global__ void expand_major_kernel(const int64_t* __restrict__ ptr, int32_t* __restrict__ major, int64_t n,
                                    int64_t nnz) {
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += (int64_t)gridDim.x * blockDim.x)
    major[p] = (int32_t)find_major(ptr, n, p);
}

hipError_t launch_expand_major(const int64_t* ptr, int32_t* major, int64_t n, int64_t nnz, hipStream_t s) {
  if (nnz == 0) return hipSuccess;
  int64_t blocks = ceil_div(nnz, 256);
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(expand_major_kernel, dim3((unsigned)blocks), dim3(256), 0, s, ptr, major, n, nnz);
  return hipGetLastError();
}

constexpr int kChunk = 256;  // non-zeros per wavefront
constexpr int kGroup = 8;     // factor rows requested together, one group ahead of the sums

// VPL neighbouring columns per lane, moved as one piece
template <int VPL>
struct Vec {
  float v[VPL];
};
template <int VPL>
__device__ __forceinline__ Vec<VPL> vec_load(const float* p) {
  Vec<VPL> o;
  if constexpr (VPL == 4) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    o.v[0] = t.x; o.v[1] = t.y; o.v[2] = t.z; o.v[3] = t.w;
  } else if constexpr (VPL == 2) {
    const float2 t = *reinterpret_cast<const float2*>(p);
    o.v[0] = t.x; o.v[1] = t.y;
  } else {
    o.v[0] = p[0];
  }
  return o;
}
template <int VPL>
__device__ __forceinline__ void vec_store(float* p, const float (&a)[VPL]) {
  if constexpr (VPL == 4) *reinterpret_cast<float4*>(p) = float4{a[0], a[1], a[2], a[3]};
  else if constexpr (VPL == 2) *reinterpret_cast<float2*>(p) = float2{a[0], a[1]};
  else p[0] = a[0];
}

// the same store, marked as streaming (written once, not read again by this launch)
template <int VPL>
__device__ __forceinline__ void vec_store_streaming(float* p, const float (&a)[VPL]) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  typedef float f2 __attribute__((ext_vector_type(2)));
  if constexpr (VPL == 4) __builtin_nontemporal_store(f4{a[0], a[1], a[2], a[3]}, reinterpret_cast<f4*>(p));
  else if constexpr (VPL == 2) __builtin_nontemporal_store(f2{a[0], a[1]}, reinterpret_cast<f2*>(p));
  else __builtin_nontemporal_store(a[0], p);
}

// The 64 lanes of a wave span a slab of 64*VPL (member, column) pairs of an entity row; lane l owns the VPL
// neighbouring ones starting at VPL*l (q*kp is a multiple of 4, so a lane is inside the row or outside it).
// One launch covers a list of segments (one product of one slice each: the iteration passes all slices and both
// products at once); a workgroup finds its segment from the segments' first workgroup numbers.  nseg == 0: the one
// segment that comes by value.
template <int VPL>
__global__ void __launch_bounds__(256)
    spmm_gather_kernel(const GatherSeg* __restrict__ segs, int nseg, GatherSeg one, int64_t n,
                       const float* __restrict__ A_int, int q, int kp, uint32_t k0, uint32_t k1, float dscaled,
                       int perturb, float* __restrict__ side) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* xs = lds + (size_t)wave * 64 * q;        // per staged non-zero: its q perturbed values
  // Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous range of chunks, so that the
  // factor rows gathered by neighbouring rows of X (one community) meet in one L2.
  int64_t blk;
  {
    const int64_t total = gridDim.x, L = blockIdx.x;
    const int64_t base = total >> 3, rem = total & 7, xcd = L & 7, slot = L >> 3;
    blk = xcd * base + (xcd < rem ? xcd : rem) + slot;
  }
  const int64_t chunk_id = blk * 4 + wave;        // this wave's chunk, counted over the whole launch
  GatherSeg sg = one;
  if (nseg > 0) {                                 // largest s with segs[s].blk_first <= blk (uniform over the workgroup)
    int lo = 0, hi = nseg - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (segs[mid].blk_first <= blk) lo = mid; else hi = mid - 1;
    }
    sg = segs[lo];
    blk -= sg.blk_first;
  }
  const int32_t* __restrict__ major = sg.major;
  const int32_t* __restrict__ minor = sg.minor;
  const float* __restrict__ val = sg.val;         // NULL: a binary tensor, every stored entry is 1
  const int64_t nnz = sg.nnz;
  const int t = sg.t, transposed = sg.transposed;
  const int64_t start = (blk * 4 + wave) * kChunk;
  if (start >= nnz) return;
  const int64_t end = start + kChunk < nnz ? start + kChunk : nnz;
  const int qk = q * kp;
  const int c0 = blockIdx.y * 64 * VPL + VPL * lane;   // this lane's first (member, column) index
  const bool on = c0 < qk;
  const int cofs = on ? c0 : 0;                   // lanes beyond the row read its start and write nothing
  const int mem0 = cofs / kp;                     // a lane's VPL neighbouring values belong to one member (16 | kp)
  const float* __restrict__ Arow = A_int + cofs;  // this lane's columns of entity row 0
  float* __restrict__ orow = sg.out + cofs;
  // Everything that steers the walk is wave-uniform and kept in scalar registers: the row in progress, the rows at
  // the chunk's two ends, and (below) the row and column of every staged non-zero, which are broadcast from the
  // lane that loaded them with a lane read instead of a trip through LDS; the factor row's address is then scalar.
  const int32_t first_major = __builtin_amdgcn_readfirstlane(major[start]);
  const int32_t last_major = __builtin_amdgcn_readfirstlane(major[end - 1]);
  // a row is shared with a neighbouring chunk only if it continues across the chunk's border; such rows were
  // cleared beforehand and are added atomically, every other row is written exactly once
  const bool first_shared = start > 0 && __builtin_amdgcn_readfirstlane(major[start > 0 ? start - 1 : 0]) == first_major;
  const bool last_shared = end < nnz && __builtin_amdgcn_readfirstlane(major[end < nnz ? end : nnz - 1]) == last_major;
  float acc[VPL];
#pragma unroll
  for (int v = 0; v < VPL; ++v) acc[v] = 0.0f;
  int32_t cur = first_major;

  auto flush = [&](int32_t mj) {
    float* o = orow + (int64_t)mj * qk;
    const bool shared_row = (mj == first_major && first_shared) || (mj == last_major && last_shared);
    if (on) {
      if (shared_row && side) {
        // reproducible mode: the piece goes to the chunk's own place (slot 0: the row continues from the chunk
        // before, slot 1: it only goes on into the next one); gather_fixup_kernel sums the pieces in chunk order
        const int slot = (mj == first_major && first_shared) ? 0 : 1;
        vec_store<VPL>(side + (chunk_id * 2 + slot) * qk + cofs, acc);
      } else if (shared_row) {
#pragma unroll
        for (int v = 0; v < VPL; ++v) unsafeAtomicAdd(o + v, acc[v]);
      } else {
        vec_store<VPL>(o, acc);
      }
    }
#pragma unroll
    for (int v = 0; v < VPL; ++v) acc[v] = 0.0f;
  };

  for (int64_t pos = start; pos < end; pos += 64) {
    // stage 64 non-zeros: every lane loads its own one and perturbs it for all members
    const int64_t p = pos + lane;
    int32_t my_mj = 0, my_mn = 0;                  // (lanes past the end: never read, the sums stop at cnt)
    if (p < end) {
      my_mj = major[p];
      my_mn = minor[p];
      const float x = val ? val[p] : 1.0f;
      const uint64_t i = transposed ? (uint64_t)my_mn : (uint64_t)my_mj;
      const uint64_t j = transposed ? (uint64_t)my_mj : (uint64_t)my_mn;
      const uint64_t e = i * (uint64_t)n + j;
      for (int b = 0; b < (q + 7) / 8; ++b) {
        u32x4 w{0, 0, 0, 0};
        if (perturb) w = philox4x32_10((uint32_t)e, (uint32_t)(e >> 32), (uint32_t)t, (uint32_t)b, k0, k1);
        for (int r = 0; r < 8 && 8 * b + r < q; ++r)
          xs[lane * q + 8 * b + r] = perturb ? perturbed(x, w, r, dscaled) : x;
      }
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    const int cnt = (int)(end - pos < 64 ? end - pos : 64);
    if (cnt == 64) {
      // kGroup non-zeros at a time: their factor rows (and their values of this lane's member) are requested a whole
      // group ahead of the sums that use them
      Vec<VPL> abuf[2][kGroup];
      float xbuf[2][kGroup];
      auto request = [&](int g0, int b) {
#pragma unroll
        for (int w = 0; w < kGroup; ++w) {
          const int32_t mn = __builtin_amdgcn_readlane(my_mn, g0 + w);
          abuf[b][w] = vec_load<VPL>(Arow + (int64_t)mn * qk);
          xbuf[b][w] = xs[(g0 + w) * q + mem0];
        }
      };
      auto sums = [&](int g0, int b) {
#pragma unroll
        for (int w = 0; w < kGroup; ++w) {
          const int32_t mj = __builtin_amdgcn_readlane(my_mj, g0 + w);
          if (mj != cur) {                          // scalar compare
            flush(cur);
            cur = mj;
          }
#pragma unroll
          for (int v = 0; v < VPL; ++v) acc[v] = fmaf(xbuf[b][w], abuf[b][w].v[v], acc[v]);
        }
      };
      request(0, 0);
      // (a loop over pairs of groups, not unrolled further: the two buffers keep their names, the lane to read from
      // is a scalar register)
#pragma unroll 1
      for (int g0 = 0; g0 < 64; g0 += 2 * kGroup) {
        request(g0 + kGroup, 1);
        sums(g0, 0);
        if (g0 + 2 * kGroup < 64) request(g0 + 2 * kGroup, 0);
        sums(g0 + kGroup, 1);
      }
    } else {
      // the last, partial stage of a segment: one non-zero at a time
      for (int u = 0; u < cnt; ++u) {
        const int32_t mj = __builtin_amdgcn_readlane(my_mj, u);
        const int32_t mn = __builtin_amdgcn_readlane(my_mn, u);
        const Vec<VPL> a = vec_load<VPL>(Arow + (int64_t)mn * qk);
        const float x = xs[u * q + mem0];
        if (mj != cur) {
          flush(cur);
          cur = mj;
        }
#pragma unroll
        for (int v = 0; v < VPL; ++v) acc[v] = fmaf(x, a.v[v], acc[v]);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  flush(cur);
}

// ---- The same products, one 128-byte line of every factor row per pass over the non-zeros ("lines" form) ----------
// The gathers of the kernel above miss the L2s because the factor rows that a community of entities refers to
// (q * kp * 4 bytes each) are together several times an L2.  Here a pass (blockIdx.y: the hardware hands out all
// workgroups of a pass before those of the next) takes only 32 neighbouring columns, one cache line, of every row,
// so the lines that a pass wants are q * kp / 32 times fewer bytes, at the price of walking the coordinates (and
// drawing the perturbation of the members that own those columns) once per pass.
// A gather instruction fetches G = 64 / L such lines: the wave's chunk of 256 non-zeros is staged in LDS (row, column,
// perturbed values) and cut into G equal sub-chunks; group g of L lanes walks sub-chunk g, each lane with VPL = 32 / L
// neighbouring columns.  A row that lies inside a sub-chunk is stored by its group.  The first and the last row of
// every sub-chunk may go on in the neighbouring one: their sums go to LDS, and at the end the wave adds up what
// belongs to one row and writes it: atomically only where the row goes on in another wave's chunk, as above.
template <int L>
__global__ void __launch_bounds__(256)
    spmm_gather_lines_kernel(const GatherSeg* __restrict__ segs, int nseg, GatherSeg one, int64_t n,
                             const float* __restrict__ A_int, int q, int kp, uint32_t k0, uint32_t k1, float dscaled,
                             int perturb, float* __restrict__ side) {
  constexpr int G = 64 / L, VPL = 32 / L, PER = kChunk / G;
  __shared__ int32_t s_major[4][kChunk];
  __shared__ int32_t s_minor[4][kChunk];
  __shared__ float s_x[4][kChunk][2];              // perturbed value for the (at most two) members that share the line
  __shared__ float s_piece[4][2 * G][32];          // per group: the sum of its first row and of its last row
  __shared__ int32_t s_prow[4][2 * G];             // the rows they belong to (-1: none)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int64_t blk;
  {
    const int64_t total = gridDim.x, Lb = blockIdx.x;
    const int64_t base = total >> 3, rem = total & 7, xcd = Lb & 7, slot = Lb >> 3;
    blk = xcd * base + (xcd < rem ? xcd : rem) + slot;
  }
  const int64_t chunk_id = blk * 4 + wave;         // this wave's chunk, counted over the whole launch
  GatherSeg sg = one;
  if (nseg > 0) {
    int lo = 0, hi = nseg - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (segs[mid].blk_first <= blk) lo = mid; else hi = mid - 1;
    }
    sg = segs[lo];
    blk -= sg.blk_first;
  }
  const int32_t* __restrict__ major = sg.major;
  const int32_t* __restrict__ minor = sg.minor;
  const float* __restrict__ val = sg.val;
  const int64_t nnz = sg.nnz;
  const int64_t start = (blk * 4 + wave) * kChunk;
  if (start >= nnz) return;
  const int64_t end = start + kChunk < nnz ? start + kChunk : nnz;
  const int cnt = (int)(end - start);
  const int qk = q * kp;
  const int coff = blockIdx.y * 32;                // first column of this pass's line
  const int mfirst = coff / kp;                    // the member that owns it; 16 | kp: at most one more shares the line
  const bool two = (coff + 31) / kp != mfirst && mfirst + 1 < q;
  const bool first_shared = start > 0 && major[start - 1] == major[start];
  const bool last_shared = end < nnz && major[end < nnz ? end : nnz - 1] == major[end - 1];

  // ---- stage the chunk: every lane four of its non-zeros
#pragma unroll
  for (int j = 0; j < kChunk / 64; ++j) {
    const int i = lane + 64 * j;
    if (i < cnt) {
      const int64_t p = start + i;
      // (read once per pass: marked as streaming, so that they do not push the factor lines out of the L2)
      const int32_t mj = __builtin_nontemporal_load(major + p), mn = __builtin_nontemporal_load(minor + p);
      const float x = val ? __builtin_nontemporal_load(val + p) : 1.0f;
      float x0 = x, x1 = x;
      if (perturb) {
        const uint64_t row = sg.transposed ? (uint64_t)mn : (uint64_t)mj;
        const uint64_t col = sg.transposed ? (uint64_t)mj : (uint64_t)mn;
        const uint64_t e = row * (uint64_t)n + col;
        u32x4 w = philox4x32_10((uint32_t)e, (uint32_t)(e >> 32), (uint32_t)sg.t, (uint32_t)(mfirst >> 3), k0, k1);
        x0 = perturbed(x, w, mfirst & 7, dscaled);
        if (two) {
          const int r1 = mfirst + 1;
          if ((r1 >> 3) != (mfirst >> 3))
            w = philox4x32_10((uint32_t)e, (uint32_t)(e >> 32), (uint32_t)sg.t, (uint32_t)(r1 >> 3), k0, k1);
          x1 = perturbed(x, w, r1 & 7, dscaled);
        }
      }
      s_major[wave][i] = mj;
      s_minor[wave][i] = mn;
      s_x[wave][i][0] = x0;
      s_x[wave][i][1] = x1;
    }
  }
  const int g = lane / L, gl = lane % L;
  if (gl == 0) {
    s_prow[wave][2 * g] = -1;
    s_prow[wave][2 * g + 1] = -1;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

  // ---- walk: group g over its sub-chunk
  const int c = coff + gl * VPL;                   // this lane's first column
  const bool on = c < qk;                          // (a last line may be half empty: q * kp is a multiple of 16)
  const int cofs = on ? c : 0;
  const int xslot = on ? c / kp - mfirst : 0;      // 0 or 1: which of the line's members this lane belongs to
  const float* __restrict__ Arow = A_int + cofs;
  float* __restrict__ orow = sg.out + cofs;
  const int s0 = g * PER;
  const int s1 = s0 + PER < cnt ? s0 + PER : cnt;  // (empty for groups beyond a short chunk's end)
  float acc[VPL];
#pragma unroll
  for (int v = 0; v < VPL; ++v) acc[v] = 0.0f;
  int32_t cur = s0 < s1 ? s_major[wave][s0] : -1;
  bool first = true;                               // no row of this group has been closed yet

  auto put_piece = [&](int idx) {
    if (gl == 0) s_prow[wave][idx] = cur;
#pragma unroll
    for (int v = 0; v < VPL; ++v) s_piece[wave][idx][gl * VPL + v] = acc[v];
  };
  auto close_row = [&]() {                         // the non-zeros of row `cur` inside this sub-chunk are summed
    if (first) {
      put_piece(2 * g);
      first = false;
    } else if (on) {
      vec_store_streaming<VPL>(orow + (int64_t)cur * qk, acc);
    }
#pragma unroll
    for (int v = 0; v < VPL; ++v) acc[v] = 0.0f;
  };

  if (cnt == kChunk) {
    // full chunk: every group makes PER steps; kGroup lines are requested together
#pragma unroll 1
    for (int b = s0; b < s0 + PER; b += kGroup) {
      Vec<VPL> a[kGroup];
      float x[kGroup];
      int32_t mjs[kGroup];
#pragma unroll
      for (int w = 0; w < kGroup; ++w) {
        const int32_t mn = s_minor[wave][b + w];
        a[w] = vec_load<VPL>(Arow + (int64_t)mn * qk);
        x[w] = s_x[wave][b + w][xslot];
        mjs[w] = s_major[wave][b + w];
      }
#pragma unroll
      for (int w = 0; w < kGroup; ++w) {
        if (mjs[w] != cur) {
          close_row();
          cur = mjs[w];
        }
#pragma unroll
        for (int v = 0; v < VPL; ++v) acc[v] = fmaf(x[w], a[w].v[v], acc[v]);
      }
    }
  } else {
    for (int b = s0; b < s1; ++b) {
      const int32_t mn = s_minor[wave][b], mj = s_major[wave][b];
      const Vec<VPL> a = vec_load<VPL>(Arow + (int64_t)mn * qk);
      const float x = s_x[wave][b][xslot];
      if (mj != cur) {
        close_row();
        cur = mj;
      }
#pragma unroll
      for (int v = 0; v < VPL; ++v) acc[v] = fmaf(x, a.v[v], acc[v]);
    }
  }
  if (s0 < s1) put_piece(first ? 2 * g : 2 * g + 1);   // the group's last row (which may also be its first)
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

  // ---- the pieces in the order of the non-zeros; neighbours of one row are added; lanes 0..31 hold a column each
  {
    const int cc = coff + (lane & 31);
    const bool on2 = lane < 32 && cc < qk;
    float* __restrict__ ocol = sg.out + (on2 ? cc : 0);
    int32_t run_row = -1;
    float run = 0.0f;
    bool at_start = true;                          // the run in progress holds the chunk's first non-zero
    auto emit = [&](bool shared_row, int slot) {
      if (on2) {
        float* o = ocol + (int64_t)run_row * qk;
        // reproducible mode: the piece goes to the chunk's own place (slot 0: the row continues from the chunk before,
        // slot 1: it only goes on into the next one), as in the kernel above; gather_fixup_kernel sums them in order
        if (shared_row && side) side[(chunk_id * 2 + slot) * qk + cc] = run;
        else if (shared_row) unsafeAtomicAdd(o, run);
        else __builtin_nontemporal_store(run, o);
      }
    };
    for (int pidx = 0; pidx < 2 * G; ++pidx) {
      const int32_t row = __builtin_amdgcn_readfirstlane(s_prow[wave][pidx]);
      if (row < 0) continue;
      const float v = s_piece[wave][pidx][lane & 31];
      if (row == run_row) {
        run += v;
      } else {
        if (run_row >= 0) {
          emit(at_start && first_shared, 0);
          at_start = false;
        }
        run_row = row;
        run = v;
      }
    }
    // this run holds the chunk's last non-zero
    if (run_row >= 0) emit((at_start && first_shared) || last_shared, at_start && first_shared ? 0 : 1);
  }
}

// Rows of the output that the gather kernel does not write exactly once: rows without non-zeros (cleared here,
// never touched again) and rows whose non-zeros cross a chunk border (cleared here, then added atomically).
// blockIdx.y: the segment.
__global__ void __launch_bounds__(256) clear_rows_kernel(const GatherSeg* __restrict__ segs, GatherSeg one, int64_t n,
                                                         int qk, int clear_empty) {
  const GatherSeg sg = segs ? segs[blockIdx.y] : one;
  const int64_t* __restrict__ ptr = sg.ptr;
  float* __restrict__ out = sg.out;
  const int lane = threadIdx.x & 63;
  const int64_t i = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 64 + lane;
  bool flag = false;
  if (i < n) {
    const int64_t a = ptr[i], b = ptr[i + 1];
    flag = a == b ? clear_empty != 0 : (a / kChunk != (b - 1) / kChunk);
  }
  uint64_t mask = __ballot(flag);
  while (mask) {
    const int src = __builtin_ctzll(mask);
    mask &= mask - 1;
    float* o = out + (i - lane + src) * qk;
    for (int c = lane; c < qk; c += 64) o[c] = 0.0f;
  }
}

// bit i % 32 of word i / 32: entity row (column) i of the slice holds a stored non-zero
__global__ void __launch_bounds__(256) presence_mask_kernel(const int64_t* __restrict__ ptr, uint32_t* __restrict__ mask,
                                                            int64_t n, int64_t nwords) {
  const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (w >= nwords) return;
  uint32_t bits = 0;
  for (int b = 0; b < 32; ++b) {
    const int64_t i = w * 32 + b;
    if (i < n && ptr[i + 1] > ptr[i]) bits |= 1u << b;
  }
  mask[w] = bits;
}

// *count += number of set bits of the mask words (unsigned long long on the device)
__global__ void __launch_bounds__(256) popcount_kernel(const uint32_t* __restrict__ mask, int64_t nwords,
                                                       unsigned long long* __restrict__ count) {
  unsigned long long c = 0;
  for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < nwords; w += (int64_t)gridDim.x * blockDim.x)
    c += __popc(mask[w]);
  for (int off = 32; off > 0; off >>= 1) c += __shfl_down(c, off, 64);
  if ((threadIdx.x & 63) == 0 && c) atomicAdd(count, c);
}

hipError_t launch_popcount(const uint32_t* mask, int64_t nwords, unsigned long long* count, hipStream_t s) {
  int64_t blocks = ceil_div(nwords, 256 * 8);
  if (blocks < 1) blocks = 1;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(popcount_kernel, dim3((unsigned)blocks), dim3(256), 0, s, mask, nwords, count);
  return hipGetLastError();
}

hipError_t launch_presence_mask(const int64_t* ptr, uint32_t* mask, int64_t n, hipStream_t s) {
  const int64_t nwords = ceil_div(n, 32);
  hipLaunchKernelGGL(presence_mask_kernel, dim3((unsigned)ceil_div(nwords, 256)), dim3(256), 0, s, ptr, mask, n, nwords);
  return hipGetLastError();
}

static int vpl_for(int qk) { return qk <= 64 ? 1 : (qk <= 128 ? 2 : 4); }

int64_t spmm_gather_blocks(int64_t nnz) { return ceil_div(ceil_div(nnz, kChunk), 4); }

// Reproducible mode: one wavefront per chunk.  The chunk in which a row that crosses chunk borders STARTS sums that
// row's pieces (its own slot 1, then slot 0 of the chunks that follow, as long as the row goes on) in chunk order and
// stores the row.  Same walk over the segments as the gather kernel (no XCD remapping: the order does not matter).
__global__ void __launch_bounds__(256) gather_fixup_kernel(const GatherSeg* __restrict__ segs, int nseg, GatherSeg one,
                                                           int qk, const float* __restrict__ side) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int64_t blk = blockIdx.x;
  const int64_t chunk_id = blk * 4 + wave;
  GatherSeg sg = one;
  if (nseg > 0) {
    int lo = 0, hi = nseg - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (segs[mid].blk_first <= blk) lo = mid; else hi = mid - 1;
    }
    sg = segs[lo];
    blk -= sg.blk_first;
  }
  const int32_t* __restrict__ major = sg.major;
  const int64_t nnz = sg.nnz;
  const int64_t start = (blk * 4 + wave) * kChunk;
  if (start >= nnz) return;
  const int64_t end = start + kChunk < nnz ? start + kChunk : nnz;
  const int32_t first_major = major[start], row = major[end - 1];
  const bool first_shared = start > 0 && major[start - 1] == first_major;
  const bool last_shared = end < nnz && major[end] == row;
  // the row starts in this chunk: it goes on behind it, and has not come in from the chunk before
  if (!last_shared || (first_shared && first_major == row)) return;
  for (int c0 = 0; c0 < qk; c0 += 64) {
    const int c = c0 + lane;
    float sum = c < qk ? side[(chunk_id * 2 + 1) * qk + c] : 0.0f;
    int64_t ch = chunk_id + 1, s2 = end;          // the chunks that follow, in order
    while (true) {
      const int64_t e2 = s2 + kChunk < nnz ? s2 + kChunk : nnz;
      if (c < qk) sum += side[(ch * 2 + 0) * qk + c];
      const bool goes_on = major[e2 - 1] == row && e2 < nnz && major[e2] == row;   // uniform over the wave
      if (!goes_on) break;
      ++ch;
      s2 = e2;
    }
    if (c < qk) sg.out[(int64_t)row * qk + c] = sum;
  }
}

template <int VPL>
static void gather_launch(const GatherSeg* segs, int nseg, const GatherSeg& one, int64_t blocks, const float* A_int,
                          const Dims& d, uint64_t seed, float delta, hipStream_t s, float* side) {
  const int qk = d.q * d.kp;
  dim3 grid((unsigned)blocks, (unsigned)ceil_div(qk, 64 * VPL));
  const size_t lds = (size_t)4 * 64 * d.q * sizeof(float);
  hipLaunchKernelGGL(spmm_gather_kernel<VPL>, grid, dim3(256), lds, s, segs, nseg, one, d.n, A_int, d.q, d.kp,
                     (uint32_t)seed, (uint32_t)(seed >> 32), delta * 0x1p-16f, delta != 0.0f ? 1 : 0, side);
}

// lanes per line in the lines form (8 lanes of four columns: eight lines per gather instruction)
constexpr int kLineLanes = 8;

bool spmm_gather_form_ok(int form, const Dims& d) {
  const int qk = d.q * d.kp;
  switch (form) {
    case kGatherRows: return true;
    case kGatherLines: return qk > 32;                       // more than one line per row
    default: return false;
  }
}

// segs (device, nseg > 0 entries with blk_first filled in, total_blocks workgroups in all) or, with nseg == 0, `one`
static hipError_t gather_any(const GatherSeg* segs, int nseg, const GatherSeg& one, int64_t total_blocks,
                             const float* A_int, const Dims& d, int clear_empty, uint64_t seed, float delta,
                             hipStream_t s, float* side, int form) {
  const int qk = d.q * d.kp;
  if (total_blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  if (!spmm_gather_form_ok(form, d)) form = kGatherRows;
  hipLaunchKernelGGL(clear_rows_kernel, dim3((unsigned)ceil_div(d.n, 256), (unsigned)(nseg > 0 ? nseg : 1)), dim3(256), 0, s,
                     nseg > 0 ? segs : nullptr, one, d.n, qk, clear_empty);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || total_blocks == 0) return e;
  if (form == kGatherLines) {
    hipLaunchKernelGGL(spmm_gather_lines_kernel<kLineLanes>, dim3((unsigned)total_blocks, (unsigned)ceil_div(qk, 32)), dim3(256), 0,
                       s, segs, nseg, one, d.n, A_int, d.q, d.kp, (uint32_t)seed, (uint32_t)(seed >> 32), delta * 0x1p-16f,
                       delta != 0.0f ? 1 : 0, side);
    e = hipGetLastError();
    if (e == hipSuccess && side)
      hipLaunchKernelGGL(gather_fixup_kernel, dim3((unsigned)total_blocks), dim3(256), 0, s, nseg > 0 ? segs : nullptr, nseg,
                         one, qk, side);
    return e == hipSuccess ? hipGetLastError() : e;
  }
  switch (vpl_for(qk)) {
    case 1: gather_launch<1>(segs, nseg, one, total_blocks, A_int, d, seed, delta, s, side); break;
    case 2: gather_launch<2>(segs, nseg, one, total_blocks, A_int, d, seed, delta, s, side); break;
    default: gather_launch<4>(segs, nseg, one, total_blocks, A_int, d, seed, delta, s, side); break;
  }
  e = hipGetLastError();
  if (e == hipSuccess && side)
    hipLaunchKernelGGL(gather_fixup_kernel, dim3((unsigned)total_blocks), dim3(256), 0, s, nseg > 0 ? segs : nullptr, nseg, one,
                       qk, side);
  return e == hipSuccess ? hipGetLastError() : e;
}

hipError_t launch_spmm_gather(const int64_t* ptr, const int32_t* major, const int32_t* minor, const float* val,
                              int64_t nnz, const float* A_int, float* out, const Dims& d, int t, int transposed,
                              int clear_empty, uint64_t seed, float delta, hipStream_t s, float* side, int form) {
  GatherSeg one{ptr, major, minor, val, out, nnz, 0, t, transposed};
  return gather_any(nullptr, 0, one, spmm_gather_blocks(nnz), A_int, d, clear_empty, seed, delta, s, side, form);
}

hipError_t launch_spmm_gather_batched(const GatherSeg* segs_dev, int nseg, int64_t total_blocks, const float* A_int,
                                      const Dims& d, int clear_empty, uint64_t seed, float delta, hipStream_t s,
                                      float* side, int form) {
  if (nseg <= 0) return hipSuccess;
  return gather_any(segs_dev, nseg, GatherSeg{}, total_blocks, A_int, d, clear_empty, seed, delta, s, side, form);
}

// CSR stream, scatter form: out[col][r][:] += x^r * A[row][r][:].  Only used when no CSC copy was given.
__global__ void __launch_bounds__(256)
    spmm_scatter_kernel(const int32_t* __restrict__ major, const int32_t* __restrict__ minor,
                        const float* __restrict__ val, int64_t nnz, int64_t n, const float* __restrict__ A_int,
                        float* __restrict__ out, int q, int kp, int t, uint32_t k0, uint32_t k1, float dscaled,
                        int perturb) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int qk = q * kp;
  const int64_t start = ((int64_t)blockIdx.x * 4 + wave) * kChunk;
  const int64_t end = start + kChunk < nnz ? start + kChunk : nnz;
  for (int64_t p = start; p < end; ++p) {
    const int32_t mj = major[p], mn = minor[p];
    const float x = val ? val[p] : 1.0f;
    const uint64_t e = (uint64_t)mj * (uint64_t)n + (uint64_t)mn;
    for (int c = lane; c < qk; c += 64) {
      const int r = c / kp;
      float xq = x;
      if (perturb) {
        const u32x4 w = philox4x32_10((uint32_t)e, (uint32_t)(e >> 32), (uint32_t)t, (uint32_t)(r >> 3), k0, k1);
        xq = perturbed(xq, w, r & 7, dscaled);
      }
      const float a = A_int[(int64_t)mj * qk + c];
      if (a != 0.0f) unsafeAtomicAdd(&out[(int64_t)mn * qk + c], xq * a);
    }
  }
}

hipError_t launch_spmm_scatter(const int32_t* major, const int32_t* minor, const float* val, int64_t nnz,
                               const float* A_int, float* out, const Dims& d, int t, uint64_t seed, float delta,
                               hipStream_t s) {
  const int qk = d.q * d.kp;
  hipError_t e = launch_fill_zero(out, (size_t)d.n * qk * sizeof(float), s);
  if (e != hipSuccess || nnz == 0) return e;
  const int64_t waves = ceil_div(nnz, kChunk);
  hipLaunchKernelGGL(spmm_scatter_kernel, dim3((unsigned)ceil_div(waves, 4)), dim3(256), 0, s, major, minor, val, nnz,
                     d.n, A_int, out, d.q, d.kp, t, (uint32_t)seed, (uint32_t)(seed >> 32), delta * 0x1p-16f,
                     delta != 0.0f ? 1 : 0);
  return hipGetLastError();
}

// Alg. 4 on the stored non-zeros of one slice (zeros are never touched: the pattern is preserved)
__global__ void sparse_perturb_kernel(const int64_t* __restrict__ ptr, const int32_t* __restrict__ idx,
                                      const float* __restrict__ val, int64_t nnz, float* __restrict__ out, int64_t n,
                                      int t, int transposed, int member, uint32_t k0, uint32_t k1, float dscaled,
                                      int perturb) {
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += (int64_t)gridDim.x * blockDim.x) {
    float v = val ? val[p] : 1.0f;
    if (perturb) {
      const uint64_t mj = (uint64_t)find_major(ptr, n, p), mn = (uint64_t)idx[p];
      const uint64_t e = transposed ? mn * (uint64_t)n + mj : mj * (uint64_t)n + mn;
      const u32x4 w = philox4x32_10((uint32_t)e, (uint32_t)(e >> 32), (uint32_t)t, (uint32_t)(member >> 3), k0, k1);
      v = perturbed(v, w, member & 7, dscaled);
    }
    out[p] = v;
  }
}

hipError_t launch_sparse_perturb(const int64_t* ptr, const int32_t* idx, const float* val, int64_t nnz, float* out,
                                 int64_t n, int t, int transposed, int member, uint64_t seed, float delta,
                                 hipStream_t s) {
  if (nnz == 0) return hipSuccess;
  int64_t blocks = ceil_div(nnz, 256);
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(sparse_perturb_kernel, dim3((unsigned)blocks), dim3(256), 0, s, ptr, idx, val, nnz, out, n, t,
                     transposed, member, (uint32_t)seed, (uint32_t)(seed >> 32), delta * 0x1p-16f,
                     delta != 0.0f ? 1 : 0);
  return hipGetLastError();
}

__global__ void __launch_bounds__(256)
    sparse_xnorm_kernel(const int32_t* __restrict__ major, const int32_t* __restrict__ minor,
                        const float* __restrict__ val, int64_t nnz, double* __restrict__ xn, int64_t n, int t, int q,
                        uint32_t k0, uint32_t k1, float dscaled, int perturb, double* __restrict__ part) {
  __shared__ double red[4];
  for (int b = 0; b < (q + 7) / 8; ++b) {
    double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int qb = (q - 8 * b) < 8 ? (q - 8 * b) : 8;
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += (int64_t)gridDim.x * blockDim.x) {
      const float v = val ? val[p] : 1.0f;
      const uint64_t e = (uint64_t)major[p] * (uint64_t)n + (uint64_t)minor[p];
      u32x4 w{0, 0, 0, 0};
      if (perturb) w = philox4x32_10((uint32_t)e, (uint32_t)(e >> 32), (uint32_t)t, (uint32_t)b, k0, k1);
#pragma unroll
      for (int qq = 0; qq < 8; ++qq)
        if (qq < qb) {
          const float xq = perturb ? perturbed(v, w, qq, dscaled) : v;
          acc[qq] += (double)xq * (double)xq;
        }
    }
#pragma unroll
    for (int qq = 0; qq < 8; ++qq) {
      if (qq < qb) {
        double v = acc[qq];
        for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
        __syncthreads();
        if (threadIdx.x == 0) {
          const double sum = red[0] + red[1] + red[2] + red[3];
          if (part) part[(int64_t)blockIdx.x * q + 8 * b + qq] = sum;   // reproducible mode: added in block order later
          else atomicAdd(&xn[8 * b + qq], sum);
        }
      }
    }
  }
}

hipError_t launch_sparse_xnorm(const int32_t* major, const int32_t* minor, const float* val, int64_t nnz, double* xn,
                               int64_t n, int t, int q, uint64_t seed, float delta, hipStream_t s, double* part) {
  if (nnz == 0) return hipSuccess;
  int64_t blocks = ceil_div(nnz, 256 * 8);
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(sparse_xnorm_kernel, dim3((unsigned)blocks), dim3(256), 0, s, major, minor, val, nnz, xn, n, t, q,
                     (uint32_t)seed, (uint32_t)(seed >> 32), delta * 0x1p-16f, delta != 0.0f ? 1 : 0, part);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && part) e = launch_reduce_parts_f64(xn, part, q, blocks, q, 1, s);
  return e;
}

}  // namespace nnr
