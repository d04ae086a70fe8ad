// Dense pass over X: for every slice t and ensemble member r, in ONE read of X_t,
//   P = X^r_t A^r   (Alg. 3: XA)      and      Q = X^r_t^T A^r   (Alg. 3: XTAR before the R_t factor),
// with X^r = X (*) Delta^r generated on the fly (Alg. 4) from a counter-based random stream, so the
// perturbed tensors are never stored and X is read once for all members of a group.
//
// Mapping to CDNA4.  The contraction runs on fp32 matrix cores, v_mfma_f32_16x16x4f32
// (D[16x16] += A[16x4] B[4x16]; lane l supplies A[l%16][l/16] and B[l/16][l%16], and holds
// D[4*(l/16)+r][l%16] in register r).  The perturbed X tile is the MFMA's left operand, built in
// registers by the lane that loaded the element; rows of the factor are the right operand, read from a
// copy of A that is stored in operand order (one 16-byte load per lane and product group).
//
// A workgroup of 8 waves owns a panel of 128 columns (8 tiles) and a chunk of rows.  In a round, every wave
// takes one 16-row strip and walks it across the panel, tile by tile:
//   - the strip's P accumulators and the right operands of the Q products (the strip's 16 factor rows) stay
//     in registers for the whole strip; P is added to memory once per strip;
//   - the tile is parked in LDS and read back transposed for the Q product, so the generator runs once per
//     element;
//   - the panel's Q accumulators live in LDS in accumulator order.  In step s wave w works on tile
//     (w + s) % 8, so at any time each tile column has one owner, which loads the accumulators as the MFMA's
//     C operand and stores the result back: no atomics and no cross-wave reduction.  A column passes from
//     wave w + 1 to wave w; every wave counts its completed steps in LDS and waits only for that neighbour,
//     before the Q half of its step (no barrier per step).  Q is added to memory once per workgroup.
// On gfx950 fp32 MFMA and ordinary vector instructions use the same ALUs and do not overlap (measured), so
// the floor of a tile is its MFMA time plus the generator's and the conversions' vector time.
// One Philox block yields eight 16-bit draws, one per member of the group, so the generator's integer
// work is shared by up to 8 members.
#include "common.h"
#include "kernels.h"

namespace nnr {

// Issue priority of a wave by the phase of its step (s_setprio; it only orders the waves of a SIMD, not streams):
// lowest in the long vector-only generator phase, higher once the matrix products start, highest from the tile
// transposition to the end of the step.  The wave that is nearer to handing its tile column on goes first; measured
// against equal priorities: 59.4 -> 52.9 ms per launch on the 16384-entity workload.  Only the order matters
// (generator < P products < rest); with the P products at or above the rest the gain is half, at the generator's
// level it is gone.
constexpr int kPrioGenerator = 0, kPrioPProducts = 1, kPrioRest = 2;


typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 8;     // two waves per SIMD
constexpr int kPanel = 128;   // columns per workgroup
constexpr int kTiles = kPanel / 16;
constexpr int kTLD = 20;      // row pitch (floats) of a 16 x 16 transposition tile in LDS: conflict-free reads

// Operand-order copy of the factor: A_op[entity / 16][member][column block][lane][r] =
//   A_int[16 * (entity / 16) + 4 * (lane / 16) + r][member][16 * block + lane % 16]
// so that the right MFMA operand of a 16-entity tile, for the four sub-steps r of a product, is one float4 per lane.
// Rows at or beyond n_rows (the source may end there) read as zero.
__global__ void pack_operand_kernel(const float* __restrict__ A_int, float* __restrict__ A_op, int64_t n_pad, int q,
                                    int kp, int64_t n_rows) {
  const int nt = kp / 16;
  const int64_t total = n_pad * q * kp / 4;   // float4 elements
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int lane = (int)(idx & 63);
    int64_t rest = idx >> 6;
    const int b = (int)(rest % nt);
    rest /= nt;
    const int mem = (int)(rest % q);
    const int64_t tile = rest / q;
    const int64_t i = tile * 16 + 4 * (lane >> 4);
    const int64_t rs = (int64_t)q * kp;
    const float* src = A_int + (i * q + mem) * kp + b * 16 + (lane & 15);
    float4 v;
    v.x = i + 0 < n_rows ? src[0] : 0.0f;
    v.y = i + 1 < n_rows ? src[rs] : 0.0f;
    v.z = i + 2 < n_rows ? src[2 * rs] : 0.0f;
    v.w = i + 3 < n_rows ? src[3 * rs] : 0.0f;
    reinterpret_cast<float4*>(A_op)[idx] = v;
  }
}

hipError_t launch_pack_operand(const float* A_int, float* A_op, const Dims& d, hipStream_t s, int64_t n_rows) {
  const int64_t total = d.n_pad * d.q * d.kp / 4;
  int64_t blocks = ceil_div(total, 256);
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(pack_operand_kernel, dim3((unsigned)blocks), dim3(256), 0, s, A_int, A_op, d.n_pad, d.q, d.kp,
                     n_rows < 0 ? d.n_pad : n_rows);
  return hipGetLastError();
}

// Load the "row" orientation of one 16 x 16 tile: lane (l16, row) gets X[i0 + l16][j0 + 4*row + r], r = 0..3.
// full: the tile lies inside the chunk and the matrix, rows are 16-byte aligned (one vector load, no mask).
__device__ __forceinline__ float4 load_tile(const float* __restrict__ xtile, bool full, int n32, int rows_left,
                                            int cols_left, int l16, int row) {
  if (full) return *reinterpret_cast<const float4*>(xtile + (l16 * n32 + 4 * row));
  // clamp the address into the valid part of the tile, then mask: no divergent branches
  const int ic = l16 < rows_left ? l16 : rows_left - 1;
  const bool rok = l16 < rows_left;
  float x[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int j = 4 * row + r;
    const int jc = j < cols_left ? j : cols_left - 1;
    const float v = xtile[ic * n32 + jc];
    x[r] = (rok && j < cols_left) ? v : 0.0f;
  }
  return float4{x[0], x[1], x[2], x[3]};
}

// The 16-bit halves [hoff, hoff + QB) of a Philox block moved to its front, so that the members of a group index the
// block with compile-time constants (hoff is wave-uniform and a multiple of QB; QB divides 8).
template <int QB>
__device__ __forceinline__ u32x4 front_halves(u32x4 w, int hoff) {
  if constexpr (QB == 4) {
    const bool hi = (hoff & 4) != 0;
    w.x = hi ? w.z : w.x;
    w.y = hi ? w.w : w.y;
  } else if constexpr (QB < 4) {
    const uint32_t a = (hoff & 2) ? w.y : w.x, b = (hoff & 2) ? w.w : w.z;
    w.x = (hoff & 4) ? b : a;
    if constexpr (QB == 1) w.x >>= 16 * (hoff & 1);
  }
  return w;
}

// Dynamic LDS layout (floats):
//   [0, kTiles*NG*256)          panel-wide Q accumulator in MFMA accumulator order: qlds[tile][group][lane][4]
//   then per wave QB*16*kTLD    transposition tiles of the members of the group
//   then kWaves ints            completed steps per wave
template <int NT, int QB, bool PERTURB>
__global__ void __launch_bounds__(kWaves * 64)
    dense_stream_kernel(const float* __restrict__ X, const float* __restrict__ A_op, float* __restrict__ P,
                        float* __restrict__ Q, int64_t n, int q, int kp, int qfirst, int ngroups, int n_panels,
                        int n_chunks, int64_t rows_per_chunk, uint32_t k0, uint32_t k1, float dscaled, int vec_ok,
                        int t_first, const float* __restrict__ A_opQ, int64_t aop_tstride, int64_t out_tstride,
                        int32_t* __restrict__ timeout_flag, int spin_limit, float* __restrict__ Ppart,
                        int64_t ppart_stride) {
  constexpr int NG = QB * NT;                       // product groups (member, 16-column block)
  constexpr int QLDS = kTiles * NG * 256;           // floats of the Q accumulator
  constexpr int TBUF = QB * 16 * kTLD;              // floats of transposition space per wave
  extern __shared__ __attribute__((aligned(16))) float lds[];
  float* qlds = lds;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, row = lane >> 4;
  float* tbuf = lds + QLDS + wave * TBUF;
  // done[w]: number of steps wave w has completed (see the hand-over of the tile columns below)
  int* done = reinterpret_cast<int*>(lds + QLDS + kWaves * TBUF);
  if (lane == 0) done[wave] = 0;

  // Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous range of logical indices so
  // that the workgroups adding to the same rows of P (same chunk, neighbouring panels) share one L2.
  int64_t logical;
  {
    const int64_t total = gridDim.x, L = blockIdx.x;
    const int64_t base = total >> 3, rem = total & 7, xcd = L & 7, slot = L >> 3;
    logical = xcd * base + (xcd < rem ? xcd : rem) + slot;
  }
  const int panel = (int)(logical % n_panels);
  const int chunk = (int)((logical / n_panels) % n_chunks);
  const int z = (int)(logical / ((int64_t)n_panels * n_chunks));
  const int t = z / ngroups, grp = z % ngroups;
  // Members [q0, q0 + QB) share one Philox block (QB divides 8 and q0 is a multiple of QB).  Slots at or
  // beyond q (a rounded-up tail group) are computed on whatever the spare operand slots hold and never written.
  const int q0 = qfirst + grp * QB;
  const int qb = (q - q0) < QB ? (q - q0) : QB;
  const uint32_t sub = (uint32_t)(q0 >> 3);         // Philox block index of this member group
  const int hoff = QB == 8 ? 0 : (q0 & 7);          // first 16-bit half used by the group
  const int64_t jp0 = (int64_t)panel * kPanel;
  const int64_t i_begin = (int64_t)chunk * rows_per_chunk;
  int64_t i_end = i_begin + rows_per_chunk;
  if (i_end > n) i_end = n;
  const float* Xt = X + (int64_t)t * n * n;
  // Reproducible mode (Ppart given): the panel's sums for X_t A are stored in the panel's own copy, and, the chunk
  // being the whole slice then, X_t^T A is stored by its only writer; nothing is added atomically.
  const bool ordered = Ppart != nullptr;
  float* Pt = ordered ? Ppart + (int64_t)panel * ppart_stride + (int64_t)t * out_tstride : P + (int64_t)t * out_tstride;
  float* Qt = Q + (int64_t)t * out_tstride;
  const int n32 = (int)n;
  int tiles = (int)((n - jp0 + 15) >> 4);           // tiles of the panel that hold columns of the matrix
  if (tiles > kTiles) tiles = kTiles;

  for (int e = tid; e < QLDS; e += kWaves * 64) qlds[e] = 0.0f;
  __syncthreads();

  // Operand address of (tile of 16 entities, product group g), in float4 units: a wave-uniform part
  // (tile, first member, g) plus the lane.
  // The two products may take their right operands from different arrays, and from a different one per slice
  // (aop_tstride floats apart): the iteration itself passes the same A for both and every slice.
  const int64_t tile_f4 = (int64_t)q * NT * 64;     // float4 per 16-entity tile
  const float4* Ag = reinterpret_cast<const float4*>(A_opQ + (int64_t)t * aop_tstride) + (int64_t)q0 * NT * 64;
  const float4* Ap = reinterpret_cast<const float4*>(A_op + (int64_t)t * aop_tstride) + (int64_t)q0 * NT * 64 +
                     (jp0 >> 4) * tile_f4;          // operands of the panel's column tiles, first group of this member group

  // A round = 8 strips of 16 rows, one per wave; in step s of a round wave w works on tile (w + s) % 8 of
  // its strip, so at any step every tile column of the Q accumulator belongs to one wave.  A column passes from
  // wave w + 1 to wave w; instead of a barrier per step each wave counts its completed steps in LDS and waits
  // only for the one wave it takes its column from.
  const int nstrips = (int)((i_end - i_begin + 15) >> 4);
  const int nrounds = (nstrips + kWaves - 1) / kWaves;
  auto tile_of = [&](int s) { return (wave + s) & (kTiles - 1); };
  // first row of this wave's strip in round rnd (a wave without a strip, or past the last round, reads the
  // chunk's first strip: valid memory, never used)
  // The workgroups of one chunk (one per panel) add to the same rows of P; each starts at a different round so
  // that they do not meet on the same rows at the same time.
  const int rnd0 = panel % nrounds;
  auto strip_of = [&](int rnd) -> int {
    int rr = rnd + rnd0;
    if (rr >= nrounds) rr -= nrounds;
    return rr * kWaves + wave;
  };
  auto strip_row = [&](int rnd) -> int64_t {
    const int strip = rnd < nrounds ? strip_of(rnd) : nstrips;
    return i_begin + 16 * (int64_t)(strip < nstrips ? strip : 0);
  };
  // X tile of global step g = 8 * round + step; the loads run two steps ahead, across strip boundaries
  auto x_fetch = [&](int g) -> float4 {
    const int64_t i0 = strip_row(g >> 3);
    const int rows_left = (int)(i_end - i0 < 16 ? i_end - i0 : 16);
    const int jt = tile_of(g & 7);
    const int jtc = jt < tiles ? jt : 0;            // a tile beyond the matrix: load something valid, never used
    const int64_t j0 = jp0 + 16 * jtc;
    const int cols_left = (int)(n - j0 < 16 ? n - j0 : 16);
    return load_tile(Xt + i0 * n + j0, vec_ok && rows_left == 16 && cols_left == 16, n32, rows_left, cols_left, l16,
                     row);
  };
  float4 bP[NG], bq[NG];
  auto bp_fetch = [&](int jt) {
#pragma unroll
    for (int g = 0; g < NG; ++g) bP[g] = (Ap + jt * tile_f4 + g * 64)[lane];   // rows < n_pad: always valid
  };
  // right operands of the Q products: the strip's 16 rows of A
  auto bq_fetch = [&](int rnd) {
    const int64_t i0 = strip_row(rnd);
#pragma unroll
    for (int g = 0; g < NG; ++g) bq[g] = (Ag + (i0 >> 4) * tile_f4 + g * 64)[lane];
  };
  float4 xn1 = x_fetch(0);
  float4 xn2 = x_fetch(1);
  bp_fetch(tile_of(0));
  bq_fetch(0);
  const int nsteps = nrounds * kTiles;
  // Hand-over of the tile columns: wave w may touch the column of its step g once wave w + 1 has completed g steps
  // (it had that column in step g - 1).  EVERY wave waits like this in every step before its own count moves, so
  // that a count of g + 1 implies counts of at least g, g - 1, ... down the chain.  (Every wave makes the same
  // number of steps and a wait only concerns an earlier step of a wave that is resident on the same CU, so the
  // waits always end, after microseconds.)  The spin count is bounded all the same (spin_limit polls; the launcher
  // passes 2^20, about 30 ms, far more than the time a neighbour can be held back at the generator's low issue
  // priority).  A wait that runs out is an error, never a silent fall-through: the wave reports it in *timeout_flag
  // (one plain store by lane 0), leaves the Q half of that step out (the column may still be its neighbour's) and
  // goes on counting, so that the kernel exits normally; the host turns the flag into an error status.
  auto wait_for_neighbour = [&](int gstep) -> bool {
    const int nb = (wave + 1) & (kWaves - 1);
    bool arrived = false;
    for (int spin = 0; spin < spin_limit; ++spin) {
      const int c = __builtin_amdgcn_readfirstlane(
          __hip_atomic_load(&done[nb], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
      if (c >= gstep) {
        arrived = true;
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    if (!arrived && lane == 0 && timeout_flag)
      __hip_atomic_store(timeout_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    return arrived;
  };

  for (int rnd = 0; rnd < nrounds; ++rnd) {
    const int strip = strip_of(rnd);
    const bool have_strip = strip < nstrips;        // wave-uniform
    const int64_t i0 = strip_row(rnd);
    floatx4 pacc[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) pacc[g] = floatx4{0.f, 0.f, 0.f, 0.f};

    for (int s = 0; s < kTiles; ++s) {
      const int jt = tile_of(s);
      const bool work = have_strip && jt < tiles;   // wave-uniform
      const float4 xc = xn1;
      xn1 = xn2;
      if (rnd * kTiles + s + 2 < nsteps) xn2 = x_fetch(rnd * kTiles + s + 2);
      if (work) {
        const float xcur[4] = {xc.x, xc.y, xc.z, xc.w};
        // ---- the generator: one Philox block per element serves all QB members
        __builtin_amdgcn_s_setprio(kPrioGenerator);
        u32x4 w[4];
        if (PERTURB) {
          const uint64_t e0 = (uint64_t)(i0 + l16) * (uint64_t)n + (uint64_t)(jp0 + 16 * jt + 4 * row);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const uint64_t e = e0 + (uint64_t)r;
            w[r] = front_halves<QB>(
                philox4x32_10((uint32_t)e, (uint32_t)(e >> 32), (uint32_t)(t + t_first), sub, k0, k1), hoff);
          }
        }
        // ---- per member: perturbed tile in "row" orientation -> P products; park it in LDS for the transpose
        __builtin_amdgcn_s_setprio(kPrioPProducts);
#pragma unroll
        for (int qq = 0; qq < QB; ++qq) {
          float xq[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) xq[r] = PERTURB ? perturbed(xcur[r], w[r], qq, dscaled) : xcur[r];
          *reinterpret_cast<float4*>(tbuf + (qq * 16 + l16) * kTLD + 4 * row) = float4{xq[0], xq[1], xq[2], xq[3]};
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const int g = qq * NT + nt;
            pacc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(xq[0], bP[g].x, pacc[g], 0, 0, 0);
            pacc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(xq[1], bP[g].y, pacc[g], 0, 0, 0);
            pacc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(xq[2], bP[g].z, pacc[g], 0, 0, 0);
            pacc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(xq[3], bP[g].w, pacc[g], 0, 0, 0);
          }
        }
      }
      __builtin_amdgcn_s_setprio(kPrioRest);
      // the operand registers are free again: fetch the next tile's
      bp_fetch(tile_of((s + 1) & (kTiles - 1)));
      if (work) {
        // ---- "column" orientation read back from LDS: lane (l16, row) gets X^q[i0 + 4*row + r][j0 + l16];
        //      the tile's Q accumulators are this wave's alone until the next barrier
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // Tile column jt was wave (wave + 1) % 8's in the previous step: wait until that wave has completed it.
        const bool mine = wait_for_neighbour(rnd * kTiles + s);   // wave-uniform
        float4* qt = reinterpret_cast<float4*>(qlds) + (jt * NG) * 64 + lane;
        // all LDS reads first (one wait), then the products back to back, then the stores
        float xt[QB][4];
        floatx4 qa[NG];
#pragma unroll
        for (int qq = 0; qq < QB; ++qq)
#pragma unroll
          for (int r = 0; r < 4; ++r) xt[qq][r] = tbuf[(qq * 16 + 4 * row + r) * kTLD + l16];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          const float4 c = qt[g * 64];
          qa[g] = floatx4{c.x, c.y, c.z, c.w};
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int qq = 0; qq < QB; ++qq)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const int g = qq * NT + nt;
            qa[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(xt[qq][0], bq[g].x, qa[g], 0, 0, 0);
            qa[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(xt[qq][1], bq[g].y, qa[g], 0, 0, 0);
            qa[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(xt[qq][2], bq[g].z, qa[g], 0, 0, 0);
            qa[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(xt[qq][3], bq[g].w, qa[g], 0, 0, 0);
          }
        __builtin_amdgcn_sched_barrier(0);
        if (mine) {
#pragma unroll
          for (int g = 0; g < NG; ++g) qt[g * 64] = float4{qa[g][0], qa[g][1], qa[g][2], qa[g][3]};
        }
      } else {
        // A wave with nothing to do in this step (no strip in the chunk's last round, or a tile beyond the matrix)
        // still is a link of the chain: its count may move only after its neighbour's, or the wave behind it
        // could take the column over while the wave in front is still working on it.
        (void)wait_for_neighbour(rnd * kTiles + s);
      }
      // the strip's last Q products are done: fetch the next strip's operands behind them
      if (s == kTiles - 1 && rnd + 1 < nrounds) bq_fetch(rnd + 1);
      // hand the tile column on: the accumulators are in LDS before the count moves
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      if (lane == 0)
        __hip_atomic_store(&done[wave], rnd * kTiles + s + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    // ---- the strip's P (16 rows, summed over the panel's columns): add to memory
    if (have_strip) {
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const int qq = g / NT, nt = g % NT;
        if (qq < qb) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int64_t i = i0 + 4 * row + r;
            const float v = pacc[g][r];
            if (ordered) {
              if (i < i_end) Pt[(i * q + q0 + qq) * kp + nt * 16 + l16] = v;
            } else if (i < i_end && v != 0.0f) {
              unsafeAtomicAdd(&Pt[(i * q + q0 + qq) * kp + nt * 16 + l16], v);
            }
          }
        }
      }
    }
  }
  __syncthreads();
  // ---- the panel's Q (summed over the chunk's rows): add to memory (every wave has made its last step)
  for (int e = tid; e < tiles * NG * 256; e += kWaves * 64) {
    const float v = qlds[e];
    const int r = e & 3, ln = (e >> 2) & 63, g = (e >> 8) % NG, jt = (e >> 8) / NG;
    const int qq = g / NT, nt = g % NT;
    const int64_t j = jp0 + 16 * jt + 4 * (ln >> 4) + r;
    if (ordered) {
      if (qq < qb && j < n) Qt[(j * q + q0 + qq) * kp + nt * 16 + (ln & 15)] = v;
    } else if (qq < qb && j < n && v != 0.0f) {
      unsafeAtomicAdd(&Qt[(j * q + q0 + qq) * kp + nt * 16 + (ln & 15)], v);
    }
  }
}

template <int NT, int QB>
constexpr size_t stream_lds_bytes() {
  return (size_t)(kTiles * QB * NT * 256 + kWaves * QB * 16 * kTLD + kWaves) * sizeof(float);
}

const char* dense_stream_kernel_name() { return "dense_stream_kernel"; }

template <int NT, int QB>
static hipError_t launch_stream_t(const float* X, const float* A_op, float* P, float* Q, const Dims& d, int qfirst,
                                  int ngroups, uint64_t seed, float delta, hipStream_t s, const DenseStreamOpts& o) {
  const int t_first = o.t_first;
  const float* A_opQ = o.A_opQ ? o.A_opQ : A_op;
  const int64_t aop_tstride = o.aop_tstride;
  const int64_t out_tstride = o.out_tstride < 0 ? d.n * d.q * (int64_t)d.kp : o.out_tstride;
  int32_t* timeout_flag = o.timeout_flag;
  const int spin_limit = o.spin_limit > 0 ? o.spin_limit : (o.spin_limit < 0 ? 0 : (1 << 20));
  float* Ppart = o.Ppart;
  const int64_t ppart_stride = (int64_t)d.m * d.n * d.q * d.kp;   // one copy of P per panel
  if (Ppart && out_tstride != d.n * d.q * (int64_t)d.kp) return hipErrorInvalidValue;   // (not with summed slices)
  static_assert(QB * NT <= 8, "at most 8 product groups per tile");
  static_assert(kTiles == kWaves && (kTiles & (kTiles - 1)) == 0, "one tile column per wave and step");
  constexpr size_t lds = stream_lds_bytes<NT, QB>();
  static_assert(lds <= 160 * 1024, "LDS budget of one CU");
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)dense_stream_kernel<NT, QB, true>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void*)dense_stream_kernel<NT, QB, false>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int64_t n_panels = ceil_div(d.n, kPanel);
  // Rows are cut into chunks (whole rounds of 8 strips = 128 rows) so that the 256 CUs, one workgroup each at a
  // time, are busy: more chunks even out the last wave of workgroups, fewer chunks save the fixed cost of a
  // workgroup (clearing and adding out its share of Q, filling its pipeline: about 7 steps, i.e. the time of
  // ~112 rows, measured).  Pick the count with the least estimated time.
  const int64_t base = n_panels * d.m * ngroups;
  const int64_t max_chunks = ceil_div(d.n, 16 * kWaves);
  int64_t n_chunks = 1, best = -1;
  for (int64_t c = 1; c <= max_chunks && c <= 256; ++c) {
    const int64_t rows = round_up(ceil_div(d.n, c), 16 * kWaves);
    const int64_t waves_of_wgs = ceil_div(base * ceil_div(d.n, rows), 256);
    // (a single wave of workgroups measured 20 % slower than two of half the length: nothing overlaps its ends)
    const int64_t cost = waves_of_wgs * (rows + 112) * (waves_of_wgs == 1 ? 5 : 4);
    if (best < 0 || cost < best) {
      best = cost;
      n_chunks = c;
    }
  }
  if (Ppart) n_chunks = 1;                          // one workgroup per panel and slice: the only writer of its X_t^T A
  const int64_t rows_per_chunk = round_up(ceil_div(d.n, n_chunks), 16 * kWaves);
  n_chunks = ceil_div(d.n, rows_per_chunk);
  const int64_t total = n_panels * n_chunks * d.m * ngroups;
  if (total > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  const int vec_ok = (d.n % 4 == 0) && (((uintptr_t)X & 15) == 0);
  if (delta != 0.0f)
    hipLaunchKernelGGL((dense_stream_kernel<NT, QB, true>), dim3((unsigned)total), dim3(kWaves * 64), lds, s, X, A_op, P,
                       Q, d.n, d.q, d.kp, qfirst, ngroups, (int)n_panels, (int)n_chunks, rows_per_chunk, (uint32_t)seed,
                       (uint32_t)(seed >> 32), delta * 0x1p-16f, vec_ok, t_first, A_opQ, aop_tstride, out_tstride,
                       timeout_flag, spin_limit, Ppart, ppart_stride);
  else
    hipLaunchKernelGGL((dense_stream_kernel<NT, QB, false>), dim3((unsigned)total), dim3(kWaves * 64), lds, s, X, A_op,
                       P, Q, d.n, d.q, d.kp, qfirst, ngroups, (int)n_panels, (int)n_chunks, rows_per_chunk,
                       (uint32_t)seed, (uint32_t)(seed >> 32), 0.0f, vec_ok, t_first, A_opQ, aop_tstride, out_tstride,
                       timeout_flag, spin_limit, Ppart, ppart_stride);
  return hipGetLastError();
}

// Members per group so that (members) x (16-column blocks) <= 8 product groups: 8 members for k <= 16,
// 4 for k <= 32, 2 for k <= 64.
static int group_members(int kp) { return kp <= 16 ? 8 : (kp <= 32 ? 4 : 2); }

int64_t dense_stream_panels(const Dims& d) { return ceil_div(d.n, kPanel); }

DensePlan dense_stream_plan(const Dims& d) {
  const int qbig = group_members(d.kp);
  DensePlan pl;
  pl.full_groups = d.q / qbig;
  pl.full_qb = qbig;
  pl.tail_members = d.q - pl.full_groups * qbig;
  pl.tail_qb = pl.tail_members == 0 ? 0 : 1;
  while (pl.tail_qb < pl.tail_members) pl.tail_qb *= 2;
  return pl;
}

template <int NT, int QB>
static hipError_t launch_tail(const float* X, const float* A_op, float* P, float* Q, const Dims& d, int qf,
                              uint64_t seed, float delta, hipStream_t s, const DenseStreamOpts& o) {
  if constexpr (QB * NT <= 8)
    return launch_stream_t<NT, QB>(X, A_op, P, Q, d, qf, 1, seed, delta, s, o);
  else
    return hipErrorInvalidValue;
}

template <int NT>
static hipError_t launch_stream_nt(const float* X, const float* A_op, float* P, float* Q, const Dims& d, int part,
                                   uint64_t seed, float delta, hipStream_t s, const DenseStreamOpts& o) {
  constexpr int QBIG = NT == 1 ? 8 : (NT == 2 ? 4 : 2);
  const DensePlan pl = dense_stream_plan(d);
  if (part == 0) {
    if (pl.full_groups == 0) return hipSuccess;
    return launch_stream_t<NT, QBIG>(X, A_op, P, Q, d, 0, pl.full_groups, seed, delta, s, o);
  }
  const int qf = pl.full_groups * QBIG;
  switch (pl.tail_qb) {
    case 0: return hipSuccess;
    case 1: return launch_tail<NT, 1>(X, A_op, P, Q, d, qf, seed, delta, s, o);
    case 2: return launch_tail<NT, 2>(X, A_op, P, Q, d, qf, seed, delta, s, o);
    case 4: return launch_tail<NT, 4>(X, A_op, P, Q, d, qf, seed, delta, s, o);
    default: return launch_tail<NT, 8>(X, A_op, P, Q, d, qf, seed, delta, s, o);
  }
}

hipError_t launch_dense_stream(const float* X, const float* A_op, float* P, float* Q, const Dims& d, int part,
                               uint64_t seed, float delta, hipStream_t s, const DenseStreamOpts& o) {
  switch (d.kp / 16) {
    case 1: return launch_stream_nt<1>(X, A_op, P, Q, d, part, seed, delta, s, o);
    case 2: return launch_stream_nt<2>(X, A_op, P, Q, d, part, seed, delta, s, o);
    case 3: return launch_stream_nt<3>(X, A_op, P, Q, d, part, seed, delta, s, o);
    case 4: return launch_stream_nt<4>(X, A_op, P, Q, d, part, seed, delta, s, o);
    default: return hipErrorInvalidValue;
  }
}

// ------------------------------------------------------------------------------------------ Alg. 4 made explicit
__global__ void dense_perturb_kernel(const float* __restrict__ X, float* __restrict__ out, int64_t n, int m,
                                     int member, uint32_t k0, uint32_t k1, float dscaled, int perturb) {
  const int64_t per = n * n;
  const int64_t total = per * m;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int t = (int)(idx / per);
    const uint64_t e = (uint64_t)(idx % per);
    float v = X[idx];
    if (perturb) {
      const u32x4 w = philox4x32_10((uint32_t)e, (uint32_t)(e >> 32), (uint32_t)t, (uint32_t)(member >> 3), k0, k1);
      v = perturbed(v, w, member & 7, dscaled);
    }
    out[idx] = v;
  }
}

hipError_t launch_dense_perturb(const float* X, float* out, int64_t n, int m, int member, uint64_t seed,
                                float delta, hipStream_t s) {
  int64_t blocks = ceil_div(n * n * m, 256);
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(dense_perturb_kernel, dim3((unsigned)blocks), dim3(256), 0, s, X, out, n, m, member,
                     (uint32_t)seed, (uint32_t)(seed >> 32), delta * 0x1p-16f, delta != 0.0f ? 1 : 0);
  return hipGetLastError();
}

// sum_t ||X^r_t||_F^2 for every member (the constant term of the expanded objective of Eq. 1)
__global__ void __launch_bounds__(256) dense_xnorm_kernel(const float* __restrict__ X, double* __restrict__ xn,
                                                          int64_t n, int m, int q, uint32_t k0, uint32_t k1,
                                                          float dscaled, int perturb, double* __restrict__ part) {
  __shared__ double red[4];
  const int64_t per = n * n;
  const int64_t total = per * m;
  for (int b = 0; b < (q + 7) / 8; ++b) {
    double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int qb = (q - 8 * b) < 8 ? (q - 8 * b) : 8;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x) {
      const int t = (int)(idx / per);
      const uint64_t e = (uint64_t)(idx % per);
      const float v = X[idx];
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
      if (qq < qb) {  // block-uniform
        double v = acc[qq];
        for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
        __syncthreads();
        if (threadIdx.x == 0) {
          const double sum = red[0] + red[1] + red[2] + red[3];
          if (part) part[(int64_t)blockIdx.x * q + 8 * b + qq] = sum;   // reproducible mode: block sums, added in order later
          else atomicAdd(&xn[8 * b + qq], sum);
        }
      }
    }
  }
}

hipError_t launch_dense_xnorm(const float* X, double* xn, int64_t n, int m, int q, uint64_t seed, float delta,
                              hipStream_t s, double* part) {
  int64_t blocks = ceil_div(n * n * m, 256 * 8);
  if (blocks > kXnormMaxBlocks) blocks = kXnormMaxBlocks;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(dense_xnorm_kernel, dim3((unsigned)blocks), dim3(256), 0, s, X, xn, n, m, q, (uint32_t)seed,
                     (uint32_t)(seed >> 32), delta * 0x1p-16f, delta != 0.0f ? 1 : 0, part);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && part) e = launch_reduce_parts_f64(xn, part, q, blocks, q, 1, s);
  return e;
}

}  // namespace nnr
