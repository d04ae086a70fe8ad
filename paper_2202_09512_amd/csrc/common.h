// Shared device helpers: Philox4x32-10, the perturbation factor, launch helpers.
// Random stream (this library's reading of Alg. 4's "uniformRandom" and Alg. 3 step 1's "rand"):
//   key = (lo32(seed), hi32(seed)); counter = (lo32(e), hi32(e), c2, (domain << 16) | sub)
//   perturbation: domain 0, e = i*n + j, c2 = slice, sub = member >> 3; member uses 16-bit half
//                 (member & 7) of the block: word (member & 7) >> 1, low half if even, high if odd
//   A init: domain 1, e = i*k + s, c2 = k, sub = member;  R init: domain 2, e = (t*k + a)*k + b
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define NNRESCAL_MAX_K_INTERNAL 64
#define NNRESCAL_MAX_Q_INTERNAL 64

namespace nnr {

constexpr uint32_t kPhiloxM0 = 0xD2511F53u;
constexpr uint32_t kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u;
constexpr uint32_t kPhiloxW1 = 0xBB67AE85u;

struct u32x4 {
  uint32_t x, y, z, w;
};

// a ^ b ^ c in one instruction (gfx950 three-input bit operation, truth table 0x96)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies and a word shuffle.
__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                               uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)kPhiloxM0 * c0;
    const uint64_t p1 = (uint64_t)kPhiloxM1 * c2;
    const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
    const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += kPhiloxW0;
    k1 += kPhiloxW1;
  }
  return u32x4{c0, c1, c2, c3};
}

// Element of the perturbed tensor (Alg. 4) for the member that owns 16-bit half `r` (0..7) of a block: word r >> 1,
// low half if r is even.  With h that half, a = delta * 2^-15 (exact) and c = fl32(1 - 65535 * delta * 2^-16):
//   X^q = fl32( fl32(x a) * h + fl32(x c) )        (the last step is ONE fused multiply-add)
// which is x * (1 + delta * (2h - 65535) / 65536) to within 1.5 ulp.  x a and x c are shared by the members that use
// the same block, so a member costs two instructions (a convert of the half-word with a sub-dword operand select,
// and the multiply-add).  dscaled = delta * 2^-16.
__device__ __forceinline__ float perturbed(float x, const u32x4& w, int r, float dscaled) {
  const uint32_t word = (r >> 1) == 0 ? w.x : (r >> 1) == 1 ? w.y : (r >> 1) == 2 ? w.z : w.w;
  const float hf = (r & 1) ? (float)(word >> 16) : (float)(word & 0xFFFFu);
  const float a = 2.0f * dscaled;
  const float c = __fmaf_rn(-65535.0f, dscaled, 1.0f);
  return __fmaf_rn(__fmul_rn(x, a), hf, __fmul_rn(x, c));
}

// Uniform in (0,1): (2*(w >> 9) + 1) * 2^-24, an odd multiple of 2^-24: exact, never 0 or 1.
__device__ __forceinline__ float unit_open(uint32_t w) { return (float)(2u * (w >> 9) + 1u) * 0x1p-24f; }

__host__ __device__ inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
__host__ __device__ inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

}  // namespace nnr
