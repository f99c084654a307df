// Pieces shared by the register-resident loss kernels: packed-bf16 helpers of the row statistics
// and of the gradient.
#pragma once
#include "dppo_common.hpp"

namespace dppo {
namespace {

typedef short s16x2 __attribute__((ext_vector_type(2)));

constexpr uint32_t kNegInfPair = 0xFF80FF80u;   // two bf16 -inf

__device__ __forceinline__ s16x2 as_s16x2(uint32_t w) { return __builtin_bit_cast(s16x2, w); }

// Replace 16-bit entry `sub` (0..7) of a packed vector by `bits`.
__device__ __forceinline__ u32x4 patch16(u32x4 v, int sub, uint32_t bits) {
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int d = 0; d < 4; ++d)
    if ((sub >> 1) == d) w[d] = (sub & 1) ? ((w[d] & 0x0000ffffu) | (bits << 16)) : ((w[d] & 0xffff0000u) | bits);
  const u32x4 r = {w[0], w[1], w[2], w[3]};
  return r;
}

// One packed word (two bf16): returns e0 + e1 and adds e*x to t, with x = z*log2e + b and
// e = 2^x (t feeds the entropy; a vanished term, e = 0 with x = -inf, adds nothing).
__device__ __forceinline__ float accum2(uint32_t w, float b, float& t) {
  const float x0 = fmaf(__uint_as_float(w << 16), kLog2e, b), x1 = fmaf(__uint_as_float(w & 0xffff0000u), kLog2e, b);
  const float e0 = fast_exp2(x0), e1 = fast_exp2(x1);
  t = fma_ex(e0, x0, fma_ex(e1, x1, t));
  return e0 + e1;
}

// 2^(z*log2e + k) for the two bf16 halves of a packed word.
__device__ __forceinline__ float exp_lo(uint32_t w, float k) { return fast_exp2(fmaf(__uint_as_float(w << 16), kLog2e, k)); }
__device__ __forceinline__ float exp_hi(uint32_t w, float k) { return fast_exp2(fmaf(__uint_as_float(w & 0xffff0000u), kLog2e, k)); }

// Gradient of the eight entries of one chunk: sgn * 2^(z*log2e + kexp), rounded to bf16.
__device__ __forceinline__ u32x4 grad8(u32x4 v, float kexp, uint32_t sgn) {
  const u32x4 o = {pack_bf16x2(exp_lo(v.x, kexp), exp_hi(v.x, kexp)) ^ sgn, pack_bf16x2(exp_lo(v.y, kexp), exp_hi(v.y, kexp)) ^ sgn,
                   pack_bf16x2(exp_lo(v.z, kexp), exp_hi(v.z, kexp)) ^ sgn, pack_bf16x2(exp_lo(v.w, kexp), exp_hi(v.w, kexp)) ^ sgn};
  return o;
}

}  // namespace
}  // namespace dppo
