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

// Keep the 16-bit entries lo .. hi-1 of a packed vector, the others become bf16 -inf.
__device__ __forceinline__ u32x4 keep16(u32x4 v, int lo, int hi) {
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const bool k0 = (2 * d >= lo && 2 * d < hi), k1 = (2 * d + 1 >= lo && 2 * d + 1 < hi);
    const uint32_t keep = (k0 ? 0x0000ffffu : 0u) | (k1 ? 0xffff0000u : 0u);
    w[d] = (w[d] & keep) | (kNegInfPair & ~keep);
  }
  const u32x4 r = {w[0], w[1], w[2], w[3]};
  return r;
}

// Entries lo .. hi-1 of a packed vector stored two bytes at a time: entry e goes to entry
// e + shift of the row the descriptor covers (range-checked).  Issued from inline assembly like
// row_store16_untracked, with the same wait states around each store.
__device__ __forceinline__ void store_entries_untracked(row_desc_t d, u32x4 o, int lo, int hi, int shift) {
  const uint32_t w[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    if (e >= lo && e < hi) {
      const uint32_t val = (e & 1) ? (w[e >> 1] >> 16) : w[e >> 1];
      const uint32_t off = static_cast<uint32_t>(e + shift) * 2u;
      asm volatile("s_nop 4\n\tbuffer_store_short %0, %1, %2, 0 offen\n\ts_nop 1" ::"v"(val), "v"(off), "s"(d) : "memory");
    }
  }
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

// Per-thread online statistics of a row, fed two 16-byte chunks at a time:
//   sd = sum 2^(z*log2e + b) with an integer offset b <= -max(z)*log2e that only ever decreases;
//   lowering it rescales the sum by an exact power of two.  t0..t3 (DIAG): sum 2^x * x, x = z*log2e + b.
// The maximum is taken on the PACKED bf16 patterns, as signed 16-bit integers: non-negative
// patterns order like the floats and every negative one stays below them, so the integer maximum
// is the float maximum whenever it is >= 0; if every entry so far is negative, the float maximum
// is the negative of smallest magnitude, which is the integer MINIMUM.
// The sum is kept in float64 and fed with the fp32 sum of each pair's exponentials (summed
// pairwise among themselves): a thread that has met a dominant entry then does not drop the small
// ones that follow it, as an fp32 accumulator would.
template <bool DIAG>
struct PackedRowStat {
  s16x2 mx = as_s16x2(0x80008000u), mn = as_s16x2(0x7FFF7FFFu);
  float b = 3.0e38f;                       // "+infinity": nothing seen yet
  double sd = 0.0;
  float t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f;
  __device__ __forceinline__ void add2(const u32x4& v0, const u32x4& v1) {
    const u32x4 v[2] = {v0, v1};
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      mx = __builtin_elementwise_max(mx, as_s16x2(v[i].x));
      mx = __builtin_elementwise_max(mx, as_s16x2(v[i].y));
      mx = __builtin_elementwise_max(mx, as_s16x2(v[i].z));
      mx = __builtin_elementwise_max(mx, as_s16x2(v[i].w));
      mn = __builtin_elementwise_min(mn, as_s16x2(v[i].x));
      mn = __builtin_elementwise_min(mn, as_s16x2(v[i].y));
      mn = __builtin_elementwise_min(mn, as_s16x2(v[i].z));
      mn = __builtin_elementwise_min(mn, as_s16x2(v[i].w));
    }
    const int hi16 = max(static_cast<int>(mx.x), static_cast<int>(mx.y));
    const int lo16 = min(static_cast<int>(mn.x), static_cast<int>(mn.y));
    const float zmax = __uint_as_float(static_cast<uint32_t>(hi16 >= 0 ? hi16 : lo16) << 16);
    const float bn = -ceilf(fmaxf(zmax, kNegBig) * kLog2e);
    // moving the offset by d: e -> e*2^d, x -> x + d, so s -> 2^d s and t -> 2^d (t + d s)
    const float d = bn - b;
    const float sc = fast_exp2(d);            // 1 when the maximum did not move
    if (DIAG) { t0 = sc * fmaf(d, static_cast<float>(sd), t0); t1 *= sc; t2 *= sc; t3 *= sc; }
    b = bn;
    float gs = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      float px, py, pz, pw;
      if (DIAG) {
        px = accum2(v[i].x, b, t0);
        py = accum2(v[i].y, b, t1);
        pz = accum2(v[i].z, b, t2);
        pw = accum2(v[i].w, b, t3);
      } else {
        px = exp_lo(v[i].x, b) + exp_hi(v[i].x, b);
        py = exp_lo(v[i].y, b) + exp_hi(v[i].y, b);
        pz = exp_lo(v[i].z, b) + exp_hi(v[i].z, b);
        pw = exp_lo(v[i].w, b) + exp_hi(v[i].w, b);
      }
      const float c = (px + py) + (pz + pw);
      gs = (i == 0) ? c : gs + c;
    }
    sd = fma(sd, static_cast<double>(sc), static_cast<double>(gs));
    __builtin_amdgcn_sched_barrier(0);   // one pair at a time: bounds the live temporaries
  }
  __device__ __forceinline__ float tsum() const { return (t0 + t1) + (t2 + t3); }
};

}  // namespace
}  // namespace dppo
