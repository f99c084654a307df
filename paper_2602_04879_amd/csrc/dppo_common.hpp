// Shared device helpers for the DPPO loss kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dppo {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;   // logits below this are treated as -inf
constexpr double kTiny = 1e-30;       // floor for a vanishing denominator inside x*ln(x/y)

enum : int { kBinaryTV = 0, kBinaryKL = 1, kTopkTV = 2, kTopkKL = 3 };

// Kernel arguments (device pointers; one call).
struct KParams {
  const uint16_t* logits;   // bf16 bits [T, ld]
  uint16_t* grad;           // bf16 bits [T, ld] or nullptr
  const int32_t* sampled;   // [T]
  const float* mu_logp;     // [T]
  const int32_t* tk_ids;    // [T, K] or nullptr
  const float* tk_lp;       // [T, K] or nullptr
  const float* adv;         // [T]
  float* loss_tok;          // [T] or nullptr
  float* divergence;        // [T]
  uint8_t* mask;            // [T]
  double* partial;          // [gridDim.x] per-workgroup loss partial sums (workspace)
  int64_t ld;
  int32_t T, V, K, variant;
  float delta, loss_scale;
};

// What the per-row epilogue hands to the gradient pass.
struct RowCoef {
  float kexp;     // g_j = sgn * exp2(z_j*log2e + kexp) for j != a_t ; -inf-like when coef == 0
  float coef;     // c_t = loss_scale * M_t * A_t * r_t
  float g_a;      // gradient entry of the sampled token, c_t * (pi(a_t) - 1)
};

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// Round-to-nearest-even pack of two floats into two bf16 (lo in bits 0..15).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte vector = 8 bf16
// Pointers known to be in global memory (address space 1): lets the compiler emit global_*
// instructions with a scalar base instead of flat_* ones.
typedef const __attribute__((address_space(1))) u32x4* gvec_cptr;
typedef __attribute__((address_space(1))) u32x4* gvec_ptr;
typedef const __attribute__((address_space(1))) uint16_t* gu16_cptr;
typedef __attribute__((address_space(1))) uint16_t* gu16_ptr;
typedef const __attribute__((address_space(1))) char* gbyte_cptr;
typedef __attribute__((address_space(1))) char* gbyte_ptr;

// 16-byte access at (uniform base) + (per-lane unsigned 32-bit byte offset): the form that maps
// to a global_load/store with a scalar base register and one vector offset register.
__device__ __forceinline__ u32x4 gload16(gbyte_cptr base, uint32_t voff) {
  return *reinterpret_cast<gvec_cptr>(base + voff);
}
__device__ __forceinline__ void gstore16_nt(gbyte_ptr base, uint32_t voff, u32x4 v) {
  __builtin_nontemporal_store(v, reinterpret_cast<gvec_ptr>(base + voff));
}

// A value every lane of the wave holds identically, moved to a scalar register.
__device__ __forceinline__ int uniform_i(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float uniform_f(float v) {
  return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v)));
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2_t v = {lo, hi};
  bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
  return *reinterpret_cast<uint32_t*>(&b);
}
__device__ __forceinline__ uint16_t float_to_bf16_bits(float x) {
  return static_cast<uint16_t>(pack_bf16x2(x, 0.f) & 0xffffu);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// x * ln(x / y) with 0 ln 0 = 0 and the denominator floored.
__device__ __forceinline__ double xlogx_over_y(double x, double y) {
  if (x <= 0.0) return 0.0;
  return x * (log(x) - log(fmax(y, kTiny)));
}

// Per-row epilogue, executed by ONE full wave (all 64 lanes call it with the same scalars).
// The row statistics arrive in the base-2 domain the streaming passes work in:
//   b      : offset (an integer-valued float) with z_j*log2e + b <= 0 for every j
//   S_rest : sum over j != a_t of 2^(z_j*log2e + b).  The sampled token's own term is left out
//            so that 1 - pi(a_t) = S_rest / S keeps full relative accuracy when pi(a_t) -> 1.
// log2e is the fp32 constant kLog2e everywhere (passes and epilogue), so the probabilities
// are mutually consistent; its rounding (1.3e-8 relative) acts as a temperature of 1+1.3e-8.
// Steps: ratio (Eq. ppo-clip), divergence (Eq. binary_tv / binary_kl / topk_tv / topk_kl),
// mask and loss term (Eq. dppo_obj), gradient coefficient (Eq. unified_grad, C = infinity).
// Lane 0 stores the per-token outputs; every lane returns the same RowCoef and *loss_term.
// Deliberately NOT inlined: its float64 arithmetic needs many registers, and as a real call its
// register traffic stays inside the one wave that runs it instead of raising the pressure of
// the streaming phases around it.
__device__ __attribute__((noinline)) static RowCoef row_epilogue(const KParams& p, int row, int a, const uint16_t* zrow,
                                                float b, double S_rest, int lane, double* loss_term) {
  constexpr double kL = static_cast<double>(kLog2e);
  constexpr double kLn2 = 0.6931471805599453;
  const double bd = static_cast<double>(b);
  const double xa = static_cast<double>(bf16_bits_to_float(zrow[a])) * kL + bd;   // log2 of a_t's term
  const double ea = exp2(xa);
  const double S = S_rest + ea;
  const double log2S = log2(S);
  const double lpi = (xa - log2S) * kLn2;
  const double lmu_raw = static_cast<double>(p.mu_logp[row]);
  const double lmu = fmin(lmu_raw, 0.0);
  const double pa = exp(lmu), qa = ea / S;
  const double one_minus_qa = S_rest / S;
  double D;
  if (p.variant == kBinaryTV || ((p.variant == kTopkTV) && p.K == 0)) {
    D = fabs(pa - qa);
  } else if (p.variant == kBinaryKL || ((p.variant == kTopkKL) && p.K == 0)) {
    D = xlogx_over_y(pa, qa) + xlogx_over_y(-expm1(lmu), one_minus_qa);
  } else {
    // reduced distributions over TopK(mu, K) U {a_t} U {other}  (Sec. 4.4)
    const bool tv = (p.variant == kTopkTV);
    double sp = 0.0, sq = 0.0, acc = 0.0;
    const int32_t* ids = p.tk_ids + static_cast<int64_t>(row) * p.K;
    const float* lps = p.tk_lp + static_cast<int64_t>(row) * p.K;
    for (int k = lane; k < p.K; k += kWave) {
      const int id = ids[k];
      if (id >= 0 && id < p.V && id != a) {
        const double pk = exp(fmin(static_cast<double>(lps[k]), 0.0));
        const double qk = exp2(static_cast<double>(bf16_bits_to_float(zrow[id])) * kL + bd - log2S);
        sp += pk;
        sq += qk;
        acc += tv ? fabs(pk - qk) : xlogx_over_y(pk, qk);
      }
    }
    sp = wave_sum(sp) + pa;
    sq = wave_sum(sq) + qa;
    acc = wave_sum(acc) + (tv ? fabs(pa - qa) : xlogx_over_y(pa, qa));
    const double po = fmax(1.0 - sp, 0.0), qo = fmax(1.0 - sq, 0.0);
    D = tv ? 0.5 * (acc + fabs(po - qo)) : acc + xlogx_over_y(po, qo);
  }
  const double A = static_cast<double>(p.adv[row]);
  const bool blocked = (D > static_cast<double>(p.delta)) &&
                       ((A > 0.0 && lpi > lmu_raw) || (A < 0.0 && lpi < lmu_raw));
  const double M = blocked ? 0.0 : 1.0;
  const double r = exp(lpi - lmu_raw);
  const double lt = -M * r * A;
  const double c = static_cast<double>(p.loss_scale) * M * A * r;
  if (lane == 0) {
    p.divergence[row] = static_cast<float>(D);
    p.mask[row] = blocked ? 0 : 1;
    if (p.loss_tok) p.loss_tok[row] = static_cast<float>(lt);
  }
  *loss_term = lt;
  RowCoef rc;
  rc.coef = static_cast<float>(c);
  rc.g_a = static_cast<float>(-c * one_minus_qa);
  // c * pi_j = sgn(c) * 2^(z_j*log2e + kexp)
  rc.kexp = (c != 0.0) ? static_cast<float>(log2(fabs(c)) + bd - log2S) : 0.f;
  return rc;
}

}  // namespace dppo
