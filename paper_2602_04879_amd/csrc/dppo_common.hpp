// Shared device helpers for the DPPO loss kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dppo {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;   // logits below this are treated as -inf

enum : int { kBinaryTV = 0, kBinaryKL = 1, kTopkTV = 2, kTopkKL = 3, kFullTV = 4, kFullKL = 5 };

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
  float* diag;              // [T, 8] or nullptr
  double* partial;          // [gridDim.x] per-workgroup loss partial sums (workspace)
  // Rows handed out at run time (register-resident kernel with the gradient, see there): a
  // counter (cleared before the launch) and one loss term per ROW instead of one partial sum per
  // workgroup, so that the scalar loss does not depend on which workgroup took which row.  Both
  // nullptr: every workgroup takes the rows its index fixes.
  int32_t* row_counters;    // [1] (eight are cleared)
  double* row_loss;         // [T]
  int64_t ld;
  int32_t T, V, K, variant;
  float delta, loss_scale;
  int32_t mask_rule;        // 0 divergence (DPPO), 1 ratio clip (PPO/GRPO), 2 none
  float eps_low, eps_high;  // ratio-clip range
  float ratio_cap;          // C of the unified gradient form; 0 = no cap
  const uint16_t* mu_logits;  // bf16 bits [T, mu_ld]: the rollout policy's logits (full-vocabulary variants) or nullptr
  int64_t mu_ld;
  // Hidden-state path, forward only: there is no logits matrix; the logit of the row's sampled id is
  // gath[row * (K + 1)], that of its top-K entry k is gath[row * (K + 1) + 1 + k].  Else nullptr.
  const float* gath;
  // [T] log-prob of a_t under the policy the mask is anchored to, where that is not the rollout
  // policy (App. C.1, MiniRL; Sec. 5.2, decoupled objective), or nullptr: mu_logp.
  const float* anchor_logp;
  // Clip relaxation for low-probability tokens (Sec. 6; ratio-clip mask only): a token is one if
  // log mu(a_t) < relax_log_alpha (-infinity: none), and then the sides in relax_sides (1: upper,
  // 2: lower threshold) do not block.
  double relax_log_alpha;
  int32_t relax_sides;
};

// The subset of the kernel arguments the per-row epilogue needs.
struct EpiParams {
  const int32_t* tk_ids;
  const float* tk_lp;
  float* loss_tok;
  float* divergence;
  uint8_t* mask;
  float* diag;
  int32_t V, K, variant;
  float delta, loss_scale;
  int32_t mask_rule;
  float eps_low, eps_high, ratio_cap;
  const float* gath;
  const float* anchor_logp;
  double relax_log_alpha;
  int32_t relax_sides;
};
__device__ __forceinline__ EpiParams epi_params(const KParams& p) {
  EpiParams e;
  e.tk_ids = p.tk_ids; e.tk_lp = p.tk_lp; e.loss_tok = p.loss_tok; e.divergence = p.divergence; e.mask = p.mask; e.diag = p.diag;
  e.V = p.V; e.K = p.K; e.variant = p.variant; e.delta = p.delta; e.loss_scale = p.loss_scale;
  e.mask_rule = p.mask_rule; e.eps_low = p.eps_low; e.eps_high = p.eps_high; e.ratio_cap = p.ratio_cap;
  e.gath = p.gath;
  e.anchor_logp = p.anchor_logp;
  e.relax_log_alpha = p.relax_log_alpha;
  e.relax_sides = p.relax_sides;
  return e;
}

// What the per-row epilogue hands to the gradient pass.
struct RowCoef {
  float kexp;     // g_j = sgn * exp2(z_j*log2e + kexp) for j != a_t ; -inf-like when coef == 0
  float coef;     // c_t = loss_scale * M_t * A_t * r_t
  float g_a;      // gradient entry of the sampled token, c_t * (pi(a_t) - 1)
};
struct RowResult {
  RowCoef rc;
  double loss_term;   // -M_t r_t A_t
};

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// Round-to-nearest-even pack of two floats into two bf16 (lo in bits 0..15).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte vector = 8 bf16
// Buffer resource over one row: base address in scalar registers, byte range checked by the
// hardware (a load past `bytes` returns 0, a store past it is dropped), so a 16-byte access is
// addressed by one per-lane 32-bit offset plus a scalar offset and needs no address arithmetic
// in vector registers.
typedef __amdgpu_buffer_rsrc_t row_rsrc_t;
__device__ __forceinline__ row_rsrc_t make_row_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, static_cast<int>(bytes), 0x00020000);
}
// NT: marked non-temporal (the third bit pair of the cache policy: 2 = nt).
template <bool NT = false>
__device__ __forceinline__ u32x4 row_load16(row_rsrc_t r, uint32_t voff, uint32_t soff) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, NT ? 2 : 0);
}

// A 16-byte store to such a row issued from inline assembly, over a descriptor built by hand.  The compiler
// then does not count it among the pending vector-memory operations.  That matters where
// loads issued around such stores are waited for one by one: with stores and loads both
// pending the compiler falls back to waiting for everything (s_waitcnt vmcnt(0)), whereas loads
// alone complete in order and it waits for exactly the one it needs (vmcnt = number of loads
// issued after it, which stays correct however many stores are in flight).
// What the compiler no longer does for a store it cannot see, and the statement therefore does
// itself:
//  * BEFORE the store, five wait states (`s_nop 4`).  On this target a vector-memory instruction
//    must not read a scalar register within five wait states of a vector-ALU instruction writing
//    it, and the compiler restores spilled scalar registers with exactly such an instruction
//    (v_readlane_b32) wherever it likes, also directly in front of this statement, whose scalar
//    operands (descriptor, offset) it then believes to be ready.  Seen in the generated code of the
//    full-vocabulary kernel: the offset register reloaded one instruction ahead of the first store
//    of a row, and that store going to the address of a stale offset.
//  * AFTER it, two wait states (`s_nop 1`) before a vector-ALU instruction may overwrite the data
//    registers of a store of more than 8 bytes (the compiler's own rule for this target, in the
//    form with an immediate scalar offset; it covers the register form used here too).  A later
//    vector-memory load into the same registers queues behind the store and needs nothing.
// The store is marked non-temporal (a gradient row is not read again by this kernel): measured
// 2.5 % faster on the headline shape; the same mark on the row loads measured slower.
typedef int row_desc_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ row_desc_t make_row_desc(const void* base, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  row_desc_t d;
  d.x = __builtin_amdgcn_readfirstlane(static_cast<int>(a));
  d.y = __builtin_amdgcn_readfirstlane(static_cast<int>((a >> 32) & 0xffffu));
  d.z = __builtin_amdgcn_readfirstlane(static_cast<int>(bytes));
  d.w = 0x00020000;
  return d;
}
__device__ __forceinline__ void row_store16_untracked(row_desc_t d, uint32_t voff, uint32_t soff, u32x4 v) {
  asm volatile("s_nop 4\n\tbuffer_store_dwordx4 %0, %1, %2, %3 offen nt\n\ts_nop 1" ::"v"(v), "v"(voff), "s"(d), "s"(soff) : "memory");
}

// First row of a workgroup in a row-per-workgroup kernel whose rows advance by gridDim.x: a
// permutation of 0 .. gridDim.x-1 that gives the workgroups of one die (id % 8) neighbouring rows.
__device__ __forceinline__ int first_row_of_workgroup() {
  const unsigned g = gridDim.x, b = blockIdx.x;
  return static_cast<int>((g & 7u) == 0 ? (b & 7u) * (g >> 3) + (b >> 3) : b);
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
// t + e * x for e = 2^x, safe for x = -inf (where e = 0): the exponent is clamped first, and
// below the clamp e has long flushed to zero, so the product is unchanged.
__device__ __forceinline__ float fma_ex(float e, float x, float t) { return fmaf(e, fmaxf(x, -256.f), t); }

// Wave-wide reductions on the data-parallel-primitive path (no LDS crossbar): a butterfly inside
// each row of 16 lanes (quad permutes, then half-row and row mirrors), then the four row results
// are read as scalars.  Every lane returns the same value.
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) { return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false); }
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) { return __int_as_float(dpp_i<CTRL>(__float_as_int(v))); }
template <int CTRL>
__device__ __forceinline__ double dpp_d(double v) {
  return __hiloint2double(dpp_i<CTRL>(__double2hiint(v)), dpp_i<CTRL>(__double2loint(v)));
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f<kDppXor1>(v));
  v = fmaxf(v, dpp_f<kDppXor2>(v));
  v = fmaxf(v, dpp_f<kDppHalfMirror>(v));
  v = fmaxf(v, dpp_f<kDppMirror>(v));
  const int i = __float_as_int(v);
  return fmaxf(fmaxf(__int_as_float(__builtin_amdgcn_readlane(i, 0)), __int_as_float(__builtin_amdgcn_readlane(i, 16))),
               fmaxf(__int_as_float(__builtin_amdgcn_readlane(i, 32)), __int_as_float(__builtin_amdgcn_readlane(i, 48))));
}
__device__ __forceinline__ double wave_sum(double v) {
  v += dpp_d<kDppXor1>(v);
  v += dpp_d<kDppXor2>(v);
  v += dpp_d<kDppHalfMirror>(v);
  v += dpp_d<kDppMirror>(v);
  const int hi = __double2hiint(v), lo = __double2loint(v);
  const double r0 = __hiloint2double(__builtin_amdgcn_readlane(hi, 0), __builtin_amdgcn_readlane(lo, 0));
  const double r1 = __hiloint2double(__builtin_amdgcn_readlane(hi, 16), __builtin_amdgcn_readlane(lo, 16));
  const double r2 = __hiloint2double(__builtin_amdgcn_readlane(hi, 32), __builtin_amdgcn_readlane(lo, 32));
  const double r3 = __hiloint2double(__builtin_amdgcn_readlane(hi, 48), __builtin_amdgcn_readlane(lo, 48));
  return (r0 + r1) + (r2 + r3);
}

// Per-thread running statistics of a row, kept in the base-2 domain:
//   s = sum_j 2^(z_j*log2e + b)   with b an INTEGER-valued offset, b <= -max_j(z_j*log2e).
// Because b is an integer, changing it rescales s by an exact power of two, and offsets of
// different threads combine without any rounding.
// The sum itself is kept in float64: the exponentials of eight entries are summed among themselves
// in fp32 (pairwise) and that sum is added to the float64 accumulator, so that a thread that has
// met a dominant entry does not drop the thousands of small ones that follow it (in an fp32
// accumulator every term below half an ulp of the running sum vanishes: a bias of several 1e-7 on
// rows with a heavy tail).
__device__ __forceinline__ float sum8(const float (&e)[8]) {
  return ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]));
}
struct OnlineStat {
  float b = 3.0e38f;   // current offset (starts at "+infinity": nothing seen yet)
  double s = 0.0;      // sum 2^x,      x = z*log2e + b
  float t = 0.f;       // sum 2^x * x   (feeds the entropy)
  __device__ __forceinline__ void cover(float zmax) {   // make the offset cover a logit value
    const float bn = fminf(b, -ceilf(fmaxf(zmax, kNegBig) * kLog2e));
    const float d = bn - b, sc = fast_exp2(d);
    t = sc * fmaf(d, static_cast<float>(s), t);     // e -> e*2^d, x -> x + d
    s *= static_cast<double>(sc);
    b = bn;
  }
  __device__ __forceinline__ void add1(float z) {
    cover(z);
    const float x = fmaf(z, kLog2e, b), e = fast_exp2(x);
    s += static_cast<double>(e);
    t = fma_ex(e, x, t);
  }
  __device__ __forceinline__ void add8(const float (&z)[8]) {
    cover(fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])), fmaxf(fmaxf(z[4], z[5]), fmaxf(z[6], z[7]))));
    float e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float x = fmaf(z[i], kLog2e, b);
      e[i] = fast_exp2(x);
      t = fma_ex(e[i], x, t);
    }
    s += static_cast<double>(sum8(e));
  }
};

__device__ __forceinline__ void unpack8(const u32x4& v, float (&z)[8]) {
  z[0] = __uint_as_float(v.x << 16); z[1] = __uint_as_float(v.x & 0xffff0000u);
  z[2] = __uint_as_float(v.y << 16); z[3] = __uint_as_float(v.y & 0xffff0000u);
  z[4] = __uint_as_float(v.z << 16); z[5] = __uint_as_float(v.z & 0xffff0000u);
  z[6] = __uint_as_float(v.w << 16); z[7] = __uint_as_float(v.w & 0xffff0000u);
}

// The same for the ROLLOUT policy's row y, with the cross term the exact KL needs:
//   s = sum_j 2^(y_j*log2e + b),   u = sum_j 2^(y_j*log2e + b) * (y_j - z_j)   (natural units),
// so that sum_j mu_j (y_j - z_j) = u / s whatever the offset.  A vanished term (y_j = -inf)
// adds nothing even where z_j = -inf too; a token pi excludes (z_j = -inf) that mu can still
// sample makes u infinite, as the divergence then is.
struct CrossStat {
  float b = 3.0e38f, u = 0.f;
  double s = 0.0;
  __device__ __forceinline__ void cover(float ymax) {
    const float bn = fminf(b, -ceilf(fmaxf(ymax, kNegBig) * kLog2e));
    const float sc = fast_exp2(bn - b);
    s *= static_cast<double>(sc);
    u *= sc;
    b = bn;
  }
  __device__ __forceinline__ float term(float y, float z) {
    const float e = fast_exp2(fmaf(y, kLog2e, b));
    const float d = fminf(fmaxf(y - z, -3.0e38f), 3.0e38f);     // NaN (-inf - -inf) -> -3e38, times e = 0
    u = fmaf(e, d, u);
    return e;
  }
  __device__ __forceinline__ void add1(float y, float z) {
    cover(y);
    s += static_cast<double>(term(y, z));
  }
  __device__ __forceinline__ void add8(const float (&y)[8], const float (&z)[8]) {
    cover(fmaxf(fmaxf(fmaxf(y[0], y[1]), fmaxf(y[2], y[3])), fmaxf(fmaxf(y[4], y[5]), fmaxf(y[6], y[7]))));
    float e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = term(y[i], z[i]);
    s += static_cast<double>(sum8(e));
  }
};

// ---- scalar math for the per-row epilogue ----------------------------------------------------
// The epilogue runs once per row on one wave while the rest of the workgroup waits.  Everything a
// per-token output is formed from (the K + 2 probabilities, the two or three logarithms, every sum
// or difference that could cancel) is evaluated in float64: exp2_d / log2_d below are good to about
// 1e-15, so what is left on a probability is the relative error of the fp32 row sum (about 1e-8).
// The single-instruction fp32 forms (exp2_split, log2_fast; about 1 ulp of fp32) remain for
// quantities that are rounded to bf16 afterwards (the gradient's exponent).

constexpr double kLn2 = 0.6931471805599453;
constexpr double kLog2eD = 1.4426950408889634;
constexpr double kLnTiny = -69.07755278982137;   // ln(1e-30): floor of a vanishing denominator

// 2^x for a float64 argument, returned in fp32 (0 for x below the fp32 range).
__device__ __forceinline__ float exp2_split(double x) {
  if (!(x > -200.0)) return 0.f;
  const double n = __builtin_rint(x);
  const float f = static_cast<float>(x - n);            // |f| <= 0.5
  return ldexpf(fast_exp2(f), static_cast<int>(n));
}

// log2(x) for a positive finite float64 x, absolute error about 1.5e-7.
__device__ __forceinline__ double log2_fast(double x) {
  const int e = __builtin_amdgcn_frexp_exp(x);
  const float m = static_cast<float>(__builtin_amdgcn_frexp_mant(x));   // [0.5, 1)
  return static_cast<double>(e) + static_cast<double>(__builtin_amdgcn_logf(m));
}

// 2^x in float64 (0 below the float64 range, +inf above it): x = n + f with |f| <= 1/2, and
// 2^f = exp(f ln 2) by the Taylor polynomial of degree 12 (|f ln 2| <= 0.347: truncation below
// 1e-16 relative), then scaled by 2^n.  Horner form on purpose: every step then has ONE constant
// operand, which the instruction can take from scalar registers; a pairwise (Estrin) evaluation is
// five steps deep instead of twelve but needs two constants per step, i.e. a dozen constants in
// vector registers, which the compiler keeps for the whole kernel and, beside a resident row, spills.
// kconst() pins a constant to scalar registers at its point of use (left to itself the compiler
// builds float64 constants in vector registers once, at the top of the kernel, and spills them).
__device__ __forceinline__ double kconst(double c) {
  asm volatile("" : "+s"(c));
  return c;
}
__device__ __forceinline__ double exp2_d(double x) {
  if (!(x > -1080.0)) return 0.0;
  if (x > 1024.0) return __builtin_inf();
  const double n = __builtin_rint(x);
  const double t = (x - n) * kconst(kLn2);
  double p = kconst(1.0 / 479001600);
  p = fma(p, t, kconst(1.0 / 39916800));
  p = fma(p, t, kconst(1.0 / 3628800));
  p = fma(p, t, kconst(1.0 / 362880));
  p = fma(p, t, kconst(1.0 / 40320));
  p = fma(p, t, kconst(1.0 / 5040));
  p = fma(p, t, kconst(1.0 / 720));
  p = fma(p, t, kconst(1.0 / 120));
  p = fma(p, t, kconst(1.0 / 24));
  p = fma(p, t, kconst(1.0 / 6));
  p = fma(p, t, 0.5);
  p = fma(p, t, 1.0);
  p = fma(p, t, 1.0);
  return ldexp(p, static_cast<int>(n));
}

// log2(x) in float64 for a positive finite x: the hardware's fp32 logarithm of the mantissa as a
// first guess y0 (about 1e-7), then one Newton step on 2^y = m: m 2^-y0 = 1 + d with |d| ~ 1e-7,
// and log2(1 + d) = (d - d^2/2) log2(e) up to d^3.
__device__ __forceinline__ double log2_d(double x) {
  const int e = __builtin_amdgcn_frexp_exp(x);
  const double m = __builtin_amdgcn_frexp_mant(x);                      // [0.5, 1)
  const double y0 = static_cast<double>(__builtin_amdgcn_logf(static_cast<float>(m)));
  const double d = fma(m, exp2_d(-y0), -1.0);
  return static_cast<double>(e) + fma(d * fma(-0.5, d, 1.0), kLog2eD, y0);
}

// x * (ln x - max(ln y, ln 1e-30)) with 0 ln 0 = 0; the logarithms are passed in.
__device__ __forceinline__ double xlogx_over_y(double x, double ln_x, double ln_y) {
  return (x > 0.0) ? x * (ln_x - fmax(ln_y, kLnTiny)) : 0.0;
}

// 1 - exp(t) for t <= 0 in float64, accurate when t -> 0.
__device__ __forceinline__ double one_minus_exp(double t, double exp_t) {
  if (t > -0.0625) {
    const double u = t * (1.0 + t * (0.5 + t * (1.0 / 6 + t * (1.0 / 24 + t * (1.0 / 120 + t * (1.0 / 720))))));
    return -u;
  }
  return 1.0 - exp_t;
}

// Per-row inputs the epilogue needs besides the row statistics.  The kernels fetch them early
// in the row so that no memory latency is left on the epilogue's critical path.
struct RowScalars {
  int a;        // sampled id (valid: 0 <= a < V)
  float za;     // z[a_t]
  float lmu;    // log mu(a_t): the importance ratio r = pi / mu
  float adv;    // A_t
  float lanc;   // log-prob of a_t under the mask's anchor policy (= lmu unless the caller gave one)
};
// The three per-row scalars of the epilogue in ONE vector register, for kernels that hold them
// across a whole row beside a resident row: lane 0 requests log mu(a_t), lane 1 the advantage, lane 2
// the anchor's log-prob (the rollout policy's again if the caller gave none).  unpack_row_scalars
// hands them out when the epilogue starts.
template <typename P>
__device__ __forceinline__ float load_row_scalars(const P& p, int row, int lane) {
  const float* src = (lane == 0) ? p.mu_logp : (lane == 1) ? p.adv : (p.anchor_logp ? p.anchor_logp : p.mu_logp);
  return (lane < 3) ? src[row] : 0.f;
}
// The anchor's log-prob of a row's sampled token: the caller's, else the rollout policy's.
template <typename P>
__device__ __forceinline__ float anchor_or(const P& p, int row, float lmu) {
  return p.anchor_logp ? p.anchor_logp[row] : lmu;
}
__device__ __forceinline__ void unpack_row_scalars(float packed, RowScalars& rs) {
  const int v = __float_as_int(packed);
  rs.lmu = __int_as_float(__builtin_amdgcn_readlane(v, 0));
  rs.adv = __int_as_float(__builtin_amdgcn_readlane(v, 1));
  rs.lanc = __int_as_float(__builtin_amdgcn_readlane(v, 2));
}
struct TopkLane {   // lane k holds top-K entry k (k < 64); id < 0 marks "no entry"
  int id;
  float lp;     // log mu(id)
  float z;      // z[id]
};

template <typename P>
__device__ __forceinline__ TopkLane load_topk_lane(const P& p, int row, int a, const uint16_t* zrow, int lane) {
  TopkLane t;
  t.id = -1; t.lp = 0.f; t.z = 0.f;
  if (lane < p.K) {
    const int id = p.tk_ids[static_cast<int64_t>(row) * p.K + lane];
    if (id >= 0 && id < p.V && id != a) {
      t.id = id;
      t.lp = p.tk_lp[static_cast<int64_t>(row) * p.K + lane];
      t.z = p.gath ? p.gath[static_cast<int64_t>(row) * (p.K + 1) + 1 + lane] : bf16_bits_to_float(zrow[id]);
    }
  }
  return t;
}

// ---- the per-row epilogue, in two parts -------------------------------------------------------
// Executed by ONE full wave (all 64 lanes call both parts with the same scalars; lane k carries
// top-K entry k).  The row statistics arrive in the base-2 domain the streaming passes work in:
//   b      : offset (an integer-valued float) with z_j*log2e + b <= 0 for every j
//   S_rest : sum over j != a_t of 2^(z_j*log2e + b).  The sampled token's own term is left out
//            so that 1 - pi(a_t) = S_rest / S keeps full relative accuracy when pi(a_t) -> 1.
//   T_rest : sum over j != a_t of 2^(x_j) * x_j with x_j = z_j*log2e + b (for the entropy:
//            sum_j pi_j log2 pi_j = T/S - log2 S).
// log2e is the fp32 constant kLog2e everywhere (passes and epilogue), so the probabilities
// are mutually consistent; its rounding (1.3e-8 relative) acts as a temperature of 1+1.3e-8.
//
// row_pre  needs only the row's INPUTS (z[a_t], log mu(a_t), the lane's top-K entry), not its
//          statistics: every exponential of the epilogue is taken here, as mantissa and integer
//          exponent where the offset b is still to come (b is an integer: 2^(x + b) is an ldexp).
//          A kernel that has those inputs early runs it in the shadow of the row's memory latency.
// row_post needs the statistics: one logarithm and one reciprocal (two more logarithms for the KL
//          forms), then ratio (Eq. ppo-clip), divergence (Eq. binary_tv / binary_kl / topk_tv /
//          topk_kl), mask and loss term (Eq. dppo_obj), gradient coefficient (Eq. unified_grad).
//          It is the part the rest of the workgroup waits for.
// row_store writes the per-token outputs (lane 0).
// D_full : the exact full-vocabulary divergence, for the variants that gate on it (App. B).

// 2^x = m * 2^n with n = rint(x) and m = 2^(x - n) in [2^-1/2, 2^1/2]; x <= about -1e6 (or NaN)
// gives m = 0, n = 0.
struct Exp2Parts {
  double m;
  int n;
};
__device__ __forceinline__ Exp2Parts exp2_parts(double x) {
  Exp2Parts r;
  if (!(x > -1.0e6)) { r.m = 0.0; r.n = 0; return r; }
  const double xc = fmin(x, 1.0e6);
  const double n = __builtin_rint(xc);
  r.m = exp2_d(xc - n);
  r.n = static_cast<int>(n);
  return r;
}
// m * 2^(n + b) for an integer-valued float b of any magnitude.
__device__ __forceinline__ double scale_parts(Exp2Parts p, float b) {
  const double e = fmin(fmax(static_cast<double>(p.n) + static_cast<double>(b), -4000.0), 4000.0);
  return ldexp(p.m, static_cast<int>(e));
}

struct RowPre {
  // uniform over the wave
  Exp2Parts ea;        // 2^(z[a_t]*log2e)
  double xa0;          // z[a_t]*log2e
  double pa;           // p(a_t) = exp(min(log p(a_t), 0)), p the mask's anchor policy (mu unless given)
  double inv_pa_raw;   // exp(-log mu(a_t)), for r = pi(a_t) / mu(a_t)
  double lmu, lmu_raw; // min(log p(a_t), 0) and log p(a_t) as given
  double A;            // advantage
  bool low;            // a low-probability token of the clip relaxation: log mu(a_t) of the rollout policy < log alpha
  // of this lane's top-K entry (valid: the entry exists and is not a_t)
  bool valid;
  Exp2Parts ek;        // 2^(z[id]*log2e)
  double xk0;          // z[id]*log2e
  double pk, lpk;      // mu(id) and min(log mu(id), 0)
};

__device__ __forceinline__ RowPre row_pre(RowScalars rs, TopkLane tk, bool topk, double relax_log_alpha) {
  constexpr double kL = static_cast<double>(kLog2e);
  RowPre q;
  q.xa0 = static_cast<double>(rs.za) * kL;
  q.ea = exp2_parts(q.xa0);
  q.lmu_raw = static_cast<double>(rs.lanc);
  q.lmu = fmin(q.lmu_raw, 0.0);
  q.pa = exp2_d(q.lmu * kLog2eD);
  q.low = static_cast<double>(rs.lmu) < relax_log_alpha;
  q.inv_pa_raw = exp2_d(-static_cast<double>(rs.lmu) * kLog2eD);
  q.A = static_cast<double>(rs.adv);
  q.valid = topk && tk.id >= 0;
  q.xk0 = 0.0; q.pk = 0.0; q.lpk = 0.0;
  q.ek.m = 0.0; q.ek.n = 0;
  if (q.valid) {
    q.lpk = fmin(static_cast<double>(tk.lp), 0.0);
    q.pk = exp2_d(q.lpk * kLog2eD);
    q.xk0 = static_cast<double>(tk.z) * kL;
    q.ek = exp2_parts(q.xk0);
  }
  return q;
}

// What row_post leaves for row_store.
struct RowOut {
  float D, lt, r, lpi, abs_diff, H, mass_mu, mass_pi;
  bool blocked;
};

// log2 of two positive values at once: lane 0 evaluates the first, every other lane the second.
__device__ __forceinline__ void log2_pair(double x0, double x1, int lane, double& l0, double& l1) {
  const double l = log2_d(lane == 0 ? x0 : x1);
  const int hi = __double2hiint(l), lo = __double2loint(l);
  l0 = __hiloint2double(__builtin_amdgcn_readlane(hi, 0), __builtin_amdgcn_readlane(lo, 0));
  l1 = __hiloint2double(__builtin_amdgcn_readlane(hi, 1), __builtin_amdgcn_readlane(lo, 1));
}

template <typename P>
__device__ __forceinline__ RowResult row_post(const P& p, int row, const RowPre& q, int a, const uint16_t* zrow, float b, double S_rest,
                                              double T_rest, int lane, double D_full, RowOut& o) {
  constexpr double kL = static_cast<double>(kLog2e);
  const double bd = static_cast<double>(b);
  const double ea = scale_parts(q.ea, b);
  const double S = S_rest + ea;
  const double inv_S = 1.0 / S;
  const double log2S = log2_d(S);
  const double xa = q.xa0 + bd;
  const double lpi = (xa - log2S) * kLn2;
  const double pa = q.pa, qa = ea * inv_S;
  const double one_minus_qa = S_rest * inv_S;
  const int variant = p.variant;
  double mass_mu = pa, mass_pi = qa;      // mass on A' (= {a_t} for the Binary variants)
  double D;
  if (variant == kFullTV || variant == kFullKL) {
    D = D_full;                           // exact divergence of the two rows (App. B), computed by the caller
    mass_mu = 1.0;
    mass_pi = 1.0;
  } else if (variant == kBinaryTV || (variant == kTopkTV && p.K == 0)) {
    D = fabs(pa - qa);
  } else if (variant == kBinaryKL || (variant == kTopkKL && p.K == 0)) {
    const double omp = one_minus_exp(q.lmu, pa);
    double l_omp, l_omq;
    log2_pair(fmax(omp, 1e-300), fmax(one_minus_qa, 1e-300), lane, l_omp, l_omq);
    D = xlogx_over_y(pa, q.lmu, lpi) + xlogx_over_y(omp, l_omp * kLn2, l_omq * kLn2);
  } else {
    // reduced distributions over TopK(mu, K) U {a_t} U {other}  (Sec. 4.4)
    const bool tv = (variant == kTopkTV);
    double sp = 0.0, sq = 0.0, acc = 0.0;
    if (q.valid) {
      const double qk = scale_parts(q.ek, b) * inv_S;
      sp = q.pk;
      sq = qk;
      acc = tv ? fabs(q.pk - qk) : xlogx_over_y(q.pk, q.lpk, (q.xk0 + bd - log2S) * kLn2);
    }
    for (int k = lane + kWave; k < p.K; k += kWave) {      // K > 64: further entries, fetched and evaluated here
      const TopkLane t = load_topk_lane(p, row, a, zrow, k);
      if (t.id >= 0) {
        const double lpk = fmin(static_cast<double>(t.lp), 0.0);
        const double xk = static_cast<double>(t.z) * kL + bd - log2S;     // log2 pi(id)
        const double pk = exp2_d(lpk * kLog2eD), qk = exp2_d(xk);
        sp += pk;
        sq += qk;
        acc += tv ? fabs(pk - qk) : xlogx_over_y(pk, lpk, xk * kLn2);
      }
    }
    sp = wave_sum(sp) + pa;
    sq = wave_sum(sq) + qa;
    mass_mu = sp;
    mass_pi = sq;
    acc = wave_sum(acc) + (tv ? fabs(pa - qa) : xlogx_over_y(pa, q.lmu, lpi));
    const double po = fmax(1.0 - sp, 0.0), qo = fmax(1.0 - sq, 0.0);
    if (tv) {
      D = 0.5 * (acc + fabs(po - qo));
    } else {
      double l_po, l_qo;
      log2_pair(fmax(po, 1e-300), fmax(qo, 1e-300), lane, l_po, l_qo);
      D = acc + xlogx_over_y(po, l_po * kLn2, l_qo * kLn2);
    }
  }
  const double A = q.A;
  // mask M_t: DPPO's divergence mask (Eq. dppo_obj), or one of the baselines' (App. C.1)
  bool blocked;
  if (p.mask_rule == 0) {
    blocked = (D > static_cast<double>(p.delta)) && ((A > 0.0 && lpi > q.lmu_raw) || (A < 0.0 && lpi < q.lmu_raw));
  } else if (p.mask_rule == 1) {
    const double dl = lpi - q.lmu_raw;     // log r, compared with log(1 + eps_high) and log(1 - eps_low)
    // Sec. 6: for tokens the rollout policy gave less than alpha, the named thresholds are infinite
    const bool hi_on = !(q.low && (p.relax_sides & 1)), lo_on = !(q.low && (p.relax_sides & 2));
    blocked = (A > 0.0 && hi_on && dl > log1p(static_cast<double>(p.eps_high))) ||
              (A < 0.0 && lo_on && dl < log1p(-static_cast<double>(p.eps_low)));
  } else {
    blocked = false;
  }
  const double M = blocked ? 0.0 : 1.0;
  const double r = qa * q.inv_pa_raw;
  // weight min(r, C) of the unified gradient form (Eq. unified_grad); no cap for DPPO
  const double w = (p.ratio_cap > 0.f && r > static_cast<double>(p.ratio_cap)) ? static_cast<double>(p.ratio_cap) : r;
  const double lt = -M * w * A;
  const double c = static_cast<double>(p.loss_scale) * M * A * w;
  o.D = static_cast<float>(D);
  o.blocked = blocked;
  o.lt = static_cast<float>(lt);
  o.r = static_cast<float>(r);
  o.lpi = static_cast<float>(lpi);
  o.abs_diff = static_cast<float>(fabs(pa - qa));
  o.mass_mu = static_cast<float>(mass_mu);
  o.mass_pi = static_cast<float>(mass_pi);
  o.H = 0.f;
  if (p.diag) {
    // token entropy: -sum pi ln pi = ln2 * (log2 S - T/S), T including a_t's own term
    const double T = T_rest + ((ea > 0.0) ? ea * xa : 0.0);
    o.H = static_cast<float>(fmax(kLn2 * (log2S - T * inv_S), 0.0));
  }
  RowResult res;
  res.loss_term = lt;
  res.rc.coef = static_cast<float>(c);
  res.rc.g_a = static_cast<float>(-c * one_minus_qa);
  // c * pi_j = sgn(c) * 2^(z_j*log2e + kexp)
  res.rc.kexp = (c != 0.0 && fabs(c) < 1e300) ? static_cast<float>(log2_fast(fabs(c)) + bd - log2S) : 0.f;
  return res;
}

template <typename P>
__device__ __forceinline__ void row_store(const P& p, int row, const RowOut& o, int lane) {
  if (lane == 0) {
    p.divergence[row] = o.D;
    p.mask[row] = o.blocked ? 0 : 1;
    if (p.loss_tok) p.loss_tok[row] = o.lt;
    if (p.diag) {
      typedef float f32x4 __attribute__((ext_vector_type(4)));
      f32x4* d = reinterpret_cast<f32x4*>(p.diag + static_cast<int64_t>(row) * 8);
      d[0] = f32x4{o.r, o.lpi, o.abs_diff, o.H};
      d[1] = f32x4{o.mass_mu, o.mass_pi, 0.f, 0.f};
    }
  }
}

// Both parts and the stores back to back, for the kernels that have nothing to hide the first
// part behind.  Every lane returns the same RowResult.
__device__ __forceinline__ RowResult row_epilogue(const EpiParams& p, int row, RowScalars rs, TopkLane tk,
                                                  const uint16_t* zrow, float b, double S_rest, double T_rest, int lane,
                                                  double D_full = 0.0) {
  const bool topk = (p.variant == kTopkTV || p.variant == kTopkKL) && p.K > 0;
  const RowPre q = row_pre(rs, tk, topk, p.relax_log_alpha);
  RowOut o;
  const RowResult res = row_post(p, row, q, rs.a, zrow, b, S_rest, T_rest, lane, D_full, o);
  row_store(p, row, o, lane);
  return res;
}

// The same epilogue as a real call.  Its float64 arithmetic needs many registers; where
// several workgroups share a compute unit, keeping those out of the kernel's register budget
// (the call saves and restores what it needs, in the one wave that makes it) buys occupancy,
// and the other workgroups hide the call's latency.
__device__ __attribute__((noinline)) static RowResult row_epilogue_call(const EpiParams& p, int row, RowScalars rs, TopkLane tk,
                                                                        const uint16_t* zrow, float b, double S_rest, double T_rest,
                                                                        int lane, double D_full = 0.0) {
  return row_epilogue(p, row, rs, tk, zrow, b, S_rest, T_rest, lane, D_full);
}

}  // namespace dppo
