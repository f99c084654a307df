// Register-resident fused forward+backward kernel.
//
// One persistent workgroup per compute unit owns one row at a time and keeps the whole bf16
// row packed in its vector registers (V = 151936 is 297 KiB; a CU's register file is 512 KiB),
// so the logits are read from HBM exactly once and the gradient written exactly once:
//
//   phase A  packed-integer maximum over the resident row            (no unpacking)
//   phase B  sum of 2^(z*log2e + b) in fp32 with a per-wave integer offset b
//            -> one LDS exchange + barrier -> per-token epilogue on wave 0 -> barrier
//   phase C  gradient of every resident element, 16-byte non-temporal stores; as each
//            register chunk is consumed it is refilled with the same chunk of the workgroup's
//            NEXT row, so HBM reads of row r+1 overlap the arithmetic and writes of row r.
//
// Preconditions (checked by the host): V % 8 == 0, V/8 <= THREADS*NCHUNK, logits and
// grad_logits 16-byte aligned with ld % 8 == 0.
#include "dppo_common.hpp"
#include "dppo_launch.hpp"

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

// Phase C for one row: write the gradient of every resident chunk and (MORE) refill the chunk
// with the workgroup's next row.  ZERO rows (masked, zero advantage, ignored) store zeros.
template <int THREADS, int NCHUNK, bool ZERO, bool MORE>
__device__ __forceinline__ void phase_c(u32x4 (&buf)[NCHUNK], int cnt, uint32_t voff, gbyte_ptr grow, gbyte_cptr znext,
                                        float kexp, uint32_t sgn) {
  constexpr uint32_t kStride = THREADS * 16u;   // bytes between a thread's consecutive chunks
#pragma unroll
  for (int i = 0; i < NCHUNK; ++i) {
    if (i < cnt) {
      u32x4 o = {0u, 0u, 0u, 0u};
      if (!ZERO) {
        const uint32_t w[4] = {buf[i].x, buf[i].y, buf[i].z, buf[i].w};
        uint32_t r[4];
#pragma unroll
        for (int d = 0; d < 4; ++d)
          r[d] = pack_bf16x2(fast_exp2(fmaf(__uint_as_float(w[d] << 16), kLog2e, kexp)),
                             fast_exp2(fmaf(__uint_as_float(w[d] & 0xffff0000u), kLog2e, kexp))) ^ sgn;
        o = u32x4{r[0], r[1], r[2], r[3]};
      }
      gstore16_nt(grow + i * kStride, voff, o);
      if (MORE) buf[i] = gload16(znext + i * kStride, voff);
    }
  }
}

template <int THREADS, int NCHUNK>
__global__ __launch_bounds__(THREADS) void dppo_resident_kernel(const KParams p) {
  static_assert(NCHUNK <= 40, "the chunk switch below is written out for up to 40 chunks");
  constexpr int NW = THREADS / kWave;
  constexpr uint32_t kStride = THREADS * 16u;
  __shared__ float sh_b[NW];
  __shared__ double sh_s[NW];
  __shared__ RowCoef sh_rc;
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wid = uniform_i(tid / kWave);
  const int nvec = p.V >> 3;
  // Thread tid owns vectors tid, tid+THREADS, ...: `cnt` of them (chunk i <-> vector i*THREADS+tid).
  const int cnt = (nvec - tid + THREADS - 1) / THREADS;
  const uint32_t voff = static_cast<uint32_t>(tid) * 16u;
  const u32x4 neg_inf = {kNegInfPair, kNegInfPair, kNegInfPair, kNegInfPair};
  const int64_t pitch = p.ld * 2;               // row pitch in bytes
  const gbyte_cptr logits = (gbyte_cptr)p.logits;
  const gbyte_ptr grad = (gbyte_ptr)p.grad;
  double loss_acc = 0.0;                        // meaningful in wave 0 only

  // The resident row.  Slots past the row hold -inf for the whole kernel: they add nothing.
  u32x4 buf[NCHUNK];
  int row = blockIdx.x;
  {
    const gbyte_cptr zr = logits + row * pitch;
#pragma unroll
    for (int i = 0; i < NCHUNK; ++i) {
      buf[i] = neg_inf;
      if (i < cnt) buf[i] = gload16(zr + i * kStride, voff);
    }
  }

  for (; row < p.T; row += gridDim.x) {
    const int a = uniform_i(p.sampled[row]);
    const bool live = (a >= 0 && a < p.V);
    const gbyte_cptr zr = logits + row * pitch;
    const uint16_t* zrow = p.logits + static_cast<int64_t>(row) * p.ld;
    const int avec = a >> 3;
    const int ia = live ? avec / THREADS : -1;               // chunk holding a_t (uniform)
    const bool owner = live && (avec - ia * THREADS == tid);
    const int sub = a & 7;

    RowCoef rc;
    rc.coef = 0.f; rc.kexp = 0.f; rc.g_a = 0.f;
    if (live) {
      // The sampled token's own term is left out of the sum (see row_epilogue): overwrite it
      // with -inf in the resident copy; the epilogue reads z[a_t] from memory.  `ia` is uniform,
      // so this is one scalar jump, not a test per chunk.
#define DPPO_PATCH_CASE(I) case I: if (I < NCHUNK && owner) buf[I < NCHUNK ? I : 0] = patch16(buf[I < NCHUNK ? I : 0], sub, 0xFF80u); break;
#define DPPO_PATCH_CASES10(B) DPPO_PATCH_CASE(B + 0) DPPO_PATCH_CASE(B + 1) DPPO_PATCH_CASE(B + 2) DPPO_PATCH_CASE(B + 3) \
  DPPO_PATCH_CASE(B + 4) DPPO_PATCH_CASE(B + 5) DPPO_PATCH_CASE(B + 6) DPPO_PATCH_CASE(B + 7) DPPO_PATCH_CASE(B + 8) DPPO_PATCH_CASE(B + 9)
      switch (ia) {
        DPPO_PATCH_CASES10(0) DPPO_PATCH_CASES10(10) DPPO_PATCH_CASES10(20) DPPO_PATCH_CASES10(30)
        default: break;
      }
#undef DPPO_PATCH_CASES10
#undef DPPO_PATCH_CASE

      // ---- phase A: maximum, on the packed bf16 patterns --------------------------------
      // As signed 16-bit integers, non-negative bf16 order like floats and every negative one
      // is below them, so the integer maximum is the float maximum whenever it is >= 0.
      s16x2 mx = as_s16x2(0x80008000u);
#pragma unroll
      for (int i = 0; i < NCHUNK; ++i) {
        mx = __builtin_elementwise_max(mx, as_s16x2(buf[i].x));
        mx = __builtin_elementwise_max(mx, as_s16x2(buf[i].y));
        mx = __builtin_elementwise_max(mx, as_s16x2(buf[i].z));
        mx = __builtin_elementwise_max(mx, as_s16x2(buf[i].w));
      }
      int m16 = max(static_cast<int>(mx.x), static_cast<int>(mx.y));
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) m16 = max(m16, __shfl_xor(m16, o, kWave));
      m16 = uniform_i(m16);
      float wmax;
      if (m16 >= 0) {
        wmax = __uint_as_float(static_cast<uint32_t>(m16) << 16);
      } else {
        // Every entry of this wave's share is negative (or -inf).  Among negative bf16 the
        // float maximum has the smallest magnitude, i.e. the smallest signed 16-bit pattern.
        s16x2 mn = as_s16x2(0xFFFFFFFFu);
#pragma unroll
        for (int i = 0; i < NCHUNK; ++i) {
          mn = __builtin_elementwise_min(mn, as_s16x2(buf[i].x));
          mn = __builtin_elementwise_min(mn, as_s16x2(buf[i].y));
          mn = __builtin_elementwise_min(mn, as_s16x2(buf[i].z));
          mn = __builtin_elementwise_min(mn, as_s16x2(buf[i].w));
        }
        int n16 = min(static_cast<int>(mn.x), static_cast<int>(mn.y));
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) n16 = min(n16, __shfl_xor(n16, o, kWave));
        wmax = __uint_as_float(static_cast<uint32_t>(uniform_i(n16)) << 16);
      }
      // per-wave integer offset; it must also cover z[a_t] for the epilogue
      const float za = uniform_f(bf16_bits_to_float(((gu16_cptr)zrow)[a]));
      const float b = -ceilf(fmaxf(fmaxf(wmax, za), kNegBig) * kLog2e);

      // ---- phase B: sum of exponentials --------------------------------------------------
      float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
      for (int i = 0; i < NCHUNK; ++i) {
        const uint32_t w[4] = {buf[i].x, buf[i].y, buf[i].z, buf[i].w};
        s0 += fast_exp2(fmaf(__uint_as_float(w[0] << 16), kLog2e, b)) + fast_exp2(fmaf(__uint_as_float(w[0] & 0xffff0000u), kLog2e, b));
        s1 += fast_exp2(fmaf(__uint_as_float(w[1] << 16), kLog2e, b)) + fast_exp2(fmaf(__uint_as_float(w[1] & 0xffff0000u), kLog2e, b));
        s2 += fast_exp2(fmaf(__uint_as_float(w[2] << 16), kLog2e, b)) + fast_exp2(fmaf(__uint_as_float(w[2] & 0xffff0000u), kLog2e, b));
        s3 += fast_exp2(fmaf(__uint_as_float(w[3] << 16), kLog2e, b)) + fast_exp2(fmaf(__uint_as_float(w[3] & 0xffff0000u), kLog2e, b));
      }
      const double sw = wave_sum(static_cast<double>(s0 + s1) + static_cast<double>(s2 + s3));
      if (lane == 0) { sh_b[wid] = b; sh_s[wid] = sw; }
      __syncthreads();
      // ---- epilogue on wave 0 -----------------------------------------------------------
      if (wid == 0) {
        float bb = sh_b[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) bb = fminf(bb, sh_b[w]);
        double S_rest = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w) S_rest += sh_s[w] * static_cast<double>(fast_exp2(bb - sh_b[w]));   // exact powers of two
        double lt;
        rc = row_epilogue(p, row, a, zrow, bb, S_rest, lane, &lt);
        loss_acc += lt;
        if (lane == 0) sh_rc = rc;
      }
      __syncthreads();
      rc.coef = uniform_f(sh_rc.coef);
      rc.kexp = uniform_f(sh_rc.kexp);
      rc.g_a = uniform_f(sh_rc.g_a);
    } else if (tid == 0) {
      p.divergence[row] = 0.f;
      p.mask[row] = 0;
      if (p.loss_tok) p.loss_tok[row] = 0.f;
    }

    // ---- phase C: gradient out, next row in -------------------------------------------------
    const gbyte_ptr gr = grad + row * pitch;
    const int next = row + gridDim.x;
    const bool more = next < p.T;
    const gbyte_cptr zn = logits + (more ? next : row) * pitch;
    const uint32_t sgn = (rc.coef < 0.f) ? 0x80008000u : 0u;
    if (rc.coef == 0.f) {
      if (more) phase_c<THREADS, NCHUNK, true, true>(buf, cnt, voff, gr, zn, 0.f, 0u);
      else      phase_c<THREADS, NCHUNK, true, false>(buf, cnt, voff, gr, zn, 0.f, 0u);
    } else {
      if (more) phase_c<THREADS, NCHUNK, false, true>(buf, cnt, voff, gr, zn, rc.kexp, sgn);
      else      phase_c<THREADS, NCHUNK, false, false>(buf, cnt, voff, gr, zn, rc.kexp, sgn);
      // The resident copy holds -inf at a_t, so the vector store above wrote 0 there.  Once
      // that store has completed, the owning thread writes the sampled token's entry.
      if (owner) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        ((gu16_ptr)(gr))[a] = float_to_bf16_bits(rc.g_a);
      }
    }
  }
  if (tid == 0) p.partial[blockIdx.x] = loss_acc;
}

}  // namespace

hipError_t launch_resident(const KParams& p, int threads, int grid, hipStream_t s) {
  if (threads == 512) hipLaunchKernelGGL((dppo_resident_kernel<512, kResidentChunksBig>), dim3(grid), dim3(512), 0, s, p);
  else                hipLaunchKernelGGL((dppo_resident_kernel<256, kResidentChunksSmall>), dim3(grid), dim3(256), 0, s, p);
  return hipGetLastError();
}

int resident_blocks_per_cu(int threads) {
  int n = 0;
  hipError_t e = (threads == 512)
      ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dppo_resident_kernel<512, kResidentChunksBig>, 512, 0)
      : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dppo_resident_kernel<256, kResidentChunksSmall>, 256, 0);
  return (e == hipSuccess && n > 0) ? n : 1;
}

}  // namespace dppo
