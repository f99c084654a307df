// Trust region on the EXACT full-vocabulary divergence (App. B), register-resident form (the
// backward of both variants, and the forward-only TV form): total variation 1/2 sum_j |mu_j - pi_j| or KL(mu || pi) = sum_j mu_j ln(mu_j / pi_j)
// between the rollout policy's and the trainer's next-token distributions, both given as rows of
// bf16 logits, and the gradient of the masked surrogate over the trainer's row.
//
// One persistent workgroup of 512 threads per compute unit owns one row at a time.  The trainer
// row z stays packed in its vector registers (as in the register-resident loss kernel: V = 151936
// is 297 KiB of a compute unit's 512 KiB register file), the rollout row y streams past it a few
// 16-byte chunks per thread at a time and is never kept in registers:
//   pass 1   statistics of z (sampled token left out) and of y, and for the KL form the cross term
//            sum_j 2^(y_j..) (y_j - z_j); KL = E_mu[y - z] - lse(y) + lse(z) needs nothing else.
//   pass 2   (TV only) sum_j min(pi_j, mu_j) with z from the registers and y read again; the first
//            chunks of y each thread consumed in pass 1 wait for it in LDS, the later ones (read a
//            few microseconds earlier, partly still in the L2) are requested again.
//   epilogue on one wave: mask, loss term, gradient coefficient.
//   gradient every resident entry, the whole row in one run of 16-byte stores; then the next row of
//            z and the first chunks of the next row of y are requested in one run of loads.
// z is read once, y once (KL) or about one and a half times (TV), the gradient written once: 6
// (7) bytes per vocabulary entry where the general kernel moves 8 (10).
// All row traffic goes through range-checked buffer views (loads past the row return 0 and are
// turned into -inf, stores past it are dropped), so the passes are straight-line code.
// Preconditions (checked by the host): V % 8 == 0, V / 8 <= 512 * NCHUNK, the three matrices
// 16-byte aligned with pitches that are multiples of 8 entries.
#include "dppo_common.hpp"
#include "dppo_launch.hpp"

namespace dppo {
namespace {

constexpr int kThreads = 512;
constexpr int kWindow = 4;        // chunks of y in flight per thread (4, 8 and 12 measure the same)
constexpr int kKeep = 18;         // TV form: chunks of y kept in LDS between the passes (18 x 8 KiB of the 160 KiB)

// Running sum of 2^(x*log2e + b) over one row with an integer offset b <= -max*log2e that only
// ever decreases (lowering it rescales the sums by an exact power of two).  T: also sum 2^x * x,
// which feeds the entropy diagnostic.  U: also sum 2^x * (x_j - other_j) in natural units, the
// cross term of the KL form (a vanished term adds nothing even where the other row is -inf too).
template <bool T, bool U>
struct RowStat {
  float b = 3.0e38f, t = 0.f, u = 0.f;
  double s = 0.0;      // float64, fed with fp32 sums of eight entries (see sum8)
  __device__ __forceinline__ void cover(float vmax) {
    const float bn = fminf(b, -ceilf(fmaxf(vmax, kNegBig) * kLog2e));
    const float d = bn - b, sc = fast_exp2(d);
    if (T) t = sc * fmaf(d, static_cast<float>(s), t);
    if (U) u *= sc;
    s *= static_cast<double>(sc);
    b = bn;
  }
  __device__ __forceinline__ float term(float v, float other) {
    const float x = fmaf(v, kLog2e, b), e = fast_exp2(x);
    if (T) t = fma_ex(e, x, t);
    if (U) u = fmaf(e, fminf(fmaxf(v - other, -3.0e38f), 3.0e38f), u);     // NaN (-inf - -inf) -> -3e38, times e = 0
    return e;
  }
  __device__ __forceinline__ void add8(const float (&v)[8], const float (&other)[8]) {
    cover(fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7]))));
    // the eight exponentials summed pairwise as they are formed (few of them alive at a time)
    const float q0 = (term(v[0], other[0]) + term(v[1], other[1])) + (term(v[2], other[2]) + term(v[3], other[3]));
    const float q1 = (term(v[4], other[4]) + term(v[5], other[5])) + (term(v[6], other[6]) + term(v[7], other[7]));
    s += static_cast<double>(q0 + q1);
  }
};

// DYN: rows handed out at run time from a counter (as in the register-resident kernel of the Binary
// / Top-K variants: the dies do not run at one speed, and with rows fixed by the workgroup index the
// slowest compute unit ends the kernel), the loss terms to one slot per row.
template <int NCHUNK, bool TV, bool DIAG, bool GRAD, bool DYN>
__global__ __launch_bounds__(kThreads) void dppo_fullvocab_resident_kernel(const KParams p) {
  static_assert(GRAD || TV, "forward only, the KL form reads each row once anyway: the general kernel serves it");
  static_assert(GRAD || !DYN, "rows at run time: the gradient forms only");
  static_assert(NCHUNK == 32 || NCHUNK == 38, "the forms the host selects: rows of more than 24 and up to 32, more than 32 and up to 38 chunks");
  constexpr int THREADS = kThreads, NW = THREADS / kWave;
  constexpr uint32_t kStride = THREADS * 16u;      // bytes between a thread's consecutive chunks
  constexpr uint32_t kNegInfPair = 0xFF80FF80u;    // two bf16 -inf
  constexpr int KEEP = TV ? (kKeep < NCHUNK ? kKeep : NCHUNK) : 0;
  constexpr int REREAD = NCHUNK - KEEP;            // TV form: chunks of y that pass 2 reads from memory again
  constexpr int FULLCHUNKS = (NCHUNK == 32) ? 24 : 32;   // chunks every row of this form fills (shorter rows take the next smaller form): only later ones can have lanes past the row
  __shared__ float sh_bz[NW], sh_by[NW];
  __shared__ double sh_sz[NW], sh_tz[NW], sh_sy[NW], sh_uy[NW], sh_acc[NW];
  __shared__ RowCoef sh_rc;
  __shared__ float sh_norm[4];
  __shared__ int sh_row[2];
  // chunks wave 0 parks around its float64 arithmetic (the TV form's kept chunks of y leave room for
  // 8), and chunks whose refill waits for the epilogue (forward only)
  constexpr int kPark = TV ? 8 : 16;
  constexpr int kLate = GRAD ? 0 : 8;
  __shared__ u32x4 sh_park[kPark > 0 ? kPark * kWave : 1];
  // every thread parks its own 16 bytes per kept chunk and takes them back itself: no synchronisation
  __shared__ u32x4 sh_y[KEEP > 0 ? KEEP * THREADS : 1];
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wid = uniform_i(tid / kWave);
  const int nvec = p.V >> 3;
  const uint32_t row_bytes = static_cast<uint32_t>(p.V) * 2u;
  const uint32_t voff = static_cast<uint32_t>(tid) * 16u;
  const u32x4 neg_inf = {kNegInfPair, kNegInfPair, kNegInfPair, kNegInfPair};
  const int64_t pitch = p.ld * 2, pitch_y = p.mu_ld * 2;
  const char* zbase = reinterpret_cast<const char*>(p.logits);
  const char* ybase = reinterpret_cast<const char*>(p.mu_logits);
  char* gbase = reinterpret_cast<char*>(p.grad);
  const EpiParams ep = epi_params(p);
  double loss_acc = 0.0;   // meaningful in wave 0 only

  u32x4 buf[NCHUNK];       // the resident row of z; chunk i of thread tid is vector i*THREADS + tid
  u32x4 yb[kWindow];       // the window on y
  // In pass 1 the rollout row is marked non-temporal where it is not read again (KL form); in the
  // TV form the first read is plain, so that the second finds what it can in the caches.
  constexpr bool kY1Nt = !TV;
  int row = first_row_of_workgroup();      // the workgroups of one die take neighbouring rows
  int next = row + static_cast<int>(gridDim.x);
  constexpr int kNoRow = 0x7fffffff;
  if (DYN) {
    if (tid == 0) {
      sh_row[0] = atomicAdd(p.row_counters, 1);
      sh_row[1] = atomicAdd(p.row_counters, 1);
    }
    __syncthreads();
    row = uniform_i(sh_row[0]);
    next = uniform_i(sh_row[1]);
    __syncthreads();
    if (row >= p.T) return;            // every row already handed out: nothing to do, and no address to form
  }
  {
    const row_rsrc_t zr = make_row_rsrc(zbase + row * pitch, row_bytes);
    const row_rsrc_t yr = make_row_rsrc(ybase + row * pitch_y, row_bytes);
#pragma unroll
    for (int i = 0; i < NCHUNK; ++i) buf[i] = row_load16<false>(zr, voff, i * kStride);
#pragma unroll
    for (int i = 0; i < kWindow; ++i) yb[i] = row_load16<kY1Nt>(yr, voff, i * kStride);
  }
  int a_next = p.sampled[row];

  for (; row < p.T;) {
    const int a = uniform_i(a_next);
    const bool more = next < p.T;
    if (more) a_next = p.sampled[next];
    // DYN: request the row after next now (thread 0); the answer is published at this row's first barrier
    int drawn = 0, next2 = kNoRow;
    if (DYN && more && tid == 0) drawn = atomicAdd(p.row_counters, 1);
    const bool live = (a >= 0 && a < p.V);
    const uint16_t* zrow = p.logits + static_cast<int64_t>(row) * p.ld;
    const row_rsrc_t yr = make_row_rsrc(ybase + row * pitch_y, row_bytes);
    // The workgroup's next rows; without one the refills go through views of zero bytes: their
    // loads touch no memory.
    const row_rsrc_t zn = make_row_rsrc(zbase + (more ? next : row) * pitch, more ? row_bytes : 0u);
    const row_rsrc_t yn = make_row_rsrc(ybase + (more ? next : row) * pitch_y, more ? row_bytes : 0u);
    const int avec = a >> 3;
    const int ia = live ? avec / THREADS : -1;               // chunk holding a_t (uniform)
    const bool owner = live && (avec - ia * THREADS == tid);
    const int sub = a & 7;

    RowCoef rc;
    rc.coef = 0.f; rc.kexp = 0.f; rc.g_a = 0.f;
    if (live) {
      const float z_a = bf16_bits_to_float(zrow[a]);
      // ---- pass 1 ------------------------------------------------------------------------------
      RowStat<DIAG, false> st;       // z, without a_t
      RowStat<false, !TV> cs;        // y, and for the KL form y - z
      st.cover(fmaxf(kNegBig, z_a));   // the offset must cover z[a_t]
#pragma unroll
      for (int i = 0; i < NCHUNK; ++i) {
        u32x4 zq = buf[i], yq = yb[i % kWindow];
        if (i + kWindow < NCHUNK) yb[i % kWindow] = row_load16<kY1Nt>(yr, voff, (i + kWindow) * kStride);
        // lanes past the row loaded 0: make them -inf in both rows (they then add nothing)
        if (i >= FULLCHUNKS && i * THREADS + tid >= nvec) { zq = neg_inf; yq = neg_inf; }
        if (TV && i < KEEP) sh_y[i * THREADS + tid] = yq;
        float z[8], y[8];
        unpack8(zq, z);
        unpack8(yq, y);
        cs.add8(y, z);
        // the sampled token's own term is left out of the sum over z (its chunk index is uniform:
        // a scalar test per chunk, the selects run once per row)
        if (i == ia) {
#pragma unroll
          for (int e = 0; e < 8; ++e) z[e] = (owner && e == sub) ? -INFINITY : z[e];
        }
        st.add8(z, z);
        // One chunk at a time: the running sums pass through an empty assembly statement, so this
        // chunk's arithmetic is done before the next one's starts.  (Without it the compiler
        // gathers the arithmetic of all chunks behind the last load, with every unpacked value
        // alive at once: over a thousand spilled registers.)
        asm volatile("" : "+v"(st.s), "+v"(st.t), "+v"(st.b), "+v"(cs.s), "+v"(cs.u), "+v"(cs.b));
        __builtin_amdgcn_sched_barrier(0);
      }
      if (TV) {
        // the second pass over y starts to travel while the statistics are combined
#pragma unroll
        for (int i = 0; i < kWindow; ++i)
          if (i < REREAD) yb[i] = row_load16<true>(yr, voff, (KEEP + i) * kStride);
      }
      // workgroup-wide offsets = the smallest ones; rescaling to them is exact
      const float wbz = -wave_max(-st.b), wby = -wave_max(-cs.b);
      if (lane == 0) { sh_bz[wid] = wbz; sh_by[wid] = wby; }
      if (DYN && tid == 0) sh_row[0] = more ? drawn : kNoRow;
      __syncthreads();
      if (DYN) next2 = uniform_i(sh_row[0]);
      float bz = sh_bz[0], by = sh_by[0];
#pragma unroll
      for (int w = 1; w < NW; ++w) { bz = fminf(bz, sh_bz[w]); by = fminf(by, sh_by[w]); }
      {
        const double dd = static_cast<double>(bz - st.b), sc = static_cast<double>(fast_exp2(bz - st.b));
        const double scy = static_cast<double>(fast_exp2(by - cs.b));
        const double sd = wave_sum(st.s * sc);
        const double td = DIAG ? wave_sum(sc * (static_cast<double>(st.t) + dd * st.s)) : 0.0;
        const double sy = wave_sum(cs.s * scy);
        const double uy = TV ? 0.0 : wave_sum(static_cast<double>(cs.u) * scy);
        if (lane == 0) { sh_sz[wid] = sd; sh_tz[wid] = td; sh_sy[wid] = sy; sh_uy[wid] = uy; }
      }
      __syncthreads();
      // Wave 0 forms the two normalisers and their logarithms (float64, with its last chunks parked
      // in shared memory meanwhile: beside the resident row there are no registers for that) and,
      // for the TV form, hands what pass 2 needs to the other waves through shared memory.
      double S_rest = 0.0, T_rest = 0.0, Sy = 0.0, Uy = 0.0, l2z = 0.0, l2y = 0.0;
      auto park = [&]() {
        if (kPark > 0) {
#pragma unroll
          for (int i = 0; i < kPark; ++i) sh_park[i * kWave + lane] = buf[NCHUNK - 1 - i];
        }
      };
      auto unpark = [&]() {
        if (kPark > 0) {
#pragma unroll
          for (int i = 0; i < kPark; ++i) buf[NCHUNK - 1 - i] = sh_park[i * kWave + lane];
        }
      };
      if (wid == 0) {
        park();
#pragma unroll
        for (int w = 0; w < NW; ++w) { S_rest += sh_sz[w]; T_rest += sh_tz[w]; Sy += sh_sy[w]; Uy += sh_uy[w]; }
        const double xa = static_cast<double>(z_a) * static_cast<double>(kLog2e) + static_cast<double>(bz);
        const double S = S_rest + exp2_d(xa);
        l2z = log2_d(S);
        l2y = log2_d(Sy);
        if (TV) {
          // The integer part of log2 S goes into the (integer) offset, which stays exact, and only
          // the fraction in [0, 1) is subtracted in fp32 (pass 2), so a probability keeps a relative
          // error of about 1e-7 however large the offset is.
          const double nz = floor(l2z), ny = floor(l2y);
          if (lane == 0) {
            sh_norm[0] = bz - static_cast<float>(nz); sh_norm[1] = by - static_cast<float>(ny);
            sh_norm[2] = static_cast<float>(l2z - nz); sh_norm[3] = static_cast<float>(l2y - ny);
          }
          unpark();
        }
      }
      double D = 0.0;               // meaningful in wave 0
      if (TV) {
        // ---- pass 2: TV = 1/2 sum |pi_j - mu_j| = 1 - sum_j min(pi_j, mu_j) -----------------------
        // One exponential per entry: the minimum is taken on the base-2 log-probabilities
        // z_j*log2e + b - log2 S
        // (offsets and fractions from wave 0, see above).
        __syncthreads();
        const float bz2 = sh_norm[0], by2 = sh_norm[1], fz = sh_norm[2], fy = sh_norm[3];
        double acc0 = 0.0, acc1 = 0.0;
#pragma unroll
        for (int j = 0; j < NCHUNK; ++j) {
          // first the chunks of y that are read again (the LAST ones pass 1 read, a few microseconds
          // ago: part of them is still in the L2), then the ones kept in LDS
          const int i = (j < REREAD) ? KEEP + j : j - REREAD;
          asm volatile("" : "+v"(buf[i]));     // unpack again here: nothing unpacked in pass 1 is kept alive
          u32x4 zq = buf[i], yq;
          if (j < REREAD) {
            yq = yb[j % kWindow];              // last use of the row: non-temporal loads
            if (j + kWindow < REREAD) yb[j % kWindow] = row_load16<true>(yr, voff, (KEEP + j + kWindow) * kStride);
            if (i >= FULLCHUNKS && i * THREADS + tid >= nvec) yq = neg_inf;
          } else {
            yq = sh_y[i * THREADS + tid];      // kept with its lanes past the row already -inf
          }
          if (i >= FULLCHUNKS && i * THREADS + tid >= nvec) zq = neg_inf;
          float z[8], y[8];
          unpack8(zq, z);
          unpack8(yq, y);
          double& acc = (j & 1) ? acc1 : acc0;
          auto mn = [&](int e) { return fast_exp2(fminf(fmaf(z[e], kLog2e, bz2) - fz, fmaf(y[e], kLog2e, by2) - fy)); };
          // eight entries among themselves (pairwise, as they are formed), then into float64
          const float q0 = (mn(0) + mn(1)) + (mn(2) + mn(3)), q1 = (mn(4) + mn(5)) + (mn(6) + mn(7));
          acc += static_cast<double>(q0 + q1);
          asm volatile("" : "+v"(acc0), "+v"(acc1));
          __builtin_amdgcn_sched_barrier(0);
        }
        if (!GRAD) {
          // forward only: nothing needs the rows any more, the next ones start to travel now -- but
          // for the last kLate chunks, whose registers the float64 epilogue of wave 0 works in; they
          // are requested behind it (they are consumed last, and the delay is the epilogue's length)
#pragma unroll
          for (int i = 0; i < NCHUNK - kLate; ++i) buf[i] = row_load16<false>(zn, voff, i * kStride);
#pragma unroll
          for (int i = 0; i < kWindow; ++i) yb[i] = row_load16<kY1Nt>(yn, voff, i * kStride);
          __builtin_amdgcn_sched_barrier(0);
        }
        const double wa = wave_sum(acc0 + acc1);
        if (lane == 0) sh_acc[wid] = wa;
        __syncthreads();
        double tot = 0.0;
        if (wid == 0) {
#pragma unroll
          for (int w = 0; w < NW; ++w) tot += sh_acc[w];
        }
        D = fmax(1.0 - tot, 0.0);
        if (tot != tot) D = tot;                  // NaN logits propagate
        if (GRAD && wid == 0) park();             // (forward only, the chunks refilled late are free anyway)
      } else if (wid == 0) {
        // KL = E_mu[y - z] - lse(y) + lse(z), the log-sum-exps in base 2 against their offsets
        const double lse2_z = l2z - static_cast<double>(bz), lse2_y = l2y - static_cast<double>(by);
        D = Uy / Sy + kLn2 * (lse2_z - lse2_y);
        D = (D > 0.0 || D != D) ? D : 0.0;       // rounding can leave -1e-8 for identical rows
      }
      // ---- epilogue on wave 0 (inlined: one workgroup per compute unit, nothing would hide a call)
      // With the gradient the resident row is still needed afterwards, and the epilogue's float64
      // arithmetic finds no registers beside it: wave 0 parks its last chunks in shared memory around
      // it (its own 16 bytes per lane and chunk, no synchronisation) instead of spilling to scratch
      // memory, whose round trips would sit on the path the other seven waves wait for.
      if (wid == 0) {
        RowScalars rs;
        rs.a = a;
        rs.za = z_a;
        rs.lmu = p.mu_logp[row];
        rs.lanc = anchor_or(p, row, rs.lmu);
        rs.adv = p.adv[row];
        TopkLane tk;
        tk.id = -1; tk.lp = 0.f; tk.z = 0.f;
        // through an empty asm statement, so that the addresses of the per-token outputs are formed
        // here and not held in registers across the passes
        int row_e = row;
        asm volatile("" : "+s"(row_e));
        const RowResult res = row_epilogue(ep, row_e, rs, tk, zrow, bz, S_rest, T_rest, lane, D);
        rc = res.rc;
        if (DYN) { if (lane == 0) p.row_loss[row] = res.loss_term; }
        else loss_acc += res.loss_term;
        if (GRAD && lane == 0) sh_rc = rc;
        if (GRAD) unpark();
      }
      // (forward only, this barrier also keeps the next row's statistics from overwriting the
      // shared sums while a slower wave still reads them)
      __syncthreads();
      if (!GRAD) {
#pragma unroll
        for (int i = NCHUNK - kLate; i < NCHUNK; ++i) buf[i] = row_load16<false>(zn, voff, i * kStride);
      }
      if (GRAD) {
        rc.coef = uniform_f(sh_rc.coef);
        rc.kexp = uniform_f(sh_rc.kexp);
        rc.g_a = uniform_f(sh_rc.g_a);
      }
    } else {
      if (tid == 0) {
        p.divergence[row] = 0.f;
        p.mask[row] = 0;
        if (p.loss_tok) p.loss_tok[row] = 0.f;
        if (p.diag) {
          for (int k = 0; k < 8; ++k) p.diag[static_cast<int64_t>(row) * 8 + k] = 0.f;
        }
        if (DYN) p.row_loss[row] = 0.0;
      }
      if (DYN) {
        if (tid == 0) sh_row[0] = more ? drawn : kNoRow;
        __syncthreads();
        next2 = uniform_i(sh_row[0]);
        __syncthreads();
      }
    }

    // ---- gradient out, next rows in -----------------------------------------------------------
    if (!GRAD) {
      if (!live) {       // an ignored row skipped the passes and with them the refill
#pragma unroll
        for (int i = 0; i < NCHUNK; ++i) buf[i] = row_load16<false>(zn, voff, i * kStride);
#pragma unroll
        for (int i = 0; i < kWindow; ++i) yb[i] = row_load16<kY1Nt>(yn, voff, i * kStride);
      }
    } else {
      char* gr = gbase + row * pitch;
      const row_desc_t gout = make_row_desc(gr, row_bytes);
      const uint32_t sgn = (rc.coef < 0.f) ? 0x80008000u : 0u;
      if (rc.coef == 0.f) {
        // Masked, zero-advantage or ignored row: its gradient is exactly zero whatever the logits
        // hold.  Overwrite the resident copy with -inf so that the loop below writes 2^-inf = 0.
#pragma unroll
        for (int i = 0; i < NCHUNK; ++i) buf[i] = neg_inf;
      }
#pragma unroll
      for (int i = 0; i < NCHUNK; ++i) {
        asm volatile("" : "+v"(buf[i]));       // unpack again here: nothing unpacked in an earlier pass is kept alive
        float z[8];
        unpack8(buf[i], z);
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = fast_exp2(fmaf(z[e], kLog2e, rc.kexp));
        const u32x4 o = {pack_bf16x2(z[0], z[1]) ^ sgn, pack_bf16x2(z[2], z[3]) ^ sgn, pack_bf16x2(z[4], z[5]) ^ sgn, pack_bf16x2(z[6], z[7]) ^ sgn};
        row_store16_untracked(gout, voff, i * kStride, o);
      }
      // Keep the instruction scheduler from hoisting the refills above the stores: a refill can
      // only reuse its chunk's registers once the store has been given them.
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < NCHUNK; ++i) buf[i] = row_load16<false>(zn, voff, i * kStride);
#pragma unroll
      for (int i = 0; i < kWindow; ++i) yb[i] = row_load16<kY1Nt>(yn, voff, i * kStride);
      __builtin_amdgcn_sched_barrier(0);
      if (rc.coef != 0.f && owner) {
        // The vector store above wrote the softmax term at a_t.  Once it has completed, the owning
        // thread writes the sampled token's own entry over it.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        reinterpret_cast<uint16_t*>(gr)[a] = float_to_bf16_bits(rc.g_a);
      }
    }
    row = next;
    next = DYN ? next2 : next + static_cast<int>(gridDim.x);
  }
  if (!DYN && tid == 0) p.partial[blockIdx.x] = loss_acc;
}

template <int NCHUNK>
hipError_t launch_chunks(const KParams& p, bool tv, bool grad, int grid, hipStream_t s) {
  const bool diag = p.diag != nullptr, dyn = p.row_counters != nullptr;
  if (dyn && !grad) return hipErrorInvalidValue;       // rows at run time: the gradient forms only
  const dim3 g(grid), b(kThreads);
#define DPPO_FORM(TVF, D, G, Y) hipLaunchKernelGGL((dppo_fullvocab_resident_kernel<NCHUNK, TVF, D, G, Y>), g, b, 0, s, p)
  if (!grad) {
    if (diag) DPPO_FORM(true, true, false, false); else DPPO_FORM(true, false, false, false);
  } else if (tv) {
    if (diag) { if (dyn) DPPO_FORM(true, true, true, true); else DPPO_FORM(true, true, true, false); }
    else      { if (dyn) DPPO_FORM(true, false, true, true); else DPPO_FORM(true, false, true, false); }
  } else {
    if (diag) { if (dyn) DPPO_FORM(false, true, true, true); else DPPO_FORM(false, true, true, false); }
    else      { if (dyn) DPPO_FORM(false, false, true, true); else DPPO_FORM(false, false, true, false); }
  }
#undef DPPO_FORM
  return hipGetLastError();
}

}  // namespace

// Chunks of 512 x 16 bytes that cover a row in this form, 0 where it does not apply.  It applies to
// the backward of both variants and to the forward-only TV form (which reads both rows twice; the
// forward-only KL form reads each row once in the general kernel too), on rows of 98312 .. 155648
// entries (shorter rows stay with the general kernel, several of whose rows fit the caches
// together), a multiple of 8, every matrix 16-byte aligned with a pitch that is a multiple of 8.
int fullvocab_resident_chunks(const KParams& p, bool tv, bool grad) {
  if (!(grad || tv) || !p.mu_logits || p.V % 8 != 0 || p.ld % 8 != 0 || p.mu_ld % 8 != 0) return 0;
  if ((reinterpret_cast<uintptr_t>(p.logits) | reinterpret_cast<uintptr_t>(p.mu_logits) | (grad ? reinterpret_cast<uintptr_t>(p.grad) : 0)) & 15u) return 0;
  const int64_t nvec = p.V / 8;
  if (nvec <= kThreads * 24) return 0;
  if (nvec <= kThreads * 32) return 32;
  if (nvec <= kThreads * 38) return 38;
  return 0;
}

hipError_t launch_fullvocab_resident(const KParams& p, bool tv, bool grad, int chunks, int grid, hipStream_t s) {
  if (chunks == 32) return launch_chunks<32>(p, tv, grad, grid, s);
  if (chunks == 38) return launch_chunks<38>(p, tv, grad, grid, s);
  return hipErrorInvalidValue;
}

}  // namespace dppo
