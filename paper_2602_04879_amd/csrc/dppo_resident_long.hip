// Register-resident kernel for rows too long for the register file alone: fused forward+backward
// for vocabularies of 155 657 .. 262 144 entries (rows of 304 .. 512 KiB; a 256 000-entry
// vocabulary is 500 KiB).
//
// One persistent workgroup of 512 threads per compute unit owns one row at a time.  The row is
// cut into chunks of 512 x 16 bytes (chunk c of thread tid is vector c*512 + tid) and kept in
// up to three places between the statistics pass and the gradient pass:
//   R chunks        in vector registers,
//   up to 18 chunks in LDS (144 of the 160 KiB), loaded straight into it (buffer_load ... lds: no
//                   registers on the way); every wave reads back only what it loaded itself, so
//                   no barrier is involved,
//   the rest        nowhere: those chunks pass through a window of W chunks of registers, once
//                   for the statistics and once more for the gradient (the re-read mostly hits
//                   the caches: a quarter of the row at most, read again within one row's time).
// Two forms: (R, W) = (38, 0) for rows of up to 56 chunks (229 376 entries), read from memory
// exactly once; (30, 8) for up to 64 chunks (262 144 entries), of which up to 16 are read twice.
// The gradient is written exactly once.  The general kernel reads every row twice.
//
// The order of the memory instructions of a row keeps what the shorter register-resident kernel
// found: one run of stores, then one run of loads.  The waits of the window follow from one rule:
// a load is never waited for while a run of stores issued AFTER it is in flight.  (The hardware
// counts loads and stores in one counter; the gradient stores are hidden from the compiler, which
// therefore waits for "all but the loads issued later", and that count includes, on the hardware's
// side, every younger store: waiting for a load in front of a run of younger stores means waiting
// for those stores to drain.)  Hence, per row:
//   statistics   register chunks (as they arrive), window batch A (tail chunks 0..W-1), request
//                batch B (tail chunks W..2W-1), LDS chunks, batch B, then request batch B AGAIN
//                (read a few microseconds ago: its lines may still be in the L2; with a tail of one
//                batch, that one): it travels during the epilogue and is the first thing the
//                gradient pass turns into stores;
//   gradient     window, registers, LDS chunks: one run of stores;
//   next row     request batch A of THIS row again, then the next row's register and LDS chunks in
//                one run of loads; batch A comes back first and leaves as (a few) stores while the
//                rest of the run is on its way; then batch A of the next row is requested.
// (Without a window the LDS chunks are requested and consumed first.)
// Preconditions (checked by the host): V % 8 == 0, 38 < ceil(V / 4096) <= 64, logits and
// grad_logits 16-byte aligned with ld % 8 == 0.
#include "dppo_common.hpp"
#include "dppo_launch.hpp"
#include "dppo_resident_parts.hpp"

namespace dppo {
namespace {

constexpr int kLThreads = 512;
constexpr int kLLds = 18;        // chunks in LDS at most
constexpr int kLPark = 8;        // chunks wave 0 parks in LDS around the float64 epilogue
constexpr int kLMinChunks = 39, kLMidChunks = 38 + kLLds, kLMaxChunks = 30 + kLLds + 2 * 8;
constexpr uint32_t kLStride = kLThreads * 16u;    // bytes between a thread's consecutive chunks

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// kLReg chunks in registers, a window of kLWin chunks (the tail is at most two windows long)
template <int kLReg, int kLWin, bool DIAG, bool DYN>
__global__ __launch_bounds__(kLThreads, 2) void dppo_resident_long_kernel(const KParams p, const int nchunks) {
  constexpr int NW = kLThreads / kWave;
  // Which part of a row is requested, and consumed, first.  Without a window: the LDS chunks
  // (measured 1.5-2 % faster from 48 chunks on, 1.3 % slower at 40).  With it: the registers, so
  // that the LDS chunks' arithmetic covers the latency of window batch B (both orders, and LDS
  // chunks - registers - window, measure within 0.2 % of each other; batch A between the LDS chunks
  // and the registers, which delays the request of the registers behind the re-read, is 1.5 % slower).
  constexpr bool kLdsFirst = (kLWin == 0);
  __shared__ float sh_b[2][NW];
  __shared__ double sh_s[2][NW], sh_t[2][NW];
  __shared__ RowCoef sh_rc;
  __shared__ int sh_row[2];
  __shared__ u32x4 sh_park[kLPark * kWave];
  __shared__ u32x4 sh_l[kLLds * kLThreads];
  int par = 0;
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wid = uniform_i(tid / kWave);
  const int nvec = p.V >> 3;
  const uint32_t row_bytes = static_cast<uint32_t>(p.V) * 2u;
  const uint32_t voff = static_cast<uint32_t>(tid) * 16u;
  const u32x4 neg_inf = {kNegInfPair, kNegInfPair, kNegInfPair, kNegInfPair};
  const int64_t pitch = p.ld * 2;
  const char* logits = reinterpret_cast<const char*>(p.logits);
  char* grad = reinterpret_cast<char*>(p.grad);
  const EpiParams ep = epi_params(p);
  double loss_acc = 0.0;                        // meaningful in wave 0 only
  const int nl = uniform_i(min(kLLds, nchunks - kLReg));                               // LDS chunks in use
  const int nt = kLWin > 0 ? uniform_i(max(0, nchunks - kLReg - kLLds)) : 0;           // tail chunks (0 .. 2 kLWin)

  u32x4 buf[kLReg];                     // the register part of the row
  u32x4 w[kLWin > 0 ? kLWin : 1];       // the window

  // Requests of a row's parts.  A row without a successor is "loaded" through a view of zero
  // bytes: such loads touch no memory.
  auto load_regs = [&](row_rsrc_t r) {
#pragma unroll
    for (int i = 0; i < kLReg; ++i) buf[i] = row_load16<false>(r, voff, i * kLStride);
  };
  auto load_lds = [&](row_rsrc_t r) {
#pragma unroll
    for (int j = 0; j < kLLds; ++j)
      if (j < nl) __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr_t)(sh_l + j * kLThreads + wid * kWave), 16, voff, (kLReg + j) * kLStride, 0, 0);
  };
  // tail chunks first .. first + 7 into the window (NT: last read of them)
  auto load_window = [&](row_rsrc_t r, int first, bool nontemporal) {
#pragma unroll
    for (int k = 0; k < kLWin; ++k)
      if (first + k < nt) {
        const uint32_t so = static_cast<uint32_t>(kLReg + kLLds + first + k) * kLStride;
        w[k] = nontemporal ? row_load16<true>(r, voff, so) : row_load16<false>(r, voff, so);
      }
  };
  // gradient of the window's chunks, which hold tail chunks first .. first + W - 1
  auto store_window = [&](row_desc_t gout, int first, float kexp, uint32_t sgn) {
#pragma unroll
    for (int k = 0; k < kLWin; ++k)
      if (first + k < nt) row_store16_untracked(gout, voff, static_cast<uint32_t>(kLReg + kLLds + first + k) * kLStride, grad8(w[k], kexp, sgn));
  };
  // With a tail of two batches, the batch read LAST for the statistics (B) is the one requested
  // again before the epilogue: its lines were fetched a few microseconds earlier and may still be
  // in the L2; batch A, read at the row's start, comes again at the head of the next run of loads.
  const int re1 = uniform_i(nt > kLWin ? kLWin : 0), re2 = uniform_i(nt > kLWin ? 0 : kLWin);
  // lanes past the row loaded 0: -inf instead (only chunks from 38 on can have any)
  auto in_row = [&](u32x4 v, int chunk) { return (chunk * kLThreads + tid >= nvec) ? neg_inf : v; };

  int row = first_row_of_workgroup();
  constexpr int kNoRow = 0x7fffffff;
  int next = row + static_cast<int>(gridDim.x);
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
  // Fetched one row ahead, so that wave 0's gathers never wait on a load that queues behind the
  // row's own run of loads (a wait for the top-K ids at the top of a row would be a wait for the
  // whole run, with wave 0's statistics still to do when the other waves are through): the sampled
  // id, and (wave 0, lane k < K) the id and log-prob of top-K entry k.
  int a_next = p.sampled[row];
  int tkid_next = -1;
  float tklp_next = 0.f;
  if (wid == 0 && lane < p.K) {
    tkid_next = p.tk_ids[static_cast<int64_t>(row) * p.K + lane];
    tklp_next = p.tk_lp[static_cast<int64_t>(row) * p.K + lane];
  }
  {
    const row_rsrc_t zr = make_row_rsrc(logits + row * pitch, row_bytes);
    if (!kLdsFirst) load_regs(zr);
    load_lds(zr);
    if (kLdsFirst) load_regs(zr);
    load_window(zr, 0, false);
  }

  for (; row < p.T;) {
    const int a = uniform_i(a_next);
    const bool more = next < p.T;
    if (more) a_next = p.sampled[next];
    const int tkid = tkid_next;
    const float tklp = tklp_next;
    if (more && wid == 0 && lane < p.K) {
      tkid_next = p.tk_ids[static_cast<int64_t>(next) * p.K + lane];
      tklp_next = p.tk_lp[static_cast<int64_t>(next) * p.K + lane];
    }
    int drawn = 0;
    if (DYN && more && tid == 0) drawn = atomicAdd(p.row_counters, 1);     // the row after next
    int next2 = kNoRow;
    auto publish_row_after_next = [&]() { sh_row[par] = more ? drawn : kNoRow; };
    const bool live = (a >= 0 && a < p.V);
    const uint16_t* zrow = p.logits + static_cast<int64_t>(row) * p.ld;
    const row_rsrc_t zr = make_row_rsrc(logits + row * pitch, row_bytes);
    const row_rsrc_t zn = make_row_rsrc(logits + (more ? next : row) * pitch, more ? row_bytes : 0u);
    const int avec = a >> 3;
    const int ia = live ? avec / kLThreads : -1;               // chunk holding a_t (uniform)
    const bool owner = live && (avec - ia * kLThreads == tid);
    const int sub = a & 7;

    RowCoef rc;
    rc.coef = 0.f; rc.kexp = 0.f; rc.g_a = 0.f;
    if (live) {
      RowScalars rs;
      TopkLane tk;
      tk.id = -1; tk.lp = 0.f; tk.z = 0.f;
      rs.a = a; rs.za = 0.f; rs.lmu = 0.f; rs.adv = 0.f; rs.lanc = 0.f;
      // Inputs of the epilogue, requested now so that they have arrived when it runs; the two
      // gathered logits stay raw bit patterns until then (see below).
      uint32_t za_bits = 0, tkz_bits = 0;
      float packed_scalars = 0.f;
      if (wid == 0) {
        za_bits = zrow[a];
        packed_scalars = load_row_scalars(p, row, lane);      // log mu(a_t), A_t, the anchor's log-prob: one register
        if (tkid >= 0 && tkid < p.V && tkid != a) {
          tk.id = tkid;
          tk.lp = tklp;
          tkz_bits = zrow[tkid];
        }
      }
      // ---- statistics: online over groups of two chunks (see the shorter kernel) ---------------
      PackedRowStat<DIAG> ps;
      auto group = [&](const u32x4 v0, const u32x4 v1) { ps.add2(v0, v1); };
      // a chunk that is not kept in registers, as the statistics see it: lanes past the row and
      // the sampled token's own entry (left out of the sum, see row_epilogue) are -inf
      auto seen = [&](u32x4 v, int chunk) {
        v = in_row(v, chunk);
        if (chunk == ia && owner) v = patch16(v, sub, 0xFF80u);
        return v;
      };
      auto stats_lds = [&]() {
#pragma unroll
        for (int j = 0; j < kLLds; j += 2)
          if (j < nl) group(seen(sh_l[j * kLThreads + tid], kLReg + j), (j + 1 < nl) ? seen(sh_l[(j + 1) * kLThreads + tid], kLReg + j + 1) : neg_inf);
      };
      auto stats_regs = [&]() {
#pragma unroll
        for (int g0 = 0; g0 < kLReg; g0 += 2) {
#pragma unroll
          for (int i = 0; i < 2; ++i)
            if (g0 + i == ia && owner) buf[g0 + i] = patch16(buf[g0 + i], sub, 0xFF80u);
          group(buf[g0], buf[g0 + 1]);
        }
      };
      // window batch A, then batch B is requested
      auto stats_a = [&]() {
#pragma unroll
        for (int k = 0; k < kLWin; k += 2)
          if (k < nt) group(seen(w[k], kLReg + kLLds + k), (k + 1 < nt) ? seen(w[k + 1], kLReg + kLLds + k + 1) : neg_inf);
        __builtin_amdgcn_sched_barrier(0);
        load_window(zr, kLWin, false);
        __builtin_amdgcn_sched_barrier(0);
      };
      // window batch B, then the first tail chunks are requested again, for the gradient
      auto stats_b = [&]() {
#pragma unroll
        for (int k = 0; k < kLWin; k += 2)
          if (kLWin + k < nt) group(seen(w[k], kLReg + kLLds + kLWin + k), (kLWin + k + 1 < nt) ? seen(w[k + 1], kLReg + kLLds + kLWin + k + 1) : neg_inf);
        __builtin_amdgcn_sched_barrier(0);
        load_window(zr, re1, false);
        __builtin_amdgcn_sched_barrier(0);
      };
      if (kLdsFirst) { stats_lds(); stats_regs(); }
      else           { stats_regs(); stats_a(); stats_lds(); stats_b(); }

      // wave-level combine: common offset = the smallest one, rescaling is exact
      const float bw = -wave_max(-ps.b);
      const double dw = static_cast<double>(bw - ps.b), scw = static_cast<double>(fast_exp2(bw - ps.b));
      const double st = ps.sd, tt = static_cast<double>(ps.tsum());
      const double sw = wave_sum(st * scw);
      const double tw = DIAG ? wave_sum(scw * (tt + dw * st)) : 0.0;
      if (lane == 0) { sh_b[par][wid] = bw; sh_s[par][wid] = sw; sh_t[par][wid] = tw; }
      // Wave 0 parks its last register chunks in LDS around the float64 epilogue (its own 16 bytes
      // per lane and chunk, no synchronisation), and runs the part of the epilogue that needs the
      // row's inputs only before the barrier.
      RowPre pre;
      if (wid == 0) {
#pragma unroll
        for (int i = 0; i < kLPark; ++i) sh_park[i * kWave + lane] = buf[kLReg - 1 - i];
        // (the epilogue's inputs are looked at HERE, behind the statistics: moved up to where they
        // were requested, their first use, be it a shift, would be a wait for the whole run of
        // loads in front of them)
        asm volatile("" : "+v"(za_bits), "+v"(packed_scalars), "+v"(tkz_bits), "+v"(tk.lp), "+v"(tk.id));
        unpack_row_scalars(packed_scalars, rs);
        rs.za = __uint_as_float(za_bits << 16);
        tk.z = __uint_as_float(tkz_bits << 16);
        pre = row_pre(rs, tk, p.K > 0, p.relax_log_alpha);
      }
      if (DYN && tid == 0) publish_row_after_next();
      __syncthreads();
      if (DYN) next2 = uniform_i(sh_row[par]);
      RowOut ro;
      if (wid == 0) {
        float bb = -ceilf(fmaxf(rs.za, kNegBig) * kLog2e);     // the offset must also cover z[a_t]
#pragma unroll
        for (int q = 0; q < NW; ++q) bb = fminf(bb, sh_b[par][q]);
        double S_rest = 0.0, T_rest = 0.0;
#pragma unroll
        for (int q = 0; q < NW; ++q) {
          const double dd = static_cast<double>(bb - sh_b[par][q]), sc = static_cast<double>(fast_exp2(bb - sh_b[par][q]));   // exact power of two
          S_rest += sh_s[par][q] * sc;
          if (DIAG) T_rest += sc * (sh_t[par][q] + dd * sh_s[par][q]);
        }
        const RowResult rr = row_post(ep, row, pre, a, zrow, bb, S_rest, T_rest, lane, 0.0, ro);
        rc = rr.rc;
        if (DYN) { if (lane == 0) p.row_loss[row] = rr.loss_term; }
        else loss_acc += rr.loss_term;
        if (lane == 0) sh_rc = rc;
#pragma unroll
        for (int i = 0; i < kLPark; ++i) buf[kLReg - 1 - i] = sh_park[i * kWave + lane];
      }
      par ^= 1;
      __syncthreads();
      rc.coef = uniform_f(sh_rc.coef);
      rc.kexp = uniform_f(sh_rc.kexp);
      rc.g_a = uniform_f(sh_rc.g_a);
      if (wid == 0) {
        int row_e = row;
        asm volatile("" : "+s"(row_e));
        row_store(ep, row_e, ro, lane);
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
        if (tid == 0) publish_row_after_next();
        __syncthreads();
        next2 = uniform_i(sh_row[par]);
        par ^= 1;
      }
    }

    // ---- gradient out, next row in ------------------------------------------------------------
    char* gr = grad + row * pitch;
    const row_desc_t gout = make_row_desc(gr, row_bytes);
    const bool zero_row = (rc.coef == 0.f);       // masked, zero-advantage or ignored: the gradient is exactly zero
    const uint32_t sgn = (rc.coef < 0.f) ? 0x80008000u : 0u;
    if (zero_row) {
      const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int c = 0; c < kLReg + kLLds + 2 * kLWin; ++c)
        if (c < nchunks) row_store16_untracked(gout, voff, c * kLStride, zero);
    } else {
      // the window first (the tail chunks requested before the epilogue), so that nothing waits
      // for a load behind younger stores
      store_window(gout, re1, rc.kexp, sgn);
#pragma unroll
      for (int i = 0; i < kLReg; ++i) row_store16_untracked(gout, voff, i * kLStride, grad8(buf[i], rc.kexp, sgn));
#pragma unroll
      for (int j = 0; j < kLLds; ++j)
        if (j < nl) row_store16_untracked(gout, voff, (kLReg + j) * kLStride, grad8(sh_l[j * kLThreads + tid], rc.kexp, sgn));
    }
    // Keep the instruction scheduler from hoisting the loads above the stores: a load can only
    // reuse its chunk's registers (or its LDS slot) once the store has been given them.
    __builtin_amdgcn_sched_barrier(0);
    if (!zero_row) load_window(zr, re2, true);        // the rest of this row's tail, once more (re2 = W: none)
    if (!kLdsFirst) load_regs(zn);
    load_lds(zn);
    if (kLdsFirst) load_regs(zn);
    __builtin_amdgcn_sched_barrier(0);
    if (!zero_row && nt > kLWin) store_window(gout, re2, rc.kexp, sgn);
    __builtin_amdgcn_sched_barrier(0);
    load_window(zn, 0, false);                        // batch A of the next row
    __builtin_amdgcn_sched_barrier(0);
    if (!zero_row && owner) {
      // The vector stores wrote the softmax term (or 0) at a_t.  Once they have completed, the
      // owning thread writes the sampled token's own entry over it.
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      reinterpret_cast<uint16_t*>(gr)[a] = float_to_bf16_bits(rc.g_a);
    }
    row = next;
    next = DYN ? next2 : next + static_cast<int>(gridDim.x);
  }
  if (!DYN && tid == 0) p.partial[blockIdx.x] = loss_acc;
}

}  // namespace

// Chunks of 512 x 16 bytes that cover a row in this form, 0 where it does not apply.
int resident_long_chunks(int64_t V) {
  if (V % 8 != 0) return 0;
  const int64_t nchunks = (V / 8 + kLThreads - 1) / kLThreads;
  return (nchunks >= kLMinChunks && nchunks <= kLMaxChunks) ? static_cast<int>(nchunks) : 0;
}

hipError_t launch_resident_long(const KParams& p, int chunks, int grid, hipStream_t s) {
  if (chunks < kLMinChunks || chunks > kLMaxChunks || !p.grad) return hipErrorInvalidValue;
  const bool diag = p.diag != nullptr, dyn = p.row_counters != nullptr;
  const dim3 g(grid), b(kLThreads);
#define DPPO_FORM(R, W, D, Y) hipLaunchKernelGGL((dppo_resident_long_kernel<R, W, D, Y>), g, b, 0, s, p, chunks)
  if (chunks <= kLMidChunks) {
    if (diag) { if (dyn) DPPO_FORM(38, 0, true, true); else DPPO_FORM(38, 0, true, false); }
    else      { if (dyn) DPPO_FORM(38, 0, false, true); else DPPO_FORM(38, 0, false, false); }
  } else {
    if (diag) { if (dyn) DPPO_FORM(30, 8, true, true); else DPPO_FORM(30, 8, true, false); }
    else      { if (dyn) DPPO_FORM(30, 8, false, true); else DPPO_FORM(30, 8, false, false); }
  }
#undef DPPO_FORM
  return hipGetLastError();
}

}  // namespace dppo
