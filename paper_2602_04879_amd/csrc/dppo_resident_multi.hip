// Register-resident kernel for rows of middle length (16 392 .. 65 536 entries, 32 .. 128 KiB):
// fused forward+backward, SEVERAL rows per workgroup.
//
// The memory system serves a compute unit best in long bursts of one direction: the kernel for
// long rows (one row of ~300 KiB per workgroup of 512 threads, one workgroup per compute unit,
// a row's stores in one run, then the next row's loads in one run) moves its bytes 10-15 % faster
// than the same code in small shapes with several workgroups per compute unit, whose bursts are one
// short row long and interleave at random.  So rows of middle length are taken in GROUPS of ROWS
// consecutive rows, ROWS x RC chunks of 512 x 16 bytes in the registers of one persistent
// workgroup per compute unit (chunk i of row r of thread tid: vector i*512 + tid of that row):
//
//   statistics   row by row over the resident chunks (every row spans all eight waves), one LDS
//                record per row and wave, ONE barrier for the group;
//   epilogue     wave r runs the per-token epilogue of row r: the group's epilogues run side by side;
//                one more barrier;
//   gradient     all ROWS x RC chunks in one run of stores, then the next group in one run of loads.
//
// Groups are handed out at run time (one atomic counter, drawn one group ahead: the dies do not run
// at one speed); the loss terms go to one slot per row.  The host takes this form only when a
// compute unit gets many groups: a group is 23 us of its time, and with few of them a call ends
// sooner on the one-row shapes, whose unit of work is a row (groups fixed by the workgroup index
// were measured too: never ahead of both).  Rows past T in the last group are views of zero
// bytes: nothing is read or written for them.
// Preconditions (checked by the host): V % 8 == 0, 512 (RC - 2) < V / 8 <= 512 RC, logits and
// grad_logits 16-byte aligned with ld % 8 == 0 (the RAGGED form: any V and pitch, rows 2-byte
// aligned, logits and grad_logits with the same address modulo 16, every frame within the shape),
// p.row_counters and p.row_loss set.
#include "dppo_common.hpp"
#include "dppo_launch.hpp"
#include "dppo_resident_parts.hpp"

namespace dppo {
namespace {

constexpr int kMThreads = 512;
// Chunks of a row whose lanes can lie past its end: the last two at most (the host takes a shape
// only with less slack than that).
constexpr int kMTailChunks = 2;

// RAGGED = true: rows that do not start on a 128-byte line, or whose length is not a multiple of 8,
// handled as in the one-row kernel's ragged form: a row in its FRAME, the aligned 16-byte blocks
// from the start of the line holding its first entry (h = (row address mod 128) / 2 entries in
// front of it) to the block holding its last; what the frame holds beside the row is read, turned
// into -inf in the resident copy, and never written (incomplete first / last blocks of the
// gradient leave as 2-byte stores of the row's own entries).
template <int ROWS, int RC, bool DIAG, bool RAGGED>
__global__ __launch_bounds__(kMThreads, 2) void dppo_resident_multi_kernel(const KParams p) {
  constexpr int NW = kMThreads / kWave, NCHUNK = ROWS * RC;
  static_assert(ROWS >= 2 && ROWS <= NW, "one epilogue wave per row of the group");
  static_assert(RC % 2 == 0 && NCHUNK <= 36, "chunks are consumed in pairs; the group has to fit the registers");
  constexpr uint32_t kStride = kMThreads * 16u;   // bytes between a thread's consecutive chunks of a row
  constexpr int kNone = 0x7fffffff;
  __shared__ float sh_b[ROWS][NW];
  __shared__ double sh_s[ROWS][NW], sh_t[ROWS][NW];
  __shared__ RowCoef sh_rc[ROWS];
  __shared__ int sh_grp[2];
  int par = 0;
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wid = uniform_i(tid / kWave);
  const int nvec_aligned = p.V >> 3;
  const uint32_t row_bytes = static_cast<uint32_t>(p.V) * 2u;
  const uint32_t voff = static_cast<uint32_t>(tid) * 16u;
  const u32x4 neg_inf = {kNegInfPair, kNegInfPair, kNegInfPair, kNegInfPair};
  const int64_t pitch = p.ld * 2;               // row pitch in bytes
  const char* logits = reinterpret_cast<const char*>(p.logits);
  char* grad = reinterpret_cast<char*>(p.grad);
  const EpiParams ep = epi_params(p);
  const int ngroups = (p.T + ROWS - 1) / ROWS;

  u32x4 buf[NCHUNK];                            // the resident group

  // groups are handed out at run time, drawn from a counter one group ahead
  if (tid == 0) {
    sh_grp[0] = atomicAdd(p.row_counters, 1);
    sh_grp[1] = atomicAdd(p.row_counters, 1);
  }
  __syncthreads();
  int grp = uniform_i(sh_grp[0]);
  int next = uniform_i(sh_grp[1]);
  __syncthreads();
  // (a workgroup that starts when every group has been handed out forms no address)
  if (grp >= ngroups) return;

  // Fetched one group ahead, before the group's own loads (so that nothing at the top of a group
  // waits behind them): the sampled ids of the group's rows, row r in lane r of every wave (-1: no
  // such row), and in wave r, lane k < K, the id and log-prob of top-K entry k of row r.
  auto load_ids = [&](int g) -> int {
    const int row = g * ROWS + lane;
    return (lane < ROWS && row < p.T) ? p.sampled[row] : -1;
  };
  auto load_topk = [&](int g, int& id, float& lp) {
    const int row = g * ROWS + wid;
    id = -1;
    lp = 0.f;
    if (wid < ROWS && row < p.T && lane < p.K) {
      id = p.tk_ids[static_cast<int64_t>(row) * p.K + lane];
      lp = p.tk_lp[static_cast<int64_t>(row) * p.K + lane];
    }
  };
  // RAGGED: entries of the frame in front of the row, 0..63 (else 0)
  auto head_of = [&](int r) -> int {
    return RAGGED ? static_cast<int>(((reinterpret_cast<uintptr_t>(logits) + static_cast<uint64_t>(r * pitch)) >> 1) & 63u) : 0;
  };
  // One run of loads: the ROWS x RC chunks of group g (has = false: views of zero bytes).  RAGGED:
  // views of the rows' frames, up to the end of the 4-byte word holding a row's last entry.
  auto load_group = [&](int g, bool has) {
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
      const int row = (has ? g : 0) * ROWS + r;
      const bool ok = has && row < p.T;
      const int hr = ok ? head_of(row) : 0;
      const row_rsrc_t zr = make_row_rsrc(logits + (ok ? row : 0) * pitch - 2 * hr,
                                          ok ? (RAGGED ? ((static_cast<uint32_t>(hr + p.V) * 2u + 3u) & ~3u) : row_bytes) : 0u);
      // (each load pinned in program order: left to the scheduler the run is issued in an order of
      // its own, another one here than at the top of the kernel; measured 1.7 % slower)
#pragma unroll
      for (int i = 0; i < RC; ++i) {
        buf[r * RC + i] = row_load16<false>(zr, voff, i * kStride);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  int a_vec_next = load_ids(grp);
  int tkid_next;
  float tklp_next;
  load_topk(grp, tkid_next, tklp_next);
  __builtin_amdgcn_sched_barrier(0);
  load_group(grp, true);

  for (; grp < ngroups;) {
    const int a_vec = a_vec_next;
    const bool more = next < ngroups;
    if (more) a_vec_next = load_ids(next);
    // request the group after next now; the answer is looked at before this group's barrier
    int drawn = 0;
    if (more && tid == 0) drawn = atomicAdd(p.row_counters, 1);
    const int tkid = tkid_next;
    const float tklp = tklp_next;
    if (more) load_topk(next, tkid_next, tklp_next);
    const int row0 = grp * ROWS;

    // ---- this wave's epilogue row: its inputs, requested now ---------------------------------
    const int erow = row0 + wid;
    const bool ewave = wid < ROWS && erow < p.T;
    const int ea = ewave ? __builtin_amdgcn_readlane(a_vec, wid < ROWS ? wid : 0) : -1;
    const bool elive = ewave && ea >= 0 && ea < p.V;
    const uint16_t* ezrow = p.logits + static_cast<int64_t>(ewave ? erow : 0) * p.ld;
    RowScalars rs;
    TopkLane tk;
    tk.id = -1; tk.lp = 0.f; tk.z = 0.f;
    rs.a = ea; rs.za = 0.f; rs.lmu = 0.f; rs.adv = 0.f; rs.lanc = 0.f;
    // (the gathered logits stay raw bit patterns until the statistics are through: their first
    // use up here would be a wait for every load of the group in front of them)
    uint32_t za_bits = 0, tkz_bits = 0;
    float packed_scalars = 0.f;
    if (elive) {
      za_bits = ezrow[ea];
      packed_scalars = load_row_scalars(p, erow, lane);      // log mu(a_t), A_t, the anchor's log-prob: one register
      if (tkid >= 0 && tkid < p.V && tkid != ea) {
        tk.id = tkid;
        tk.lp = tklp;
        tkz_bits = ezrow[tkid];
      }
    }

    // ---- statistics, row by row (PackedRowStat), in the order the chunks were requested -------
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
      const int a = __builtin_amdgcn_readlane(a_vec, r);
      const bool live = (a >= 0 && a < p.V);
      // RAGGED: the row in its frame: h entries in front of it, nvec blocks in all, the last one
      // (block vl = chunk il of thread tl) holding t of the row's entries
      const int h = head_of(row0 + r);
      const int nvec = RAGGED ? (h + p.V + 7) >> 3 : nvec_aligned;
      const int vl = nvec - 1, il = vl / kMThreads, tl = vl - il * kMThreads, t = h + p.V - 8 * vl;
      const int avec = (a + h) >> 3;
      const int ia = live ? avec / kMThreads : -1;             // chunk of the row holding a_t (uniform)
      const bool owner = live && (avec - ia * kMThreads == tid);
      const int sub = (a + h) & 7;
      PackedRowStat<DIAG> ps;
#pragma unroll
      for (int g0 = 0; g0 < RC; g0 += 2) {
        // the sampled token's own term is left out of the sum: -inf in the resident copy,
        // where its chunk is first consumed
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          if (g0 + i == ia) {
            if (owner) buf[r * RC + g0 + i] = patch16(buf[r * RC + g0 + i], sub, 0xFF80u);
          }
          // RAGGED: what the frame holds in front of the row (threads 0..7 of chunk 0) and behind it
          // in its last block is -inf from here on
          if (RAGGED && g0 + i == 0) {
            if (tid < 8 && h > 8 * tid) buf[r * RC] = keep16(buf[r * RC], min(h - 8 * tid, 8), 8);
          }
          if (RAGGED && g0 + i >= RC - kMTailChunks - 1 && g0 + i == il) {
            if (tid == tl && t < 8) buf[r * RC + g0 + i] = keep16(buf[r * RC + g0 + i], 0, t);
          }
        }
        u32x4 v[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          v[i] = buf[r * RC + g0 + i];
          // lanes past the row loaded 0: make them -inf (only the last chunks can have any)
          if (g0 + i >= RC - kMTailChunks && (g0 + i) * kMThreads + tid >= nvec) v[i] = neg_inf;
        }
        ps.add2(v[0], v[1]);
      }
      // wave-level combine: common offset = the smallest one, rescaling is exact
      const float bw = -wave_max(-ps.b);
      const double dw = static_cast<double>(bw - ps.b), scw = static_cast<double>(fast_exp2(bw - ps.b));
      const double st = ps.sd, tt = static_cast<double>(ps.tsum());
      const double sw = wave_sum(st * scw);
      const double tw = DIAG ? wave_sum(scw * (tt + dw * st)) : 0.0;
      if (lane == 0) { sh_b[r][wid] = bw; sh_s[r][wid] = sw; sh_t[r][wid] = tw; }
    }

    // ---- epilogues: wave r takes row r; the part that needs the row's inputs only comes before
    // the barrier, while the other waves are still on their way to it ---------------------------
    RowPre pre;
    // With the diagnostics the float64 arithmetic of the epilogue finds no registers beside the
    // resident group: an epilogue wave parks its last chunks in shared memory around it (its own
    // 16 bytes per lane and chunk, no synchronisation) instead of spilling to scratch memory.
    constexpr int kPark = DIAG ? (NCHUNK > 32 ? (RAGGED ? 24 : 20) : 16) : 0;
    __shared__ u32x4 sh_park[kPark > 0 ? ROWS * kPark * kWave : 1];
    if (kPark > 0 && wid < ROWS) {
#pragma unroll
      for (int i = 0; i < kPark; ++i) sh_park[(wid * kPark + i) * kWave + lane] = buf[NCHUNK - 1 - i];
    }
    if (wid < ROWS) {
      asm volatile("" : "+v"(za_bits), "+v"(packed_scalars), "+v"(tkz_bits), "+v"(tk.lp), "+v"(tk.id));
      unpack_row_scalars(packed_scalars, rs);
      rs.za = __uint_as_float(za_bits << 16);
      tk.z = __uint_as_float(tkz_bits << 16);
      if (elive) pre = row_pre(rs, tk, p.K > 0, p.relax_log_alpha);
    }
    if (tid == 0) sh_grp[par] = more ? drawn : kNone;
    __syncthreads();
    const int next2 = uniform_i(sh_grp[par]);
    par ^= 1;
    RowOut ro;
    if (wid < ROWS) {
      RowCoef rc;
      rc.coef = 0.f; rc.kexp = 0.f; rc.g_a = 0.f;
      if (elive) {
        const int w_r = wid < ROWS ? wid : 0;
        // the offset must also cover z[a_t], whose own term the epilogue adds
        float bb = -ceilf(fmaxf(rs.za, kNegBig) * kLog2e);
#pragma unroll
        for (int w = 0; w < NW; ++w) bb = fminf(bb, sh_b[w_r][w]);
        double S_rest = 0.0, T_rest = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          const double dd = static_cast<double>(bb - sh_b[w_r][w]), sc = static_cast<double>(fast_exp2(bb - sh_b[w_r][w]));   // exact power of two
          S_rest += sh_s[w_r][w] * sc;
          if (DIAG) T_rest += sc * (sh_t[w_r][w] + dd * sh_s[w_r][w]);
        }
        const RowResult rr = row_post(ep, erow, pre, ea, ezrow, bb, S_rest, T_rest, lane, 0.0, ro);
        rc = rr.rc;
        if (lane == 0) p.row_loss[erow] = rr.loss_term;
      } else if (ewave && lane == 0) {
        // ignored row (sampled id outside the vocabulary): all outputs zero
        p.divergence[erow] = 0.f;
        p.mask[erow] = 0;
        if (p.loss_tok) p.loss_tok[erow] = 0.f;
        if (p.diag) {
          for (int k = 0; k < 8; ++k) p.diag[static_cast<int64_t>(erow) * 8 + k] = 0.f;
        }
        p.row_loss[erow] = 0.0;
      }
      if (lane == 0) sh_rc[wid < ROWS ? wid : 0] = rc;
      if (kPark > 0) {
#pragma unroll
        for (int i = 0; i < kPark; ++i) buf[NCHUNK - 1 - i] = sh_park[(wid * kPark + i) * kWave + lane];
      }
    }
    __syncthreads();
    // the per-token outputs leave after the other waves have been released
    if (elive) {
      int row_e = erow;
      asm volatile("" : "+s"(row_e));
      row_store(ep, row_e, ro, lane);
    }

    // ---- gradient out (one run of stores), next group in (one run of loads) --------------------
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
      const int row = row0 + r;
      const bool ok = row < p.T;
      const float coef = uniform_f(sh_rc[r].coef), kexp = uniform_f(sh_rc[r].kexp);
      char* gr = grad + (ok ? row : 0) * pitch;
      // RAGGED: the 16-byte stores cover the row's complete blocks only: the view ends in front of
      // an incomplete last block, and the threads holding the blocks in front of the row's first
      // complete one give their store an offset out of range, so that it is dropped.
      const int h = ok ? head_of(row) : 0;
      const row_desc_t gout = RAGGED ? make_row_desc(gr - 2 * h, ok ? static_cast<uint32_t>((h + p.V) >> 3) * 16u : 0u)
                                     : make_row_desc(gr, ok ? row_bytes : 0u);
      const uint32_t voff0 = (RAGGED && tid < 8 && h > 8 * tid) ? 0x80000000u : voff;
      const uint32_t sgn = (coef < 0.f) ? 0x80008000u : 0u;
      if (coef == 0.f) {
        // masked, zero-advantage or ignored row: exact zeros (2^-inf) whatever the logits hold
#pragma unroll
        for (int i = 0; i < RC; ++i) buf[r * RC + i] = neg_inf;
      }
      if (RAGGED && ok) {
        // the row's own entries of an incomplete first / last block, two bytes at a time
        const row_desc_t gex = make_row_desc(gr, row_bytes);
        const int vl = ((h + p.V + 7) >> 3) - 1, il = vl / kMThreads, tl = vl - il * kMThreads, t = h + p.V - 8 * vl;
        if (tid == (h >> 3) && (h & 7) != 0) store_entries_untracked(gex, grad8(buf[r * RC], kexp, sgn), h & 7, 8, 8 * (h >> 3) - h);
#pragma unroll
        for (int c = (RC > kMTailChunks + 1 ? RC - kMTailChunks - 1 : 0); c < RC; ++c) {
          if (c == il) {
            if (tid == tl && t < 8) store_entries_untracked(gex, grad8(buf[r * RC + c], kexp, sgn), 0, t, 8 * vl - h);
          }
        }
      }
#pragma unroll
      for (int i = 0; i < RC; ++i) row_store16_untracked(gout, i == 0 ? voff0 : voff, i * kStride, grad8(buf[r * RC + i], kexp, sgn));
    }
    // (a refill can only reuse its chunk's registers once the store has been given them)
    __builtin_amdgcn_sched_barrier(0);
    load_group(next, more);
    __builtin_amdgcn_sched_barrier(0);
    // The resident copies held -inf at the sampled tokens, so the vector stores wrote 0 there.  Once
    // those have completed, the owning threads write the sampled tokens' entries.
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
      const int a = __builtin_amdgcn_readlane(a_vec, r);
      if (a >= 0 && a < p.V && (((a + head_of(row0 + r)) >> 3) & (kMThreads - 1)) == tid) {
        if (sh_rc[r].coef != 0.f) {
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          reinterpret_cast<uint16_t*>(grad + (row0 + r) * pitch)[a] = float_to_bf16_bits(sh_rc[r].g_a);
        }
      }
    }
    grp = next;
    next = next2;
  }
}

}  // namespace

// (rows per group, chunks per row): rows of up to 24576, 32768, 40960, 49152, 57344, 65536 entries,
// each taken with less than two chunks of slack (lanes past the end of a row idle: at a quarter of
// slack the form measured no faster than one row per workgroup).  (Eight rows of up to 16384 entries
// measured 4 % faster than one row per workgroup only from 64 groups per compute unit on: not
// instantiated.)
#define DPPO_MULTI_SHAPES(X) X(6, 6) X(4, 8) X(3, 10) X(3, 12) X(2, 14) X(2, 16)

// Rows per group and chunks per row for a row of V entries, false where this form does not apply.
bool resident_multi_shape(int64_t V, bool ragged, int* rows, int* chunks) {
  if (!ragged && V % 8 != 0) return false;
  // 16-byte blocks of a row; of a row's frame (ragged): between these two, by where in a 128-byte line the row starts
  const int64_t nvec_min = ragged ? (V + 7) / 8 : V / 8, nvec_max = ragged ? (V + 70) / 8 : V / 8;
  // (the kernel would also take a frame that ends exactly with chunk C - kMTailChunks - 1; with two
  // chunks of slack it is no faster than one row per workgroup, so the host does not ask for that)
#define DPPO_TRY(R, C) if (nvec_max <= static_cast<int64_t>(kMThreads) * C) { *rows = R; *chunks = C; return nvec_min > static_cast<int64_t>(kMThreads) * (C - kMTailChunks); }
  DPPO_MULTI_SHAPES(DPPO_TRY)
#undef DPPO_TRY
  return false;
}

hipError_t launch_resident_multi(const KParams& p, bool ragged, int rows, int chunks, int grid, hipStream_t s) {
  if (!p.grad || !p.row_loss || !p.row_counters) return hipErrorInvalidValue;
  const bool diag = p.diag != nullptr;
  const dim3 g(grid), b(kMThreads);
#define DPPO_FORM(R, C, D, G) hipLaunchKernelGGL((dppo_resident_multi_kernel<R, C, D, G>), g, b, 0, s, p)
#define DPPO_LAUNCH(R, C) \
  if (rows == R && chunks == C) { \
    if (ragged) { if (diag) DPPO_FORM(R, C, true, true); else DPPO_FORM(R, C, false, true); } \
    else        { if (diag) DPPO_FORM(R, C, true, false); else DPPO_FORM(R, C, false, false); } \
    return hipGetLastError(); \
  }
  DPPO_MULTI_SHAPES(DPPO_LAUNCH)
#undef DPPO_LAUNCH
#undef DPPO_FORM
  return hipErrorInvalidValue;
}

}  // namespace dppo
