// Register-resident kernel: fused forward+backward, or forward only.
//
// One persistent workgroup per compute unit owns one row at a time and keeps the whole bf16
// row packed in its vector registers (V = 151936 is 297 KiB; a CU's register file is 512 KiB),
// so the logits are read from HBM exactly once and the gradient written exactly once:
//
//   phases A+B  online over groups of chunks: packed-integer maximum (no unpacking), then
//               sum of 2^(z*log2e + b) in fp32 with an integer offset b
//               -> one LDS exchange + barrier -> per-token epilogue on wave 0 -> barrier
//   phase C     gradient of every resident element, 16-byte stores, the whole row in one run of
//               stores; then the workgroup's NEXT row is requested into the same registers in one
//               run of loads, which travel while the statistics of that row start.  (Refilling
//               each chunk right behind its store, so that reads and writes alternate one by one,
//               measured 3.5 % slower: the memory system prefers them in bursts.)
//   forward only: no phase C; the first half of the registers is refilled mid-row, the second
//               after the epilogue, so at least half a row is in flight at any time.
//
// Shorter rows use the same code in smaller shapes: several workgroups of 256 threads per compute
// unit (V up to 40960), and for rows of up to 8192 entries ONE WAVE per row (64 threads), many of
// them per compute unit, each running its own row's epilogue.
//
// Preconditions (checked by the host): V % 8 == 0, V/8 <= THREADS*NCHUNK, logits and
// grad_logits 16-byte aligned with ld % 8 == 0.  The RAGGED form lifts the alignment conditions
// (any V, any pitch, rows 2-byte aligned, logits and grad_logits sharing their misalignment): it
// works on the aligned FRAME of a row, the 16-byte blocks from the start of the 128-byte line that
// holds its first entry to the block that holds its last.
#include "dppo_common.hpp"
#include "dppo_launch.hpp"
#include "dppo_resident_parts.hpp"

namespace dppo {
namespace {

// Chunks whose lanes can lie past the end of the row: with NCHUNK a multiple of kChunkStep (or
// the maximum), at most the last kChunkStep of them.
constexpr int kChunkStep = 4;

// The kernel.  THREADS x NCHUNK 16-byte vectors cover the row (V/8 <= THREADS*NCHUNK, with less
// than kChunkStep chunks of slack).  Chunk i of thread tid is vector i*THREADS + tid of the row.
// All row traffic goes through range-checked buffer resources, so the phases are straight-line
// code with a fixed sequence of memory instructions: loads past the row return 0 (turned into
// -inf where the row statistics consume them) and stores past it are dropped.
// GRAD = false is the forward-only form: no gradient, no stores, refills in two halves.
// DIAG = true also accumulates sum e*x for the entropy diagnostic (two more instructions per
// element in the statistics loop), selected when the caller passes a diagnostics buffer.
// DYN = true: rows are handed out at run time.  With one workgroup per compute unit and rows fixed
// by the workgroup index, the kernel ends when its slowest compute unit does, and the dies do not
// run at one speed (measured on the headline shape: four of the eight dies finish 2.5 % after the
// other four, the last workgroup 2.5 % after the mean).  So a workgroup takes its next row from a
// counter (rows in the order they are asked for: one counter per die over a contiguous eighth of
// the rows, with stealing at the end, measured 1.5 % slower than this).  The row after next is
// requested one row ahead (one thread, an atomic that returns while the row streams) and
// published through shared memory at the row's barrier.  The loss terms go to one slot per ROW,
// so the scalar loss does not depend on which workgroup took which row.
// Waves per SIMD the register allocation must leave room for: the 512-thread shapes are one
// workgroup of two waves per SIMD, except the shortest (12 chunks: 48 registers of row data; left
// to itself the compiler takes 130 registers, two over the limit for a second workgroup per compute
// unit, which is worth 8-14 % on those rows of 96 KiB); the 256-thread shapes (one wave per SIMD
// and workgroup) keep four workgroups per compute unit up to 12 chunks (the 12-chunk shape too
// compiled to 130 registers: +3..8 % on rows of 36-48 KiB) and three with 16 chunks (a budget of 168
// registers; left to itself the compiler lands within a register or two of that limit, on either
// side; a fourth workgroup there, 128 registers, spills and measured 7-12 % slower).
constexpr int resident_min_waves(int threads, int nchunk) { return threads == 512 ? (nchunk <= 12 ? 4 : 2) : (nchunk <= 12 ? 4 : nchunk <= 16 ? 3 : 2); }

// RAGGED = true: rows that do not start on a 16-byte boundary or whose length is not a multiple
// of 8 (a vocabulary of 50257 entries; a pitch that is not a multiple of 8), and rows that start
// on one but not on a 128-byte line.  A row is then handled in its FRAME: the 16-byte blocks from
// the start of the 128-byte line holding its first entry to the block holding its last, so that
// every wave-level access of 1 KiB is eight whole lines, as with aligned rows (a frame that starts
// at the row's own first block, wherever in a line that is, measured 6-9 % slower: nine lines per
// access, partial lines at both ends of a store).  With h = (row address mod 128) / 2 the row
// occupies entries h .. h+V-1 of the frame; what the frame holds in front of the row (up to 126
// bytes: the end of the previous row, pad columns, or bytes in front of the first row) and in its
// last block behind it (and up to 2 bytes behind the last row) lies within an aligned line
// that holds row data, so in mapped memory; it is read, turned into -inf in the resident copy,
// and never written: of the gradient only complete blocks of the row's own entries leave as
// 16-byte stores, an incomplete first or last block as 2-byte stores of the row's own entries.
template <int THREADS, int NCHUNK, bool GRAD, bool DIAG, bool DYN, bool RAGGED>
__global__ __launch_bounds__(THREADS, resident_min_waves(THREADS, NCHUNK)) void dppo_resident_kernel(const KParams p) {
  static_assert(NCHUNK <= 40, "the chunk switch below is written out for up to 40 chunks");
  constexpr int NW = THREADS / kWave;
  // Forward only, the row loads are marked non-temporal (measured 3.5 % faster on the headline shape);
  // with the gradient stores in the mix the same mark measured 4 % slower, so there they are plain.
  constexpr bool kNtLoads = !GRAD;
  constexpr uint32_t kStride = THREADS * 16u;   // bytes between a thread's consecutive chunks
  constexpr int GC = 2;                          // chunks per group of the online row statistics (PackedRowStat::add2)
  constexpr int kSplit = ((NCHUNK / 2 + GC - 1) / GC) * GC;   // forward only: chunks refilled mid-row
  // Per-wave statistics, two sets used by alternate rows: forward only there is no barrier behind
  // wave 0's epilogue, so the other waves may already publish the next row's statistics while
  // wave 0 still reads this row's.  (A third row cannot follow before wave 0 has passed the next
  // row's barrier, i.e. has finished with this set.)
  __shared__ float sh_b[2][NW];
  __shared__ double sh_s[2][NW], sh_t[2][NW];
  __shared__ RowCoef sh_rc;
  __shared__ int sh_row[2];
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
  double loss_acc = 0.0;                        // meaningful in wave 0 only

  // The resident row.
  u32x4 buf[NCHUNK];
  // Workgroup ids go round-robin over the 8 dies.  With the gradient and one workgroup per compute
  // unit, the workgroups of one die take neighbouring rows (die d: rows d*G/8 .. (d+1)*G/8 - 1 of
  // every G, G = workgroups): measured 1.7 % faster on the headline shape than row = workgroup
  // id.  The shapes with several workgroups per compute unit and the forward-only form measure
  // 1-3 % slower that way and keep row = workgroup id.
  int row = (GRAD && THREADS == 512) ? first_row_of_workgroup() : static_cast<int>(blockIdx.x);
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
    // A workgroup that starts when every row has been handed out (the launch need not be resident
    // all at once) has nothing to do, and must not form an address from "no row".
    if (row >= p.T) return;
  }
  // Fetched one row ahead, so that neither the row loop nor wave 0's gathers ever wait on a load
  // that queues behind the row's own refills: the sampled id, and (wave 0, lane k < K) the id
  // and log-prob of top-K entry k.  (For the first row too they are requested BEFORE the row: the
  // compiler places one wait at the head of the loop for both ways into it, and it is as long as
  // the longer of the two.)
  int a_next = p.sampled[row];
  int tkid_next = -1;
  float tklp_next = 0.f;
  if (wid == 0 && lane < p.K) {
    tkid_next = p.tk_ids[static_cast<int64_t>(row) * p.K + lane];
    tklp_next = p.tk_lp[static_cast<int64_t>(row) * p.K + lane];
  }
  __builtin_amdgcn_sched_barrier(0);
  // RAGGED: entries of the frame in front of the row, 0..63 (else 0)
  auto head_of = [&](int r) -> int {
    return RAGGED ? static_cast<int>(((reinterpret_cast<uintptr_t>(logits) + static_cast<uint64_t>(r * pitch)) >> 1) & 63u) : 0;
  };
  // View of a row for loading (has = false: of zero bytes).  RAGGED: of its frame, up to the end of
  // the 4-byte word holding the row's last entry (the range check works per word).
  auto load_view = [&](int r, bool has) -> row_rsrc_t {
    if (!RAGGED) return make_row_rsrc(logits + r * pitch, has ? row_bytes : 0u);
    const int h = head_of(r);
    return make_row_rsrc(logits + r * pitch - 2 * h, has ? ((static_cast<uint32_t>(h + p.V) * 2u + 3u) & ~3u) : 0u);
  };
  {
    const row_rsrc_t zr = load_view(row, true);
#pragma unroll
    for (int i = 0; i < NCHUNK; ++i) buf[i] = row_load16<kNtLoads>(zr, voff, i * kStride);
  }

  for (; row < p.T;) {
    const int a = uniform_i(a_next);
    const bool more = next < p.T;
    if (more) a_next = p.sampled[next];
    // DYN: request the row after next now; the answer is looked at before this row's barrier.
    int drawn = 0;
    if (DYN && more && tid == 0) drawn = atomicAdd(p.row_counters, 1);
    int next2 = kNoRow;
    // thread 0, before the barrier the others read it behind (a number >= T means: no row)
    auto publish_row_after_next = [&]() { sh_row[par] = more ? drawn : kNoRow; };
    const int tkid = tkid_next;
    const float tklp = tklp_next;
    if (more && wid == 0 && lane < p.K) {
      tkid_next = p.tk_ids[static_cast<int64_t>(next) * p.K + lane];
      tklp_next = p.tk_lp[static_cast<int64_t>(next) * p.K + lane];
    }
    const bool live = (a >= 0 && a < p.V);
    const uint16_t* zrow = p.logits + static_cast<int64_t>(row) * p.ld;
    // The workgroup's next row; without one the refills go through a resource of zero bytes:
    // their loads touch no memory.
    const row_rsrc_t zn = load_view(more ? next : row, more);
    // RAGGED: the row in its frame: h entries in front of it, nvec 16-byte blocks in all, the last
    // one (block vl = chunk il of thread tl, il among the last kChunkStep + 1 chunks) holding t of
    // the row's entries.
    const int h = head_of(row);
    const int nvec = RAGGED ? (h + p.V + 7) >> 3 : nvec_aligned;
    const int vl = nvec - 1, il = vl / THREADS, tl = vl - il * THREADS, t = h + p.V - 8 * vl;
    const int avec = (a + h) >> 3;
    const int ia = live ? avec / THREADS : -1;               // chunk holding a_t (uniform)
    const bool owner = live && (avec - ia * THREADS == tid);
    const int sub = (a + h) & 7;

    RowCoef rc;
    rc.coef = 0.f; rc.kexp = 0.f; rc.g_a = 0.f;
    if (live) {
      // Inputs of the epilogue, requested now so that they have arrived when it runs.
      RowScalars rs;
      TopkLane tk;
      tk.id = -1; tk.lp = 0.f; tk.z = 0.f;
      rs.a = a; rs.za = 0.f; rs.lmu = 0.f; rs.adv = 0.f; rs.lanc = 0.f;
      // (The two gathered logits stay raw bit patterns until the statistics are through: their
      // first use, be it a shift, placed up here would be a wait for every refill in front of them.)
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
      // ---- phases A+B, online over groups of GC chunks (PackedRowStat) -------------------------
      // The first groups were loaded first, so their arithmetic hides the latency of the chunks
      // requested last.
      PackedRowStat<DIAG> ps;
#pragma unroll
      for (int g0 = 0; g0 < NCHUNK; g0 += GC) {
        // The sampled token's own term is left out of the sum (see row_epilogue): overwrite it
        // with -inf in the resident copy, right where its chunk is first consumed.  `ia` is
        // uniform: a scalar test per chunk, the patch itself runs once per row.
#pragma unroll
        for (int i = 0; i < GC; ++i) {
          if (g0 + i < NCHUNK && g0 + i == ia) {
            if (owner) buf[g0 + i < NCHUNK ? g0 + i : 0] = patch16(buf[g0 + i < NCHUNK ? g0 + i : 0], sub, 0xFF80u);
          }
          // RAGGED: what the frame holds in front of the row (in its first eight blocks at most: threads
          // 0..7 of chunk 0) and behind it in its last block is -inf from here on
          if (RAGGED && g0 + i == 0) {
            if (tid < 8 && h > 8 * tid) buf[0] = keep16(buf[0], min(h - 8 * tid, 8), 8);
          }
          if (RAGGED && g0 + i < NCHUNK && g0 + i >= NCHUNK - kChunkStep - 1 && g0 + i == il) {
            if (tid == tl && t < 8) buf[g0 + i < NCHUNK ? g0 + i : 0] = keep16(buf[g0 + i < NCHUNK ? g0 + i : 0], 0, t);
          }
        }
        u32x4 v[GC];
#pragma unroll
        for (int i = 0; i < GC; ++i) {
          const int c = (g0 + i < NCHUNK) ? g0 + i : NCHUNK - 1;
          v[i] = (g0 + i < NCHUNK) ? buf[c] : neg_inf;
          // lanes past the row loaded 0: make them -inf (only the last chunks can have any)
          if (g0 + i < NCHUNK && g0 + i >= NCHUNK - kChunkStep && c * THREADS + tid >= nvec) v[i] = neg_inf;
        }
        ps.add2(v[0], v[1]);
        // Forward only: nothing needs the row after its statistics, so the first part of the
        // registers is refilled from the next row as soon as it has been consumed.  Those loads
        // are in flight during the rest of this row and its epilogue; the rest is refilled after
        // the epilogue and is in flight during the first part of the next row's statistics.
        if (!GRAD && g0 + GC == kSplit) {
#pragma unroll
          for (int i = 0; i < kSplit; ++i) buf[i] = row_load16<kNtLoads>(zn, voff, i * kStride);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // wave-level combine: common offset = the smallest one, rescaling is exact
      const float bw = -wave_max(-ps.b);
      const double dw = static_cast<double>(bw - ps.b), scw = static_cast<double>(fast_exp2(bw - ps.b));
      const double st = ps.sd, tt = static_cast<double>(ps.tsum());
      const double sw = wave_sum(st * scw);
      const double tw = DIAG ? wave_sum(scw * (tt + dw * st)) : 0.0;
      if (lane == 0) { sh_b[par][wid] = bw; sh_s[par][wid] = sw; sh_t[par][wid] = tw; }
      // Wave 0: the part of the epilogue that needs the row's inputs only (every exponential),
      // before the barrier: the other waves are still on their way to it.
      // Shapes whose row data alone leaves room for one workgroup per compute unit: nothing
      // hides a call there, so the epilogue is inlined, in its two parts.  The shorter shapes keep
      // the call and with it the second or third workgroup per compute unit.
      constexpr bool kInlineEpilogue = (THREADS == 512 && NCHUNK >= (GRAD ? 16 : 28));
      RowPre pre;
      // With the gradient the whole row is still needed after the epilogue, whose float64 arithmetic
      // finds no registers beside it: wave 0 parks its last chunks in shared memory around the
      // epilogue (its own 16 bytes per lane and chunk, no synchronisation) instead of letting the
      // compiler spill to scratch memory, whose round trips would sit on the path the other seven
      // waves wait for (measured on the headline shapes: 1.8 % faster Binary, 3.6 % faster Top-K;
      // 8, 16 and 24 chunks measure the same).
      constexpr int kPark = (GRAD && kInlineEpilogue) ? 16 : 0;
      __shared__ u32x4 sh_park[kPark > 0 ? kPark * kWave : 1];
      if (kPark > 0 && wid == 0) {
#pragma unroll
        for (int i = 0; i < kPark; ++i) sh_park[i * kWave + lane] = buf[NCHUNK - 1 - i];
      }
      if (wid == 0) {
        asm volatile("" : "+v"(za_bits), "+v"(packed_scalars), "+v"(tkz_bits), "+v"(tk.lp), "+v"(tk.id));
        unpack_row_scalars(packed_scalars, rs);
        rs.za = __uint_as_float(za_bits << 16);
        tk.z = __uint_as_float(tkz_bits << 16);
      }
      if (GRAD && kInlineEpilogue && wid == 0) pre = row_pre(rs, tk, p.K > 0, p.relax_log_alpha);
      if (DYN && tid == 0) publish_row_after_next();
      __syncthreads();
      if (!GRAD && kInlineEpilogue && wid == 0) pre = row_pre(rs, tk, p.K > 0, p.relax_log_alpha);
      if (DYN) next2 = uniform_i(sh_row[par]);
      // ---- epilogue on wave 0 -----------------------------------------------------------
      RowOut ro;
      if (wid == 0) {
        // the offset must also cover z[a_t], whose own term the epilogue adds
        float bb = -ceilf(fmaxf(rs.za, kNegBig) * kLog2e);
#pragma unroll
        for (int w = 0; w < NW; ++w) bb = fminf(bb, sh_b[par][w]);
        double S_rest = 0.0, T_rest = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          const double dd = static_cast<double>(bb - sh_b[par][w]), sc = static_cast<double>(fast_exp2(bb - sh_b[par][w]));   // exact power of two
          S_rest += sh_s[par][w] * sc;
          if (DIAG) T_rest += sc * (sh_t[par][w] + dd * sh_s[par][w]);
        }
        RowResult rr;
        if (kInlineEpilogue) {
          rr = row_post(ep, row, pre, a, zrow, bb, S_rest, T_rest, lane, 0.0, ro);
        } else {
          int row_e = row;
          asm volatile("" : "+s"(row_e));
          rr = row_epilogue_call(ep, row_e, rs, tk, zrow, bb, S_rest, T_rest, lane);
        }
        rc = rr.rc;
        if (DYN) { if (lane == 0) p.row_loss[row] = rr.loss_term; }
        else loss_acc += rr.loss_term;
        if (GRAD && lane == 0) sh_rc = rc;
        if (kPark > 0) {
#pragma unroll
          for (int i = 0; i < kPark; ++i) buf[NCHUNK - 1 - i] = sh_park[i * kWave + lane];
        }
      }
      par ^= 1;
      if (GRAD) {
        __syncthreads();
        rc.coef = uniform_f(sh_rc.coef);
        rc.kexp = uniform_f(sh_rc.kexp);
        rc.g_a = uniform_f(sh_rc.g_a);
      }
      // The per-token outputs leave after the other waves have been released.  The row index goes
      // through an empty asm statement first, so that the output addresses are formed here and not
      // hoisted to the top of the row, where they would sit in registers across the streaming phases.
      if (kInlineEpilogue && wid == 0) {
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

    // ---- phase C: gradient out, next row in -------------------------------------------------
    // Store the gradient of every chunk, then refill the chunks with the workgroup's next row,
    // in the order the next row's arithmetic will consume them.
    if (GRAD) {
      char* gr = grad + row * pitch;
      // RAGGED: the 16-byte stores cover the row's complete blocks only: the view ends in front of
      // an incomplete last block, and the threads holding the blocks in front of the row's first
      // complete one give their store an offset out of range, so that it is dropped.
      const row_desc_t gout = RAGGED ? make_row_desc(gr - 2 * h, static_cast<uint32_t>((h + p.V) >> 3) * 16u) : make_row_desc(gr, row_bytes);
      const uint32_t voff0 = (RAGGED && tid < 8 && h > 8 * tid) ? 0x80000000u : voff;
      const uint32_t sgn = (rc.coef < 0.f) ? 0x80008000u : 0u;
      if (rc.coef == 0.f) {
        // Masked, zero-advantage or ignored row: its gradient is exactly zero whatever the logits
        // hold.  Overwrite the resident copy with -inf so that the loop below writes 2^-inf = 0.
#pragma unroll
        for (int i = 0; i < NCHUNK; ++i) buf[i] = neg_inf;
      }
      if (RAGGED) {
        // the row's own entries of an incomplete first / last block, two bytes at a time
        const row_desc_t gex = make_row_desc(gr, row_bytes);
        if (tid == (h >> 3) && (h & 7) != 0) store_entries_untracked(gex, grad8(buf[0], rc.kexp, sgn), h & 7, 8, 8 * (h >> 3) - h);
#pragma unroll
        for (int c = (NCHUNK > kChunkStep + 1 ? NCHUNK - kChunkStep - 1 : 0); c < NCHUNK; ++c) {
          if (c == il) {
            if (tid == tl && t < 8) store_entries_untracked(gex, grad8(buf[c], rc.kexp, sgn), 0, t, 8 * vl - h);
          }
        }
      }
#pragma unroll
      for (int i = 0; i < NCHUNK; ++i) row_store16_untracked(gout, i == 0 ? voff0 : voff, i * kStride, grad8(buf[i], rc.kexp, sgn));
      // Keep the instruction scheduler from hoisting the refills above the stores: a refill can
      // only reuse its chunk's registers once the store has been given them (a vector-memory load
      // into those registers then queues behind that store).
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < NCHUNK; ++i) buf[i] = row_load16<kNtLoads>(zn, voff, i * kStride);
      __builtin_amdgcn_sched_barrier(0);
      if (rc.coef != 0.f && owner) {
        // The resident copy held -inf at a_t, so the vector store above wrote 0 there.  Once
        // that store has completed, the owning thread writes the sampled token's entry.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        reinterpret_cast<uint16_t*>(gr)[a] = float_to_bf16_bits(rc.g_a);
      }
    } else {
      // rows whose statistics ran refilled the first part there
#pragma unroll
      for (int i = 0; i < NCHUNK; ++i)
        if (i >= kSplit || !live) buf[i] = row_load16<kNtLoads>(zn, voff, i * kStride);
    }
    row = next;
    next = DYN ? next2 : next + static_cast<int>(gridDim.x);
  }
  if (!DYN && tid == 0) p.partial[blockIdx.x] = loss_acc;
}

// One instantiation per (threads, chunks) shape; chunks in steps of kChunkStep up to the maximum.
// Rows of up to 8192 entries belong to ONE wave each (64 threads: a workgroup's barriers cost nothing,
// no wave waits for another one's epilogue, and 12-20 independent rows are in flight per compute
// unit); measured against the two-pass kernel at V = 4096: 4.5 against 2.0 TB/s, and at V = 8192
// against 256 threads x 4 chunks: 4.9 against 4.1 TB/s.  From 16384 entries on, the 256-thread
// shapes measure the same or better (V = 16384: 4.94 against 4.83 TB/s with 64 threads x 32 chunks).
// Rows are handed out at run time when the host sets p.row_counters.
template <int THREADS, int NCHUNK, bool RAGGED>
hipError_t launch_shape(const KParams& p, bool grad, int grid, hipStream_t s) {
  const bool diag = p.diag != nullptr;
  constexpr bool kDyn = (THREADS == 512);     // the forms with run-time rows exist for the 512-thread shapes, with the gradient
  const bool dyn = kDyn && grad && p.row_counters != nullptr;
  if (p.row_counters != nullptr && !dyn) return hipErrorInvalidValue;
  const dim3 g(grid), b(THREADS);
#define DPPO_FORM(G, D, Y) hipLaunchKernelGGL((dppo_resident_kernel<THREADS, NCHUNK, G, D, Y, RAGGED>), g, b, 0, s, p)
  if (grad) {
    if (diag) { if (dyn) DPPO_FORM(true, true, kDyn); else DPPO_FORM(true, true, false); }
    else      { if (dyn) DPPO_FORM(true, false, kDyn); else DPPO_FORM(true, false, false); }
  } else {
    if (diag) DPPO_FORM(false, true, false); else DPPO_FORM(false, false, false);
  }
#undef DPPO_FORM
  return hipGetLastError();
}
// The diagnostics form needs a few more registers; its occupancy bounds both.
template <int THREADS, int NCHUNK, bool RAGGED>
int occupancy_shape(bool grad, bool dyn) {
  int n = 0;
  constexpr bool kDyn = (THREADS == 512);
  hipError_t e;
  if (grad && dyn && kDyn) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dppo_resident_kernel<THREADS, NCHUNK, true, true, kDyn, RAGGED>, THREADS, 0);
  else if (grad)           e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dppo_resident_kernel<THREADS, NCHUNK, true, true, false, RAGGED>, THREADS, 0);
  else                     e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dppo_resident_kernel<THREADS, NCHUNK, false, true, false, RAGGED>, THREADS, 0);
  return (e == hipSuccess && n > 0) ? n : 1;
}

}  // namespace

#define DPPO_SHAPES(X) \
  X(64, 4) X(64, 8) X(64, 12) X(64, 16) X(256, 4) X(256, 8) X(256, 12) X(256, 16) X(256, 20) \
  X(512, 12) X(512, 16) X(512, 20) X(512, 24) X(512, 28) X(512, 32) X(512, 36) X(512, 38)

bool resident_shape(int64_t V, bool ragged, int* threads, int* chunks) {
  if (V < 1024 || (!ragged && V % 8 != 0)) return false;
  // 16-byte blocks of a row: V / 8; of a row's frame (ragged): between these two, by where in a 128-byte line the row starts
  const int64_t nvec_min = ragged ? (V + 7) / 8 : V / 8, nvec_max = ragged ? (V + 70) / 8 : V / 8;
  // (a shape is only taken with less than kChunkStep chunks of slack: the kernel turns lanes past
  // the row into -inf in its last kChunkStep chunks only)
  // (ragged: the shortest frame may end exactly with chunk C - kChunkStep - 1, whose last block the kernel still looks at)
#define DPPO_TRY(T, C) if (nvec_max <= static_cast<int64_t>(T) * C) { *threads = T; *chunks = C; return nvec_min + (ragged ? 1 : 0) > static_cast<int64_t>(T) * (C - kChunkStep); }
  DPPO_SHAPES(DPPO_TRY)
#undef DPPO_TRY
  return false;
}

hipError_t launch_resident(const KParams& p, bool grad, bool ragged, int threads, int chunks, int grid, hipStream_t s) {
#define DPPO_LAUNCH(T, C) if (threads == T && chunks == C) return ragged ? launch_shape<T, C, true>(p, grad, grid, s) : launch_shape<T, C, false>(p, grad, grid, s);
  DPPO_SHAPES(DPPO_LAUNCH)
#undef DPPO_LAUNCH
  return hipErrorInvalidValue;
}

int resident_blocks_per_cu(bool grad, bool dyn, bool ragged, int threads, int chunks) {
#define DPPO_OCC(T, C) if (threads == T && chunks == C) return ragged ? occupancy_shape<T, C, true>(grad, dyn) : occupancy_shape<T, C, false>(grad, dyn);
  DPPO_SHAPES(DPPO_OCC)
#undef DPPO_OCC
  return 1;
}

}  // namespace dppo
