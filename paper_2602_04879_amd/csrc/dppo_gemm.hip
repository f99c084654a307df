// bf16 matrix product on the matrix cores, C[M, N] = A[M, K] * B[N, K]^T with fp32 accumulation:
// both operands row-major with the contraction index contiguous (what an nn.Linear forward is:
// activations [T, d] times weight [V, d] transposed), C row-major: bf16 rounded to nearest even,
// or fp32, optionally added to what C holds.
//
// One workgroup of 256 threads (4 waves, one per SIMD) per 256 x 256 tile of C, each wave a
// 128 x 128 quadrant as 8 x 8 products of v_mfma_f32_16x16x32_bf16 (256 fp32 accumulators per
// lane, the whole accumulation register file).  That shape is chosen for power: with every
// compute unit busy the clock is set by the power limit, and a loop of nothing but 16x16x32
// products sustains about 13 % more than one of 32x32x16 products (measured, 2.2-2.3 against
// 1.9-2.0 PFLOP/s).  The contraction runs in steps of 64: the A and B panels of a step (256 x 64
// each, 32 KiB) are loaded from global memory straight into one of two LDS stages, 16 bytes per
// lane, in a layout swizzled so that the fragment reads (one 16-byte read per lane: 8 consecutive
// k of one row) spread over all banks.
// A 16x16x32 product occupies the matrix pipe for 16 cycles and a wave issues at most one
// instruction every 4, so whatever else the wave issues has to sit in the shadow of a product:
// the matrix-core instructions are written as assembly statements in a fixed order (that also
// keeps each accumulator in place in its own registers, which the register allocator does not
// manage by itself at this pressure), with one fragment read or one panel load pinned behind
// every second to fourth of them.
// Panel rows past M or N re-read the last valid row (their products are never stored); all
// loads go through range-checked buffer resources over exactly the rows a tile owns.  K must be
// a multiple of 64, rows 16-byte aligned (checked by the host).
//
// A second form of the same kernel takes both operands with the contraction index as the ROW
// index, C[M, N] = A[K, M]^T * B[K, N] (what the gradient of a weight is: logit gradients [T, V]
// transposed times activations [T, d]), with no transposed copies: the panels of a step are 64
// rows of 512 bytes, and the LDS transpose read (ds_read_b64_tr_b16) hands every lane the
// consecutive k of one column.  There K is arbitrary: rows past it read as zeros.
#include <type_traits>
#include "dppo_common.hpp"
#include "dppo_launch.hpp"

namespace dppo {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kRowBytes = kBK * 2;                    // one panel row in LDS: 128 bytes = 8 vectors
constexpr int kPanelBytes = kBM * kRowBytes;          // 32 KiB (kBM == kBN)
constexpr int kStageBytes = 2 * kPanelBytes;          // A panel then B panel

// LDS byte offset of the 16-byte vector `kvec` (0..7) of panel row `row`: the vector index is
// XOR-ed with bits 1..3 of the row, so 16 consecutive rows at one kvec cover all 64 banks once.
__device__ __forceinline__ uint32_t lds_off(int row, int kvec) {
  return static_cast<uint32_t>(row) * kRowBytes + static_cast<uint32_t>((kvec ^ ((row >> 1) & 7)) << 4);
}

// One 256 x 256 tile.  FULL: all 256 rows and columns of the tile exist, so the stores need no
// range checks.  A panel row past the matrix re-reads the last valid row: its products are never stored.
// OUT selects what leaves the tile: bf16 (rounded to nearest even), fp32, or fp32 added to what C holds.
// kOutStats: nothing of C is stored.  The tile's logits, rounded to bf16 as a stored tile would be,
// leave as softmax statistics per row (GemmStats below): the forward of the hidden-state path then
// never writes a logit to memory.
enum : int { kOutBf16 = 0, kOutF32 = 1, kOutF32Add = 2, kOutStats = 3 };

// TA: A is [K, M]; TB: B is [K, N] (the contraction index is the ROW index of that operand; with
// both, C = A^T B; with TB alone, C = A B).  The panel of such an operand
// is then 64 rows of 512 bytes per step, and its fragment reads use the LDS transpose read
// (ds_read_b64_tr_b16: out of a 16-lane group's sixteen 8-byte blocks, lane i gets element i%4 of
// the blocks i/4, i/4 + 4, i/4 + 8, i/4 + 12), which turns four k rows of four neighbouring m
// into the four consecutive k of one m that a matrix-core operand wants.
template <bool FULL, int OUT, bool TA, bool TB>
__device__ __forceinline__ void gemm_tile(unsigned char* lds0, unsigned char* lds1, const uint16_t* __restrict__ A, int64_t lda,
                                          const uint16_t* __restrict__ B, int64_t ldb, void* __restrict__ Cv, int64_t ldc,
                                          int M, int N, int K, int m0, int n0, const GemmStats& gs) {
  const int tid = threadIdx.x, lane = tid & 63, wid = uniform_i(tid >> 6);
  const int wm = wid >> 1, wn = wid & 1;
  const int rows_a = min(kBM, M - m0), rows_b = min(kBN, N - n0);     // (TA / TB: columns of A / of B)
  const uint32_t pitch_a = static_cast<uint32_t>(lda) * 2u, pitch_b = static_cast<uint32_t>(ldb) * 2u;

  // Loader role: thread t moves LDS vector slot (t % 8) of rows t/8 + 32 i, i = 0..7, of each panel;
  // the slot holds global k-vector slot ^ ((row >> 1) & 7), the same for all eight rows.
  const int lrow = tid >> 3, lslot = tid & 7;
  const uint32_t lkv = static_cast<uint32_t>((lslot ^ ((lrow >> 1) & 7)) << 4);

  f32x4 acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;

  // Fragment role: lane holds 8 consecutive k (k quarter `fk` of a 32-wide sub-step) of row `frow`
  // of a 16-row block.  The swizzle depends on the row only through frow, so one offset per
  // k-vector serves every block of both panels.
  const int frow = lane & 15, fk = lane >> 4;
  uint32_t foff[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) foff[ks] = lds_off(frow, ks * 4 + fk);
  const uint32_t fbase_a = static_cast<uint32_t>(wm * 128) * kRowBytes;
  const uint32_t fbase_b = kPanelBytes + static_cast<uint32_t>(wn * 128) * kRowBytes;
  // TN panels: LDS row k (512 bytes = 32 slots of 16 bytes) holds in slot s the 8 columns of
  // global slot s ^ (2 g(k)), g(k) = (k & 3) | ((k >> 3) & 1) << 2: the sixteen k rows one transpose
  // read touches (k = 8 kg + j, kg = lane / 16, j = (lane % 16) / 4) then spread their 32-byte pieces
  // over all banks.  Lane (kg, j, q = lane % 4) reads the 8 bytes of columns 4 q .. 4 q + 3 of block t
  // in row 8 kg + j (+ 4 for the second half of the fragment, + 32 for the second sub-step).
  uint32_t toff_a[8], toff_b[8];
  if (TA || TB) {
    const int kg = lane >> 4, j = (lane >> 2) & 3, q = lane & 3;
    const uint32_t g2 = static_cast<uint32_t>(2 * (j | ((kg & 1) << 2)));
    const uint32_t rowoff = static_cast<uint32_t>(8 * kg + j) * 512u + static_cast<uint32_t>(q & 1) * 8u;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      toff_a[t] = rowoff + ((static_cast<uint32_t>(wm * 16 + 2 * t + (q >> 1)) ^ g2) << 4);
      toff_b[t] = kPanelBytes + rowoff + ((static_cast<uint32_t>(wn * 16 + 2 * t + (q >> 1)) ^ g2) << 4);
    }
  }
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
  // fragment t of a sub-step: 0..7 the B blocks, 8..15 the A blocks
  auto read_frag = [&](const unsigned char* stage, int ks, int t) -> bf16x8 {
    if (t < 8 ? TB : TA) {
      const unsigned char* p = stage + (t < 8 ? toff_b[t & 7] : toff_a[t & 7]) + ks * (32 * 512);
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * 512));
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, v);
    }
    return *reinterpret_cast<const bf16x8*>(stage + (t < 8 ? fbase_b : fbase_a) + (t & 7) * 16 * kRowBytes + foff[ks]);
  };
#define DPPO_MFMA16(ACC, X, Y) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(ACC) : "v"(X), "v"(Y))

  // Pipeline over the contraction: step kt is multiplied out of LDS stage kt % 2; once every wave
  // has read its last fragments of that stage (the barrier in the middle of the step) the panels
  // of step kt+2 are loaded into it.  The fragments of each 32-wide sub-step are read from LDS one
  // sub-step ahead of the matrix-core instructions that consume them.  One barrier per step.
  const int nk = (TA && TB) ? (K + kBK - 1) / kBK : K / kBK;     // both by rows: rows past K read as zeros (range check)
  // Global memory -> LDS directly (buffer_load ... lds): lane l of a wave-level load deposits its
  // 16 bytes at (LDS base of the instruction) + 16 l, which is exactly the loader layout above for
  // the base stage + panel + i * 4096 + wave * 1024.  No staging registers, no LDS store
  // instructions; completion is counted with the other vector-memory loads.
  typedef __attribute__((address_space(3))) void* lds_ptr_t;
  // Load i of a panel moves rows lrow + 32 i (clamped to the last row the tile owns), through a
  // range-checked view of exactly the rows this tile owns.  The k offset of a step goes into the
  // base of that view (scalar arithmetic), so the per-lane offsets never change.
  uint32_t vo_a[8], vo_b[8];
  uint32_t bytes_a, bytes_b;
  // by rows: load i of a panel (one KiB: two LDS rows) moves k rows 8 i + 2 wave + lane / 32, LDS slot lane % 32
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int k = 8 * i + 2 * wid + (lane >> 5);
    const uint32_t gs = static_cast<uint32_t>(lane & 31) ^ static_cast<uint32_t>(2 * ((k & 3) | (((k >> 3) & 1) << 2)));
    vo_a[i] = TA ? static_cast<uint32_t>(k) * pitch_a + (gs << 4) : static_cast<uint32_t>(min(lrow + 32 * i, rows_a - 1)) * pitch_a + lkv;
    vo_b[i] = TB ? static_cast<uint32_t>(k) * pitch_b + (gs << 4) : static_cast<uint32_t>(min(lrow + 32 * i, rows_b - 1)) * pitch_b + lkv;
  }
  // by rows: bytes of a row from the tile's first column on, in whole 16-byte vectors (the range
  // check works per 4 bytes, and the pitch, a multiple of 8 entries, covers them); else: bytes of the tile's rows
  bytes_a = TA ? ((static_cast<uint32_t>(M - m0) * 2u + 15u) & ~15u) : static_cast<uint32_t>(rows_a - 1) * pitch_a + static_cast<uint32_t>(K) * 2u;
  bytes_b = TB ? ((static_cast<uint32_t>(N - n0) * 2u + 15u) & ~15u) : static_cast<uint32_t>(rows_b - 1) * pitch_b + static_cast<uint32_t>(K) * 2u;
  auto dma_one = [&](unsigned char* stage, int step, int idx) {     // load idx of the 16 of a step: 0..7 A panel, 8..15 B panel
    const bool b_panel = idx >= 8;
    const int i = idx & 7;
    unsigned char* dst = stage + (b_panel ? kPanelBytes : 0) + wid * 1024 + i * 4096;
    row_rsrc_t r;
    // By rows: view of the step's k rows (those that exist) from the tile's first column on: what
    // lies past the last row's end reads as zero, what lies past a row's M (N) columns belongs to
    // C rows (columns) that are never stored.  Else: the tile's rows, from the step's k on.
    const int kr = min(kBK, K - step * kBK);
    const uint32_t koff = static_cast<uint32_t>(step) * (kBK * 2);
    if (b_panel) r = TB ? make_row_rsrc(B + static_cast<int64_t>(step) * kBK * ldb + n0, static_cast<uint32_t>(kr - 1) * pitch_b + bytes_b)
                        : make_row_rsrc(B + static_cast<int64_t>(n0) * ldb + step * kBK, bytes_b - koff);
    else         r = TA ? make_row_rsrc(A + static_cast<int64_t>(step) * kBK * lda + m0, static_cast<uint32_t>(kr - 1) * pitch_a + bytes_a)
                        : make_row_rsrc(A + static_cast<int64_t>(m0) * lda + step * kBK, bytes_a - koff);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr_t)dst, 16, b_panel ? vo_b[i] : vo_a[i], 0, 0, 0);
  };
#pragma unroll
  for (int q = 0; q < 16; ++q) dma_one(lds0, 0, q);
  __syncthreads();                       // waits for this wave's loads, then for everyone's
  bf16x8 f0[16], f1[16];      // [0..7] B blocks, [8..15] A blocks
  // fragment q of the read order: the first A block, the 8 B blocks, then the other A blocks
  constexpr int kOrder[16] = {8, 0, 1, 2, 3, 4, 5, 6, 7, 9, 10, 11, 12, 13, 14, 15};
#pragma unroll
  for (int t = 0; t < 16; ++t) f0[t] = read_frag(lds0, 0, t);
  // One step of the contraction out of stage `cur`: two 32-wide sub-steps of 64 matrix-core
  // instructions each (A block i = m / 8 against B block j = m % 8).  Every other instruction sits
  // directly behind a matrix-core instruction, where it issues while that one executes.
  // First sub-step: the 16 fragment reads of the second, behind the first 32 instructions, so they
  // have landed when the barrier is reached.  Second sub-step: the 16 fragment reads of the next
  // step's first sub-step and the 16 panel loads of the step after next.
#define DPPO_PIN __builtin_amdgcn_sched_barrier(0)
  auto step = [&](unsigned char* cur, unsigned char* nxt, int kt, auto steady) {
    constexpr bool STEADY = decltype(steady)::value;
    const bool more = STEADY || kt + 1 < nk, more2 = STEADY || kt + 2 < nk;
#pragma unroll
    for (int m = 0; m < 64; ++m) {
      DPPO_MFMA16(acc[m >> 3][m & 7], f0[m & 7], f0[8 + (m >> 3)]); DPPO_PIN;
      if (m < 32 && (m & 1) == 0) { f1[kOrder[m >> 1]] = read_frag(cur, 1, kOrder[m >> 1]); DPPO_PIN; }
    }
    // the next stage is complete (own loads waited for, then everyone's) and this one fully read
    __syncthreads();
    DPPO_PIN;
#pragma unroll
    for (int m = 0; m < 64; ++m) {
      DPPO_MFMA16(acc[m >> 3][m & 7], f1[m & 7], f1[8 + (m >> 3)]); DPPO_PIN;
      if ((m & 3) == 0) { if (more) f0[kOrder[m >> 2]] = read_frag(nxt, 0, kOrder[m >> 2]); DPPO_PIN; }
      if ((m & 3) == 2) { if (more2) dma_one(cur, kt + 2, m >> 2); DPPO_PIN; }
    }
  };
  if (nk > 1) {
#pragma unroll
    for (int q = 0; q < 16; ++q) dma_one(lds1, 1, q);
  }
  int kt = 0;
  for (; kt + 3 < nk; kt += 2) {
    step(lds0, lds1, kt, std::true_type{});
    step(lds1, lds0, kt + 1, std::true_type{});
  }
  for (; kt + 1 < nk; kt += 2) {
    step(lds0, lds1, kt, std::false_type{});
    step(lds1, lds0, kt + 1, std::false_type{});
  }
  if (kt < nk) step(lds0, lds1, kt, std::false_type{});
  // the matrix-core results must have landed before other instructions read the accumulators
  // (the products are assembly statements, so the compiler does not keep that distance by itself;
  // the scheduling barrier keeps the accumulator reads of the store behind the wait)
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  DPPO_PIN;

  // The products were formed with the operands swapped (B fragment first), so a lane's four
  // accumulators of a 16 x 16 block are four consecutive COLUMNS (lane/16)*4 + 0..3 of row lane%16.
  if (OUT == kOutStats) {
    // ---- softmax statistics of the tile instead of the tile ------------------------------------
    // Per row of the tile, over its 256 columns (those below N), of the logits ROUNDED to bf16:
    // the integer offset b = -ceil(max * log2e), s = sum 2^(z*log2e + b) and t = sum 2^x * x (for
    // the entropy), the row's sampled token left out as in the loss kernels.  A lane holds 32
    // columns of each of its 8 rows; the four lanes of a row (lane, lane+16, +32, +48) combine by
    // shuffles, the two waves of a row through shared memory.  The rounded tile itself goes to
    // shared memory (the two stages are free now: 128 rows of 512 bytes each, 32-byte blocks
    // XOR-ed with the row so that a 16-lane write spreads over the banks), from where the logits at
    // the sampled and the top-K ids that fall into this tile are picked.
    __shared__ float sh_part[2][kBM][3];
    // the sampled ids of the lane's eight rows, requested in one go (one memory latency, which
    // the barrier covers in part, instead of one per row block)
    int samp[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = m0 + wm * 128 + i * 16 + frow;
      samp[i] = (row < M) ? gs.sampled[row] : -1;
    }
    __syncthreads();                       // every wave has read its last fragments: the stages can be overwritten
    unsigned char* half = wm ? lds1 : lds0;
    const int col0 = n0 + wn * 128;        // first column of this wave's quadrant
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int rl = i * 16 + frow;                       // row inside the wave's 128
      const int row = m0 + wm * 128 + rl;
      const int a_loc = (row < M && samp[i] >= 0) ? samp[i] - col0 : -1;
      float z[8][4];
      float mx = -INFINITY;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint32_t lo = pack_bf16x2(acc[i][j][0], acc[i][j][1]), hi = pack_bf16x2(acc[i][j][2], acc[i][j][3]);
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        *reinterpret_cast<u32x2*>(half + rl * 512 + (((wn * 8 + j) ^ frow) << 5) + fk * 8) = u32x2{lo, hi};
        z[j][0] = __uint_as_float(lo << 16); z[j][1] = __uint_as_float(lo & 0xffff0000u);
        z[j][2] = __uint_as_float(hi << 16); z[j][3] = __uint_as_float(hi & 0xffff0000u);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int cl = j * 16 + fk * 4 + e;
          if ((!FULL && col0 + cl >= N) || cl == a_loc) z[j][e] = -INFINITY;
          mx = fmaxf(mx, z[j][e]);
        }
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float b = -ceilf(fmaxf(mx, kNegBig) * kLog2e);
      float s = 0.f, t = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float e4[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float x = fmaf(z[j][e], kLog2e, b);
          e4[e] = fast_exp2(x);
          t = fma_ex(e4[e], x, t);
        }
        s += (e4[0] + e4[1]) + (e4[2] + e4[3]);
      }
      s += __shfl_xor(s, 16); s += __shfl_xor(s, 32);
      t += __shfl_xor(t, 16); t += __shfl_xor(t, 32);
      if (fk == 0) { sh_part[wn][wm * 128 + rl][0] = b; sh_part[wn][wm * 128 + rl][1] = s; sh_part[wn][wm * 128 + rl][2] = t; }
    }
    __syncthreads();
    {
      const int row = m0 + tid;
      const float b0 = sh_part[0][tid][0], b1 = sh_part[1][tid][0], b = fminf(b0, b1);
      const float d0 = b - b0, d1 = b - b1, c0 = fast_exp2(d0), c1 = fast_exp2(d1);       // exact powers of two
      const float s = sh_part[0][tid][1] * c0 + sh_part[1][tid][1] * c1;
      const float t = c0 * fmaf(d0, sh_part[0][tid][1], sh_part[0][tid][2]) + c1 * fmaf(d1, sh_part[1][tid][1], sh_part[1][tid][2]);
      if (row < M) gs.part[static_cast<int64_t>(row) * gs.tiles_n + n0 / kBN] = f32x4{b, s, t, 0.f};
    }
    // the rounded logits at the rows' sampled and top-K ids that fall into this tile; ids fetched
    // four at a time (one memory latency per four entries)
    const int K1 = gs.Ktop + 1;
    for (int idx0 = tid; idx0 < kBM * K1; idx0 += 4 * 256) {
      int id[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = idx0 + u * 256, rl = idx / K1, k = idx - rl * K1, row = m0 + rl;
        id[u] = -1;
        if (idx < kBM * K1 && row < M) id[u] = (k == 0) ? gs.sampled[row] : gs.tk_ids[static_cast<int64_t>(row) * gs.Ktop + (k - 1)];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = idx0 + u * 256, rl = idx / K1, k = idx - rl * K1, row = m0 + rl;
        const int c = id[u] - n0;
        if (id[u] >= 0 && c >= 0 && c < kBN && id[u] < N) {
          const unsigned char* src = ((rl >> 7) ? lds1 : lds0) + (rl & 127) * 512 + (((c >> 4) ^ (rl & 15)) << 5) + (c & 15) * 2;
          gs.gath[static_cast<int64_t>(row) * K1 + k] = bf16_bits_to_float(*reinterpret_cast<const uint16_t*>(src));
        }
      }
    }
    return;
  }
  // Store.  bf16: two neighbouring blocks exchange halves between lane rows (one
  // v_permlane16_swap per register pair), after which a lane owns 8 consecutive columns: one
  // 16-byte store, 64 contiguous bytes per row and instruction.  fp32: 16 bytes per lane as they are.
  const bool quad_aligned = ((reinterpret_cast<uintptr_t>(Cv) & 15u) == 0) && (ldc % 8 == 0);
  if (OUT == kOutF32Add && FULL) {
    // C += tile: what C holds is requested one block of 16 rows AHEAD of the block being added and
    // stored (eight 16-byte loads per lane in flight behind eight stores), so that a lane waits for
    // memory eight times per tile and not sixty-four times.  (Written as load - add - store per
    // vector, the compiler keeps that order, every load behind the store in front of it.)
    auto cptr = [&](int i, int j) {
      const int row = m0 + wm * 128 + i * 16 + frow, col = n0 + wn * 128 + j * 16 + fk * 4;
      return reinterpret_cast<f32x4*>(static_cast<float*>(Cv) + static_cast<int64_t>(row) * ldc + col);
    };
    f32x4 cur[8], nxt[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) cur[j] = __builtin_nontemporal_load(cptr(0, j));
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (i + 1 < 8) {
#pragma unroll
        for (int j = 0; j < 8; ++j) nxt[j] = __builtin_nontemporal_load(cptr(i + 1, j));
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) *cptr(i, j) = acc[i][j] + cur[j];
#pragma unroll
      for (int j = 0; j < 8; ++j) cur[j] = nxt[j];
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = m0 + wm * 128 + i * 16 + frow;
    if (OUT == kOutBf16) {
#pragma unroll
      for (int j = 0; j < 8; j += 2) {
        const uint32_t lo0 = pack_bf16x2(acc[i][j][0], acc[i][j][1]), hi0 = pack_bf16x2(acc[i][j][2], acc[i][j][3]);
        const uint32_t lo1 = pack_bf16x2(acc[i][j + 1][0], acc[i][j + 1][1]), hi1 = pack_bf16x2(acc[i][j + 1][2], acc[i][j + 1][3]);
        if (FULL && quad_aligned) {
          const auto l = __builtin_amdgcn_permlane16_swap(lo0, lo1, false, false);
          const auto h = __builtin_amdgcn_permlane16_swap(hi0, hi1, false, false);
          const u32x4 v = {l[0], h[0], l[1], h[1]};
          const int col = n0 + wn * 128 + (j + (fk & 1)) * 16 + (fk >> 1) * 8;
          *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(Cv) + static_cast<int64_t>(row) * ldc + col) = v;
        } else if (row < M) {
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const int col = n0 + wn * 128 + (j + h) * 16 + fk * 4;
            const uint32_t lo = h ? lo1 : lo0, hi = h ? hi1 : hi0;
            uint16_t* dst = static_cast<uint16_t*>(Cv) + static_cast<int64_t>(row) * ldc + col;
            if (col < N) dst[0] = static_cast<uint16_t>(lo & 0xffffu);
            if (col + 1 < N) dst[1] = static_cast<uint16_t>(lo >> 16);
            if (col + 2 < N) dst[2] = static_cast<uint16_t>(hi & 0xffffu);
            if (col + 3 < N) dst[3] = static_cast<uint16_t>(hi >> 16);
          }
        }
      }
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        // fp32 out (the host requires 16-byte aligned rows for these forms)
        const int col = n0 + wn * 128 + j * 16 + fk * 4;
        float* dst = static_cast<float*>(Cv) + static_cast<int64_t>(row) * ldc + col;
        f32x4 v = acc[i][j];
        if (FULL || (row < M && col + 3 < N)) {
          if (OUT == kOutF32Add) v += *reinterpret_cast<const f32x4*>(dst);
          *reinterpret_cast<f32x4*>(dst) = v;
        } else if (row < M) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (col + e < N) dst[e] = (OUT == kOutF32Add ? dst[e] : 0.f) + v[e];
        }
      }
    }
  }
}

// Workgroup ids go round-robin over the 8 accelerator dies, each with its own L2.  Tiles are
// grouped in blocks of 8 (M) x 4 (N) = 32, the number of workgroups that run together on a die, and
// each die gets a contiguous range of blocks: the workgroups sharing an L2 at any time then share
// 8 A panels and 4 B panels (12 panel streams for 32 tiles).  Positions of a block that fall
// outside the matrix exit at once.
constexpr int kGroupM = 8, kGroupN = 4;

template <int OUT, bool TA, bool TB>
__global__ __launch_bounds__(256) void dppo_gemm_nt_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                           const uint16_t* __restrict__ B, int64_t ldb,
                                                           void* __restrict__ C, int64_t ldc, int M, int N, int K,
                                                           int tiles_m, int tiles_n, int blocks_m, int blocks_per_die, const GemmStats gs) {
  // two stages of (A panel | B panel): 2 x 64 KiB of the compute unit's 160 KiB
  __shared__ __attribute__((aligned(16))) unsigned char lds0[kStageBytes];
  __shared__ __attribute__((aligned(16))) unsigned char lds1[kStageBytes];
  const int die = static_cast<int>(blockIdx.x) & 7, slot = static_cast<int>(blockIdx.x) >> 3;      // slot-th workgroup of its die
  const int block = die * blocks_per_die + slot / (kGroupM * kGroupN), within = slot % (kGroupM * kGroupN);
  const int bn = block / blocks_m, bm = block - bn * blocks_m;
  const int tm = bm * kGroupM + (within % kGroupM), tn = bn * kGroupN + (within / kGroupM);
  if (tm >= tiles_m || tn >= tiles_n) return;
  const int m0 = tm * kBM, n0 = tn * kBN;
  if (M - m0 >= kBM && N - n0 >= kBN) gemm_tile<true, OUT, TA, TB>(lds0, lds1, A, lda, B, ldb, C, ldc, M, N, K, m0, n0, gs);
  else                                gemm_tile<false, OUT, TA, TB>(lds0, lds1, A, lda, B, ldb, C, ldc, M, N, K, m0, n0, gs);
}

}  // namespace

hipError_t launch_gemm_nt(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, void* C, int64_t ldc,
                          int M, int N, int K, int out, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  const int tiles_m = (M + kBM - 1) / kBM, tiles_n = (N + kBN - 1) / kBN;
  const int blocks_m = (tiles_m + kGroupM - 1) / kGroupM, blocks_n = (tiles_n + kGroupN - 1) / kGroupN;
  const int blocks_per_die = (blocks_m * blocks_n + 7) / 8;
  const dim3 grid(8 * blocks_per_die * kGroupM * kGroupN), wg(256);
  if (out == 0)      hipLaunchKernelGGL((dppo_gemm_nt_kernel<kOutBf16, false, false>), grid, wg, 0, s, A, lda, B, ldb, C, ldc, M, N, K, tiles_m, tiles_n, blocks_m, blocks_per_die, GemmStats{});
  else if (out == 1) hipLaunchKernelGGL((dppo_gemm_nt_kernel<kOutF32, false, false>), grid, wg, 0, s, A, lda, B, ldb, C, ldc, M, N, K, tiles_m, tiles_n, blocks_m, blocks_per_die, GemmStats{});
  else               hipLaunchKernelGGL((dppo_gemm_nt_kernel<kOutF32Add, false, false>), grid, wg, 0, s, A, lda, B, ldb, C, ldc, M, N, K, tiles_m, tiles_n, blocks_m, blocks_per_die, GemmStats{});
  return hipGetLastError();
}

// The first product of the hidden-state path with nothing of C stored: per row and column tile the
// softmax statistics of the bf16-rounded logits, and the logits at the sampled and top-K ids.
hipError_t launch_gemm_stats(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, int M, int N, int K,
                             const GemmStats& gs, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  const int tiles_m = (M + kBM - 1) / kBM, tiles_n = (N + kBN - 1) / kBN;
  if (gs.tiles_n != tiles_n) return hipErrorInvalidValue;
  const int blocks_m = (tiles_m + kGroupM - 1) / kGroupM, blocks_n = (tiles_n + kGroupN - 1) / kGroupN;
  const int blocks_per_die = (blocks_m * blocks_n + 7) / 8;
  const dim3 grid(8 * blocks_per_die * kGroupM * kGroupN), wg(256);
  hipLaunchKernelGGL((dppo_gemm_nt_kernel<kOutStats, false, false>), grid, wg, 0, s, A, lda, B, ldb, static_cast<void*>(nullptr), int64_t(0), M, N, K,
                     tiles_m, tiles_n, blocks_m, blocks_per_die, gs);
  return hipGetLastError();
}

// C[M, N] (fp32; out 1: written, 2: added to) = A^T B with A [K, M], B [K, N] (row-major, the contraction index the row index)
hipError_t launch_gemm_tn(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, void* C, int64_t ldc,
                          int M, int N, int K, int out, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  const int tiles_m = (M + kBM - 1) / kBM, tiles_n = (N + kBN - 1) / kBN;
  const int blocks_m = (tiles_m + kGroupM - 1) / kGroupM, blocks_n = (tiles_n + kGroupN - 1) / kGroupN;
  const int blocks_per_die = (blocks_m * blocks_n + 7) / 8;
  const dim3 grid(8 * blocks_per_die * kGroupM * kGroupN), wg(256);
  if (out == 1) hipLaunchKernelGGL((dppo_gemm_nt_kernel<kOutF32, true, true>), grid, wg, 0, s, A, lda, B, ldb, C, ldc, M, N, K, tiles_m, tiles_n, blocks_m, blocks_per_die, GemmStats{});
  else          hipLaunchKernelGGL((dppo_gemm_nt_kernel<kOutF32Add, true, true>), grid, wg, 0, s, A, lda, B, ldb, C, ldc, M, N, K, tiles_m, tiles_n, blocks_m, blocks_per_die, GemmStats{});
  return hipGetLastError();
}

// C[M, N] bf16 = A B with A [M, K] (contraction index contiguous) and B [K, N] (contraction index the row index); K % 64 == 0
hipError_t launch_gemm_nn(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, void* C, int64_t ldc,
                          int M, int N, int K, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  const int tiles_m = (M + kBM - 1) / kBM, tiles_n = (N + kBN - 1) / kBN;
  const int blocks_m = (tiles_m + kGroupM - 1) / kGroupM, blocks_n = (tiles_n + kGroupN - 1) / kGroupN;
  const int blocks_per_die = (blocks_m * blocks_n + 7) / 8;
  const dim3 grid(8 * blocks_per_die * kGroupM * kGroupN), wg(256);
  hipLaunchKernelGGL((dppo_gemm_nt_kernel<kOutBf16, false, true>), grid, wg, 0, s, A, lda, B, ldb, C, ldc, M, N, K, tiles_m, tiles_n, blocks_m, blocks_per_die, GemmStats{});
  return hipGetLastError();
}

}  // namespace dppo
