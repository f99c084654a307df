// bf16 matrix product on the matrix cores, C[M, N] = A[M, K] * B[N, K]^T with fp32 accumulation:
// both operands row-major with the contraction index contiguous (what an nn.Linear forward is:
// activations [T, d] times weight [V, d] transposed), C row-major: bf16 rounded to nearest even,
// or fp32, optionally added to what C holds.
//
// One workgroup of 256 threads (4 waves, one per SIMD) per 256 x 256 tile of C, each wave a
// 128 x 128 quadrant as 4 x 4 products of v_mfma_f32_32x32x16_bf16 (256 fp32 accumulators per
// lane).  The contraction runs in steps of 64: the A and B panels of a step (256 x 64 each,
// 32 KiB) are loaded from global memory straight into one of two LDS stages a step ahead,
// 16 bytes per lane, in a layout swizzled so that the matrix-core fragment reads (one 16-byte
// read per lane: 8 consecutive k of one row) spread over all banks.
// Panel rows past M or N re-read the last valid row (their products are never stored); all
// loads go through range-checked buffer resources over exactly the rows a tile owns.  K must be
// a multiple of 64, rows 16-byte aligned (checked by the host).
#include "dppo_common.hpp"
#include "dppo_launch.hpp"

namespace dppo {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kRowBytes = kBK * 2;                    // one panel row in LDS: 128 bytes = 8 vectors
constexpr int kPanelBytes = kBM * kRowBytes;          // 32 KiB (kBM == kBN)
constexpr int kStageBytes = 2 * kPanelBytes;          // A panel then B panel

// LDS byte offset of the 16-byte vector `kvec` (0..7) of panel row `row`: the vector index is
// XOR-ed with bits 1..3 of the row, so 16 consecutive rows at one kvec cover all 64 banks once.
__device__ __forceinline__ uint32_t lds_off(int row, int kvec) {
  return static_cast<uint32_t>(row) * kRowBytes + static_cast<uint32_t>((kvec ^ ((row >> 1) & 7)) << 4);
}

// One 256 x 256 tile.  FULL: all 256 rows of both panels exist, so the eight rows a loader thread
// moves per panel differ by a uniform stride (carried in the scalar offset of the load).
// Otherwise a panel row past the matrix re-reads the last valid row: its products are never stored.
// OUT selects what leaves the tile: bf16 (rounded to nearest even), fp32, or fp32 added to what C holds.
enum : int { kOutBf16 = 0, kOutF32 = 1, kOutF32Add = 2 };

template <bool FULL, int OUT>
__device__ __forceinline__ void gemm_tile(unsigned char* lds0, unsigned char* lds1, const uint16_t* __restrict__ A, int64_t lda,
                                          const uint16_t* __restrict__ B, int64_t ldb, void* __restrict__ Cv, int64_t ldc,
                                          int M, int N, int K, int m0, int n0) {
  const int tid = threadIdx.x, lane = tid & 63, wid = uniform_i(tid >> 6);
  const int wm = wid >> 1, wn = wid & 1;
  const int rows_a = min(kBM, M - m0), rows_b = min(kBN, N - n0);
  const uint32_t pitch_a = static_cast<uint32_t>(lda) * 2u, pitch_b = static_cast<uint32_t>(ldb) * 2u;
  // range-checked views of exactly the rows this tile owns
  const row_rsrc_t ra = make_row_rsrc(A + static_cast<int64_t>(m0) * lda, static_cast<uint32_t>(rows_a - 1) * pitch_a + static_cast<uint32_t>(K) * 2u);
  const row_rsrc_t rb = make_row_rsrc(B + static_cast<int64_t>(n0) * ldb, static_cast<uint32_t>(rows_b - 1) * pitch_b + static_cast<uint32_t>(K) * 2u);

  // Loader role: thread t moves LDS vector slot (t % 8) of rows t/8 + 32 i, i = 0..7, of each panel;
  // the slot holds global k-vector slot ^ ((row >> 1) & 7), the same for all eight rows.
  const int lrow = tid >> 3, lslot = tid & 7;
  const uint32_t lkv = static_cast<uint32_t>((lslot ^ ((lrow >> 1) & 7)) << 4);
  const uint32_t voff_a = static_cast<uint32_t>(lrow) * pitch_a + lkv, voff_b = static_cast<uint32_t>(lrow) * pitch_b + lkv;

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Fragment role: lane holds 8 consecutive k (k half `fk` of a 16-wide step) of row `frow` of a
  // 32-row block.  The swizzle depends on the row only through frow, so one offset per k-vector
  // serves every block of both panels.
  const int frow = lane & 31, fk = lane >> 5;
  // 8-byte stores need C rows that keep 8-byte alignment (uniform over the launch)
  const bool pair_aligned = ((reinterpret_cast<uintptr_t>(Cv) & 7u) == 0) && (ldc % 4 == 0);
  uint32_t foff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) foff[ks] = lds_off(frow, ks * 2 + fk);
  const uint32_t fbase_a = static_cast<uint32_t>(wm * 128) * kRowBytes;
  const uint32_t fbase_b = kPanelBytes + static_cast<uint32_t>(wn * 128) * kRowBytes;
  auto read_frags = [&](const unsigned char* stage, int ks, bf16x8 (&fa)[4], bf16x8 (&fb)[4]) {
    const uint32_t o = foff[ks];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      fa[t] = *reinterpret_cast<const bf16x8*>(stage + fbase_a + t * 32 * kRowBytes + o);
      fb[t] = *reinterpret_cast<const bf16x8*>(stage + fbase_b + t * 32 * kRowBytes + o);
    }
  };
  auto mma16 = [&](const bf16x8 (&fa)[4], const bf16x8 (&fb)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
  };

  // Pipeline over the contraction: while step kt is multiplied out of LDS stage kt % 2, the
  // panels of step kt+1 are loaded into the other stage; the fragments of each 16-wide sub-step
  // are read from LDS one sub-step ahead of the matrix-core instructions that consume them.
  // One barrier per step, before the first fragments of the next stage are read.
  const int nk = K / kBK;
  // Global memory -> LDS directly (buffer_load ... lds): lane l of a wave-level load deposits its
  // 16 bytes at (LDS base of the instruction) + 16 l, which is exactly the loader layout above for
  // the base stage + panel + i * 4096 + wave * 1024.  No staging registers, no LDS store
  // instructions; completion is counted with the other vector-memory loads.
  typedef __attribute__((address_space(3))) void* lds_ptr_t;
  auto dma_panel = [&](unsigned char* stage, int step, bool b_panel) {
    const uint32_t koff = static_cast<uint32_t>(step) * (kBK * 2);
    unsigned char* dst = stage + (b_panel ? kPanelBytes : 0) + wid * 1024;
    const row_rsrc_t r = b_panel ? rb : ra;
    const uint32_t pitch = b_panel ? pitch_b : pitch_a;
    const uint32_t voff = (b_panel ? voff_b : voff_a) + koff;
    const int rows = b_panel ? rows_b : rows_a;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (FULL) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr_t)(dst + i * 4096), 16, voff, static_cast<uint32_t>(i * 32) * pitch, 0, 0);
      } else {
        const uint32_t row = static_cast<uint32_t>(min(lrow + 32 * i, rows - 1));
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr_t)(dst + i * 4096), 16, row * pitch + lkv + koff, 0, 0, 0);
      }
    }
  };
  dma_panel(lds0, 0, false);
  dma_panel(lds0, 0, true);
  __syncthreads();                       // waits for this wave's loads, then for everyone's
  bf16x8 fa0[4], fb0[4], fa1[4], fb1[4];
  read_frags(lds0, 0, fa0, fb0);
  // The two stages are two separate arrays and the loop takes two steps per trip, so that every
  // LDS access names its array: the compiler then knows that fragment reads of one stage need not
  // wait for the loads in flight into the other.
  auto step = [&](const unsigned char* cur, unsigned char* nxt, int kt) {
    const bool more = kt + 1 < nk;
    read_frags(cur, 1, fa1, fb1);
    if (more) dma_panel(nxt, kt + 1, false);
    __builtin_amdgcn_sched_barrier(0);
    mma16(fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(cur, 2, fa0, fb0);
    if (more) dma_panel(nxt, kt + 1, true);
    __builtin_amdgcn_sched_barrier(0);
    mma16(fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(cur, 3, fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
    mma16(fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    // the next stage is complete (own loads waited for, then everyone's) and this one fully read
    __syncthreads();
    if (more) read_frags(nxt, 0, fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    mma16(fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
  };
  int kt = 0;
  for (; kt + 1 < nk; kt += 2) {
    step(lds0, lds1, kt);
    step(lds1, lds0, kt + 1);
  }
  if (kt < nk) step(lds0, lds1, kt);      // odd number of steps: the last one reads stage 0 again

  // Store.  The products were formed with the operands swapped (B fragment first), so a lane's
  // accumulators r = 4q .. 4q+3 of a 32 x 32 block are four consecutive COLUMNS
  // q*8 + (lane/32)*4 + 0..3 of row lane%32: one 8-byte store of four bf16 (16 bytes of fp32) each.
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = m0 + wm * 128 + i * 32 + frow;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = n0 + wn * 128 + j * 32 + q * 8 + fk * 4;
        if (OUT == kOutBf16) {
          const uint32_t lo = pack_bf16x2(acc[i][j][4 * q], acc[i][j][4 * q + 1]), hi = pack_bf16x2(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
          uint16_t* dst = static_cast<uint16_t*>(Cv) + static_cast<int64_t>(row) * ldc + col;
          if (FULL && pair_aligned) {
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            const u32x2 v = {lo, hi};
            *reinterpret_cast<u32x2*>(dst) = v;
          } else if (row < M) {
            if (col < N) dst[0] = static_cast<uint16_t>(lo & 0xffffu);
            if (col + 1 < N) dst[1] = static_cast<uint16_t>(lo >> 16);
            if (col + 2 < N) dst[2] = static_cast<uint16_t>(hi & 0xffffu);
            if (col + 3 < N) dst[3] = static_cast<uint16_t>(hi >> 16);
          }
        } else {
          // fp32 out (the host requires 16-byte aligned rows for these forms)
          typedef float f32x4 __attribute__((ext_vector_type(4)));
          float* dst = static_cast<float*>(Cv) + static_cast<int64_t>(row) * ldc + col;
          f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
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
}

// Workgroup ids go round-robin over the 8 accelerator dies, each with its own L2.  Tiles are
// grouped in blocks of 8 (M) x 4 (N) = 32, the number of workgroups that run together on a die, and
// each die gets a contiguous range of blocks: the workgroups sharing an L2 at any time then share
// 8 A panels and 4 B panels (12 panel streams for 32 tiles).  Positions of a block that fall
// outside the matrix exit at once.
constexpr int kGroupM = 8, kGroupN = 4;

template <int OUT>
__global__ __launch_bounds__(256) void dppo_gemm_nt_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                           const uint16_t* __restrict__ B, int64_t ldb,
                                                           void* __restrict__ C, int64_t ldc, int M, int N, int K,
                                                           int tiles_m, int tiles_n, int blocks_m, int blocks_per_die) {
  // two stages of (A panel | B panel): 2 x 64 KiB of the compute unit's 160 KiB
  __shared__ __attribute__((aligned(16))) unsigned char lds0[kStageBytes];
  __shared__ __attribute__((aligned(16))) unsigned char lds1[kStageBytes];
  const int die = static_cast<int>(blockIdx.x) & 7, slot = static_cast<int>(blockIdx.x) >> 3;      // slot-th workgroup of its die
  const int block = die * blocks_per_die + slot / (kGroupM * kGroupN), within = slot % (kGroupM * kGroupN);
  const int bn = block / blocks_m, bm = block - bn * blocks_m;
  const int tm = bm * kGroupM + (within % kGroupM), tn = bn * kGroupN + (within / kGroupM);
  if (tm >= tiles_m || tn >= tiles_n) return;
  const int m0 = tm * kBM, n0 = tn * kBN;
  if (M - m0 >= kBM && N - n0 >= kBN) gemm_tile<true, OUT>(lds0, lds1, A, lda, B, ldb, C, ldc, M, N, K, m0, n0);
  else                                gemm_tile<false, OUT>(lds0, lds1, A, lda, B, ldb, C, ldc, M, N, K, m0, n0);
}

// dst[c, r] = src[r, c] for 2-byte elements, 64 x 64 tiles through LDS, 16-byte accesses (8 elements
// per lane) on both sides; the LDS rows are 66 elements long, which spreads the transposed 2-byte
// reads over the banks.  Columns R .. R_pad-1 of dst are written as zeros.  Needs Cn, R_pad, both
// pitches multiples of 8 and 16-byte aligned bases (checked by the launcher).
__global__ __launch_bounds__(256) void dppo_transpose_kernel(const uint16_t* __restrict__ src, int64_t ld_src,
                                                             uint16_t* __restrict__ dst, int64_t ld_dst, int R, int Cn, int R_pad) {
  __shared__ __attribute__((aligned(4))) uint16_t tile[64][66];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int sub = threadIdx.x & 7, line = threadIdx.x >> 3;      // 8 lanes x 16 bytes per 64-element line
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = r0 + line + 32 * i, c = c0 + sub * 8;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (r < R && c < Cn) v = *reinterpret_cast<const u32x4*>(src + static_cast<int64_t>(r) * ld_src + c);   // Cn % 8 == 0: all 8 in range
    uint32_t* t = reinterpret_cast<uint32_t*>(&tile[line + 32 * i][sub * 8]);
    t[0] = v.x; t[1] = v.y; t[2] = v.z; t[3] = v.w;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int cl = line + 32 * i, c = c0 + cl, r = r0 + sub * 8;
    uint32_t w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) w[k] = static_cast<uint32_t>(tile[sub * 8 + 2 * k][cl]) | (static_cast<uint32_t>(tile[sub * 8 + 2 * k + 1][cl]) << 16);
    if (c < Cn && r < R_pad) {                                   // R_pad % 8 == 0: all 8 in range
      const u32x4 v = {w[0], w[1], w[2], w[3]};
      *reinterpret_cast<u32x4*>(dst + static_cast<int64_t>(c) * ld_dst + r) = v;
    }
  }
}

}  // namespace

hipError_t launch_transpose(const uint16_t* src, int64_t ld_src, uint16_t* dst, int64_t ld_dst, int R, int Cn, int R_pad, hipStream_t s) {
  if (R_pad < R) R_pad = R;
  if (R_pad <= 0 || Cn <= 0) return hipSuccess;
  if ((Cn % 8) || (R_pad % 8) || (ld_src % 8) || (ld_dst % 8) || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u))
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(dppo_transpose_kernel, dim3((Cn + 63) / 64, (R_pad + 63) / 64), dim3(256), 0, s, src, ld_src, dst, ld_dst, R, Cn, R_pad);
  return hipGetLastError();
}

hipError_t launch_gemm_nt(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, void* C, int64_t ldc,
                          int M, int N, int K, int out, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  const int tiles_m = (M + kBM - 1) / kBM, tiles_n = (N + kBN - 1) / kBN;
  const int blocks_m = (tiles_m + kGroupM - 1) / kGroupM, blocks_n = (tiles_n + kGroupN - 1) / kGroupN;
  const int blocks_per_die = (blocks_m * blocks_n + 7) / 8;
  const dim3 grid(8 * blocks_per_die * kGroupM * kGroupN), wg(256);
  if (out == 0)      hipLaunchKernelGGL(dppo_gemm_nt_kernel<kOutBf16>, grid, wg, 0, s, A, lda, B, ldb, C, ldc, M, N, K, tiles_m, tiles_n, blocks_m, blocks_per_die);
  else if (out == 1) hipLaunchKernelGGL(dppo_gemm_nt_kernel<kOutF32>, grid, wg, 0, s, A, lda, B, ldb, C, ldc, M, N, K, tiles_m, tiles_n, blocks_m, blocks_per_die);
  else               hipLaunchKernelGGL(dppo_gemm_nt_kernel<kOutF32Add>, grid, wg, 0, s, A, lda, B, ldb, C, ldc, M, N, K, tiles_m, tiles_n, blocks_m, blocks_per_die);
  return hipGetLastError();
}

}  // namespace dppo
