// bf16 matrix product on the matrix cores, C[M, N] = A[M, K] * B[N, K]^T with fp32 accumulation:
// both operands row-major with the contraction index contiguous (what an nn.Linear forward is:
// activations [T, d] times weight [V, d] transposed), C row-major bf16, rounded to nearest even.
//
// One workgroup of 256 threads (4 waves, one per SIMD) per 256 x 256 tile of C, each wave a
// 128 x 128 quadrant as 4 x 4 products of v_mfma_f32_32x32x16_bf16 (256 fp32 accumulators per
// lane).  The contraction runs in steps of 64: the A and B panels of a step (256 x 64 each,
// 32 KiB) go from global memory to registers while the previous step is multiplied, then into
// LDS, 16 bytes per lane, in a layout swizzled so that the matrix-core fragment reads (one
// 16-byte read per lane: 8 consecutive k of one row) spread over all banks.
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

// LDS byte offset of the 16-byte vector `kvec` (0..7) of panel row `row`: the vector index is
// XOR-ed with bits 1..3 of the row, so 16 consecutive rows at one kvec cover all 64 banks once.
__device__ __forceinline__ uint32_t lds_off(int row, int kvec) {
  return static_cast<uint32_t>(row) * kRowBytes + static_cast<uint32_t>((kvec ^ ((row >> 1) & 7)) << 4);
}

__global__ __launch_bounds__(256) void dppo_gemm_nt_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                           const uint16_t* __restrict__ B, int64_t ldb,
                                                           uint16_t* __restrict__ C, int64_t ldc, int M, int N, int K,
                                                           int tiles_m, int tiles_n) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[(kBM + kBN) * kRowBytes];   // 64 KiB
  unsigned char* ldsA = lds;
  unsigned char* ldsB = lds + kBM * kRowBytes;
  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int wm = wid >> 1, wn = wid & 1;

  // Workgroup ids go round-robin over the 8 accelerator dies, each with its own L2: give each
  // die a contiguous range of tiles, ordered with the M index fastest, so that the workgroups
  // running together on a die share their B panels (and all of them the A panels).
  const int ntiles = tiles_m * tiles_n;
  const int per_xcd = (ntiles + 7) / 8;
  const int logical = (static_cast<int>(blockIdx.x) & 7) * per_xcd + (static_cast<int>(blockIdx.x) >> 3);
  if (logical >= ntiles) return;
  const int tn = logical / tiles_m, tm = logical - tn * tiles_m;
  const int m0 = tm * kBM, n0 = tn * kBN;

  // range-checked views of the two panels
  const int rows_a = min(kBM, M - m0), rows_b = min(kBN, N - n0);
  const uint64_t bytes_a = static_cast<uint64_t>(rows_a - 1) * lda * 2 + static_cast<uint64_t>(K) * 2;
  const uint64_t bytes_b = static_cast<uint64_t>(rows_b - 1) * ldb * 2 + static_cast<uint64_t>(K) * 2;
  const row_rsrc_t ra = make_row_rsrc(A + static_cast<int64_t>(m0) * lda, static_cast<uint32_t>(bytes_a));
  const row_rsrc_t rb = make_row_rsrc(B + static_cast<int64_t>(n0) * ldb, static_cast<uint32_t>(bytes_b));

  // Loader role: thread t moves vector slot (t % 8) of rows t/8 + 32 i, i = 0..7, of each panel.
  const int lrow = tid >> 3, lslot = tid & 7;
  uint32_t goff_a[8], goff_b[8], loff[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = lrow + 32 * i;
    const int kvec = lslot ^ ((row >> 1) & 7);          // which global vector lands in this LDS slot
    // a panel row past the matrix re-reads the last valid row: its products are never stored
    goff_a[i] = static_cast<uint32_t>(static_cast<uint64_t>(min(row, rows_a - 1)) * lda * 2 + kvec * 16);
    goff_b[i] = static_cast<uint32_t>(static_cast<uint64_t>(min(row, rows_b - 1)) * ldb * 2 + kvec * 16);
    loff[i] = static_cast<uint32_t>(row) * kRowBytes + static_cast<uint32_t>(lslot << 4);
  }

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4 sa[8], sb[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    sa[i] = row_load16(ra, goff_a[i], 0);
    sb[i] = row_load16(rb, goff_b[i], 0);
  }
  const int frow = lane & 31, fk = lane >> 5;           // fragment role: row within a 32-row block, k half
  const int nk = K / kBK;
  for (int kt = 0; kt < nk; ++kt) {
    __syncthreads();                                     // everyone is done reading the previous step
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      *reinterpret_cast<u32x4*>(ldsA + loff[i]) = sa[i];
      *reinterpret_cast<u32x4*>(ldsB + loff[i]) = sb[i];
    }
    __syncthreads();
    if (kt + 1 < nk) {
      const uint32_t koff = static_cast<uint32_t>(kt + 1) * (kBK * 2);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        sa[i] = row_load16(ra, goff_a[i], koff);
        sb[i] = row_load16(rb, goff_b[i], koff);
      }
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 fa[4], fb[4];
      const int kvec = ks * 2 + fk;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        fa[t] = *reinterpret_cast<const bf16x8*>(ldsA + lds_off(wm * 128 + t * 32 + frow, kvec));
        fb[t] = *reinterpret_cast<const bf16x8*>(ldsB + lds_off(wn * 128 + t * 32 + frow, kvec));
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  }

  // Store: accumulator r of a 32 x 32 block is row (r/4)*8 + (lane/32)*4 + r%4, column lane%32.
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + wn * 128 + j * 32 + frow;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * 128 + i * 32 + (r >> 2) * 8 + fk * 4 + (r & 3);
        if (row < M && col < N) C[static_cast<int64_t>(row) * ldc + col] = float_to_bf16_bits(acc[i][j][r]);
      }
    }
  }
}

// dst[c, r] = src[r, c] for 2-byte elements, 64 x 64 tiles through LDS (one padding column keeps
// the transposed reads off a single bank).
__global__ __launch_bounds__(256) void dppo_transpose_kernel(const uint16_t* __restrict__ src, int64_t ld_src,
                                                             uint16_t* __restrict__ dst, int64_t ld_dst, int R, int Cn) {
  __shared__ uint16_t tile[64][66];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4) {
    const int r = r0 + i, c = c0 + tx;
    tile[i][tx] = (r < R && c < Cn) ? src[static_cast<int64_t>(r) * ld_src + c] : uint16_t(0);
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int c = c0 + i, r = r0 + tx;
    if (c < Cn && r < R) dst[static_cast<int64_t>(c) * ld_dst + r] = tile[tx][i];
  }
}

}  // namespace

hipError_t launch_transpose(const uint16_t* src, int64_t ld_src, uint16_t* dst, int64_t ld_dst, int R, int Cn, hipStream_t s) {
  if (R <= 0 || Cn <= 0) return hipSuccess;
  hipLaunchKernelGGL(dppo_transpose_kernel, dim3((Cn + 63) / 64, (R + 63) / 64), dim3(256), 0, s, src, ld_src, dst, ld_dst, R, Cn);
  return hipGetLastError();
}

hipError_t launch_gemm_nt(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, uint16_t* C, int64_t ldc,
                          int M, int N, int K, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  const int tiles_m = (M + kBM - 1) / kBM, tiles_n = (N + kBN - 1) / kBN;
  const int ntiles = tiles_m * tiles_n;
  const int grid = ((ntiles + 7) / 8) * 8;
  hipLaunchKernelGGL(dppo_gemm_nt_kernel, dim3(grid), dim3(256), 0, s, A, lda, B, ldb, C, ldc, M, N, K, tiles_m, tiles_n);
  return hipGetLastError();
}

}  // namespace dppo
