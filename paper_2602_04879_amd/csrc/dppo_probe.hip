// Measurement utilities: a plain 16-byte-vector device copy and a read-only pass over a buffer.
// They calibrate the HBM byte counters (a copy of known size) and give the streaming ceiling
// of the device that the loss kernels are compared with.  And a loop of nothing but bf16
// matrix-core products on every compute unit: what the matrix cores sustain under the board's
// power limit, the ceiling the matrix-product kernel is compared with.
#include <hip/hip_runtime.h>
#include "dppo_probe.h"
#include "dppo_common.hpp"

namespace {

// Copy: ONE WAVE per compute unit, sixteen 16-byte loads in flight per lane before the sixteen
// stores, both marked non-temporal: the pattern that streamed fastest on MI355X among those tried
// (6.0 TB/s; four waves per compute unit with four loads each reach 5.5, more waves less).
__global__ __launch_bounds__(64) void dppo_probe_copy_kernel(const dppo::u32x4* __restrict__ src, dppo::u32x4* __restrict__ dst, size_t nvec) {
  constexpr int U = 16;
  const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
  size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  for (; i + (U - 1) * stride < nvec; i += U * stride) {
    dppo::u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
    __builtin_amdgcn_sched_barrier(0);          // all sixteen loads before the first store
#pragma unroll
    for (int u = 0; u < U; ++u) __builtin_nontemporal_store(v[u], dst + i + u * stride);
    __builtin_amdgcn_sched_barrier(0);
  }
  for (; i < nvec; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

__global__ __launch_bounds__(256) void dppo_probe_read_kernel(const dppo::u32x4* __restrict__ src, size_t nvec, uint32_t* sink) {
  const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
  uint32_t acc = 0;
  for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < nvec; i += stride) {
    const dppo::u32x4 v = __builtin_nontemporal_load(src + i);
    acc |= v.x | v.y | v.z | v.w;
  }
  if (acc == 0x12345678u) *sink = acc;   // keeps the loads alive; practically never taken
}

__global__ __launch_bounds__(256) void dppo_probe_fill_kernel(dppo::u32x4* __restrict__ dst, size_t nvec, uint32_t value) {
  const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
  const dppo::u32x4 v = {value, value, value, value};
  for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < nvec; i += stride) dst[i] = v;
}

// The same copy with the address pattern of the loss kernels: each workgroup copies whole rows,
// one after the other, four 16-byte vectors per thread in flight.
__global__ __launch_bounds__(512) void dppo_probe_copy_rows_kernel(const dppo::u32x4* __restrict__ src, dppo::u32x4* __restrict__ dst,
                                                                   int rows, int row_vecs, size_t pitch_vecs) {
  for (int row = blockIdx.x; row < rows; row += gridDim.x) {
    const dppo::u32x4* s = src + static_cast<size_t>(row) * pitch_vecs;
    dppo::u32x4* d = dst + static_cast<size_t>(row) * pitch_vecs;
    int i = threadIdx.x;
    for (; i + 3 * 512 < row_vecs; i += 4 * 512) {
      dppo::u32x4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = s[i + u * 512];
#pragma unroll
      for (int u = 0; u < 4; ++u) d[i + u * 512] = v[u];
    }
    for (; i < row_vecs; i += 512) d[i] = s[i];
  }
}

// The copy with the memory pattern of the register-resident loss kernel and none of its arithmetic:
// one persistent workgroup of 512 threads per compute unit holds a whole row in its registers
// (38 chunks of 16 bytes per thread through range-checked buffer resources), writes it out in one
// run of non-temporal stores and then requests its next row in one run of loads; rows advance by
// the number of workgroups, the workgroups of one die on neighbouring rows.  What this reaches is
// the ceiling of that pattern on the device.
__global__ __launch_bounds__(512) void dppo_probe_copy_resident_kernel(const char* __restrict__ src, char* __restrict__ dst, int rows,
                                                                       uint32_t row_bytes, int64_t pitch_bytes) {
  constexpr int NCHUNK = 38;
  constexpr uint32_t kStride = 512 * 16u;
  const uint32_t voff = threadIdx.x * 16u;
  dppo::u32x4 buf[NCHUNK];
  int row = dppo::first_row_of_workgroup();
  {
    const dppo::row_rsrc_t zr = dppo::make_row_rsrc(src + row * pitch_bytes, row_bytes);
#pragma unroll
    for (int i = 0; i < NCHUNK; ++i) buf[i] = dppo::row_load16<false>(zr, voff, i * kStride);
  }
  for (; row < rows; row += gridDim.x) {
    const int next = row + gridDim.x;
    const bool more = next < rows;
    const dppo::row_rsrc_t zn = dppo::make_row_rsrc(src + (more ? next : row) * pitch_bytes, more ? row_bytes : 0u);
    const dppo::row_desc_t out = dppo::make_row_desc(dst + row * pitch_bytes, row_bytes);
#pragma unroll
    for (int i = 0; i < NCHUNK; ++i) dppo::row_store16_untracked(out, voff, i * kStride, buf[i]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NCHUNK; ++i) buf[i] = dppo::row_load16<false>(zn, voff, i * kStride);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Matrix-core ceiling: each wave keeps 256 fp32 accumulators (as the product kernel does) and
// issues `iters` rounds of independent products on operands held in registers: SHAPE 16: 64 of
// v_mfma_f32_16x16x32_bf16 per round (524288 multiply-adds); SHAPE 32: 16 of
// v_mfma_f32_32x32x16_bf16 (262144 multiply-adds).  Operands are pseudo-random bf16 in
// +-[1, 2) so that the multipliers toggle as they do on real data.
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x4 __attribute__((ext_vector_type(4)));
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));
template <int SHAPE>
__global__ __launch_bounds__(256) void dppo_probe_mfma_kernel(float* __restrict__ out, int iters) {
  uint32_t s = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
  probe_bf16x8 a[4], b[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    union { uint32_t u[4]; probe_bf16x8 v; } ua, ub;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      s = s * 1664525u + 1013904223u; ua.u[e] = (s & 0x807f807fu) | 0x3f803f80u;
      s = s * 1664525u + 1013904223u; ub.u[e] = (s & 0x807f807fu) | 0x3f803f80u;
    }
    a[t] = ua.v; b[t] = ub.v;
  }
  float r = 0.f;
  if (SHAPE == 32) {
    probe_f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) r += acc[i][j][e];
  } else {
    probe_f32x4 acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j & 3], a[i & 3], acc[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) r += acc[i][j][e];
  }
  out[blockIdx.x * 256 + threadIdx.x] = r;    // keeps the products alive
}

int probe_cus() {
  int dev = 0, cus = 256;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    cus = 256;
  return cus;
}

}  // namespace

extern "C" {

dppo_status_t dppo_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src) return DPPO_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src) | bytes) & 15u) return DPPO_ERR_ALIGN;
  if (bytes == 0) return DPPO_OK;
  hipLaunchKernelGGL(dppo_probe_copy_kernel, dim3(probe_cus()), dim3(64), 0, static_cast<hipStream_t>(stream),
                     static_cast<const dppo::u32x4*>(src), static_cast<dppo::u32x4*>(dst), bytes / 16);
  return hipGetLastError() == hipSuccess ? DPPO_OK : DPPO_ERR_LAUNCH;
}

dppo_status_t dppo_probe_copy_rows(void* dst, const void* src, int64_t rows, size_t row_bytes, size_t pitch_bytes, void* stream) {
  if (!dst || !src) return DPPO_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src) | row_bytes | pitch_bytes) & 15u) return DPPO_ERR_ALIGN;
  if (rows < 0 || rows >= (int64_t(1) << 31) || pitch_bytes < row_bytes || row_bytes / 16 >= (size_t(1) << 31)) return DPPO_ERR_SHAPE;
  if (rows == 0 || row_bytes == 0) return DPPO_OK;
  const int grid = static_cast<int>(rows < probe_cus() ? rows : probe_cus());
  hipLaunchKernelGGL(dppo_probe_copy_rows_kernel, dim3(grid), dim3(512), 0, static_cast<hipStream_t>(stream),
                     static_cast<const dppo::u32x4*>(src), static_cast<dppo::u32x4*>(dst), static_cast<int>(rows),
                     static_cast<int>(row_bytes / 16), pitch_bytes / 16);
  return hipGetLastError() == hipSuccess ? DPPO_OK : DPPO_ERR_LAUNCH;
}

dppo_status_t dppo_probe_copy_resident(void* dst, const void* src, int64_t rows, size_t row_bytes, size_t pitch_bytes, void* stream) {
  if (!dst || !src) return DPPO_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src) | row_bytes | pitch_bytes) & 15u) return DPPO_ERR_ALIGN;
  // a row must fit the registers of one workgroup: 512 threads x 38 chunks of 16 bytes
  if (rows < 0 || rows >= (int64_t(1) << 31) || pitch_bytes < row_bytes || row_bytes > 512u * 38u * 16u) return DPPO_ERR_SHAPE;
  if (rows == 0 || row_bytes == 0) return DPPO_OK;
  const int grid = static_cast<int>(rows < probe_cus() ? rows : probe_cus());
  hipLaunchKernelGGL(dppo_probe_copy_resident_kernel, dim3(grid), dim3(512), 0, static_cast<hipStream_t>(stream),
                     static_cast<const char*>(src), static_cast<char*>(dst), static_cast<int>(rows),
                     static_cast<uint32_t>(row_bytes), static_cast<int64_t>(pitch_bytes));
  return hipGetLastError() == hipSuccess ? DPPO_OK : DPPO_ERR_LAUNCH;
}

dppo_status_t dppo_probe_fill(void* dst, size_t bytes, uint32_t value, void* stream) {
  if (!dst) return DPPO_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(dst) | bytes) & 15u) return DPPO_ERR_ALIGN;
  if (bytes == 0) return DPPO_OK;
  // one workgroup per compute unit: 6.4 TB/s; with eight per compute unit the same kernel writes at 5.0
  hipLaunchKernelGGL(dppo_probe_fill_kernel, dim3(probe_cus()), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<dppo::u32x4*>(dst), bytes / 16, value);
  return hipGetLastError() == hipSuccess ? DPPO_OK : DPPO_ERR_LAUNCH;
}

dppo_status_t dppo_probe_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink) return DPPO_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(src) | bytes) & 15u) return DPPO_ERR_ALIGN;
  if (bytes == 0) return DPPO_OK;
  hipLaunchKernelGGL(dppo_probe_read_kernel, dim3(probe_cus() * 8), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const dppo::u32x4*>(src), bytes / 16, static_cast<uint32_t*>(sink));
  return hipGetLastError() == hipSuccess ? DPPO_OK : DPPO_ERR_LAUNCH;
}

dppo_status_t dppo_probe_mfma(int shape, int iters, void* out, size_t out_bytes, double* flop, void* stream) {
  if (!out) return DPPO_ERR_NULL;
  if ((shape != 16 && shape != 32) || iters < 0) return DPPO_ERR_SHAPE;
  const int cus = probe_cus();
  if (out_bytes < static_cast<size_t>(cus) * 256 * sizeof(float)) return DPPO_ERR_WORKSPACE;
  // per round and wave: 64 x (16 x 16 x 32) or 16 x (32 x 32 x 16) multiply-adds
  if (flop) *flop = 2.0 * (shape == 16 ? 524288.0 : 262144.0) * 4.0 * static_cast<double>(cus) * static_cast<double>(iters);
  if (shape == 16) hipLaunchKernelGGL(dppo_probe_mfma_kernel<16>, dim3(cus), dim3(256), 0, static_cast<hipStream_t>(stream), static_cast<float*>(out), iters);
  else             hipLaunchKernelGGL(dppo_probe_mfma_kernel<32>, dim3(cus), dim3(256), 0, static_cast<hipStream_t>(stream), static_cast<float*>(out), iters);
  return hipGetLastError() == hipSuccess ? DPPO_OK : DPPO_ERR_LAUNCH;
}

}  // extern "C"
