// Measurement utilities: a plain 16-byte-vector device copy and a read-only pass over a buffer.
// They calibrate the HBM byte counters (a copy of known size) and give the streaming ceiling
// of the device that the loss kernels are compared with.
#include <hip/hip_runtime.h>
#include "dppo.h"
#include "dppo_common.hpp"

namespace {

// Copy: one workgroup per compute unit, four 16-byte loads in flight per thread before the four
// stores (the pattern that streamed fastest on MI355X among those tried).
__global__ __launch_bounds__(256) void dppo_probe_copy_kernel(const dppo::u32x4* __restrict__ src, dppo::u32x4* __restrict__ dst, size_t nvec) {
  const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
  size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < nvec; i += 4 * stride) {
    dppo::u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + i + u * stride);
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
  hipLaunchKernelGGL(dppo_probe_copy_kernel, dim3(probe_cus()), dim3(256), 0, static_cast<hipStream_t>(stream),
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

dppo_status_t dppo_probe_fill(void* dst, size_t bytes, uint32_t value, void* stream) {
  if (!dst) return DPPO_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(dst) | bytes) & 15u) return DPPO_ERR_ALIGN;
  if (bytes == 0) return DPPO_OK;
  hipLaunchKernelGGL(dppo_probe_fill_kernel, dim3(probe_cus() * 8), dim3(256), 0, static_cast<hipStream_t>(stream),
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

}  // extern "C"
