// Host-side launch entry points of the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include "dppo_common.hpp"

namespace dppo {

// General two-pass kernel.  vec=false selects the element-wise variant (needed when logits
// and grad_logits rows do not share their 16-byte misalignment).
hipError_t launch_streaming(const KParams& p, bool vec, bool grad, int threads, int grid, hipStream_t s);

// Register-resident fused forward+backward kernel (threads = 256 or 1024; 20 register chunks
// of one 16-byte vector per thread).  Needs V % 8 == 0, V/8 <= threads*20, 16-byte aligned
// rows of logits and grad.  resident_blocks_per_cu() is the occupancy the runtime reports.
constexpr int kResidentChunks = 20;
hipError_t launch_resident(const KParams& p, int threads, int grid, hipStream_t s);
int resident_blocks_per_cu(int threads);

// loss[0] = loss_scale * sum(partial[0..n)) in a fixed order.
hipError_t launch_finalize(const double* partial, int n, float loss_scale, float* loss, hipStream_t s);

}  // namespace dppo
