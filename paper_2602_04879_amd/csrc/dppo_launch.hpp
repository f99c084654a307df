// Host-side launch entry points of the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include "dppo_common.hpp"

namespace dppo {

// General two-pass kernel.  vec=false selects the element-wise variant (needed when logits
// and grad_logits rows do not share their 16-byte misalignment).
hipError_t launch_streaming(const KParams& p, bool vec, bool grad, int threads, int grid, hipStream_t s);

// Register-resident fused forward+backward kernel.  Two shapes: 512 threads x 38 register
// chunks (rows up to 155648 entries, one workgroup per compute unit) and 256 threads x 20
// chunks (rows up to 40960 entries).  A chunk is one 16-byte vector per thread.  Needs
// V % 8 == 0 and 16-byte aligned rows of logits and grad.  resident_blocks_per_cu() is the
// occupancy the runtime reports for the shape.
constexpr int kResidentChunksBig = 38;
constexpr int kResidentChunksSmall = 20;
hipError_t launch_resident(const KParams& p, int threads, int grid, hipStream_t s);
int resident_blocks_per_cu(int threads);

// loss[0] = loss_scale * sum(partial[0..n)) in a fixed order.
hipError_t launch_finalize(const double* partial, int n, float loss_scale, float* loss, hipStream_t s);

}  // namespace dppo
