// Host-side launch entry points of the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include "dppo_common.hpp"

namespace dppo {

// General two-pass kernel.  vec=false selects the element-wise variant (needed when logits
// and grad_logits rows do not share their 16-byte misalignment).
hipError_t launch_streaming(const KParams& p, bool vec, bool grad, int threads, int grid, hipStream_t s);

// loss[0] = loss_scale * sum(partial[0..n)) in a fixed order.
hipError_t launch_finalize(const double* partial, int n, float loss_scale, float* loss, hipStream_t s);

}  // namespace dppo
