// C ABI of the DPPO loss library: argument checks, kernel-path choice, launches.
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdint>
#include <mutex>

#include "dppo.h"
#include "dppo_common.hpp"
#include "dppo_launch.hpp"

namespace {

struct DeviceInfo {
  int cus = 0;
};

// Compute-unit count of a device, queried once per device.
const DeviceInfo& device_info(int dev) {
  static DeviceInfo info[64];
  static std::once_flag once[64];
  if (dev < 0 || dev >= 64) dev = 0;
  std::call_once(once[dev], [dev]() {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    info[dev].cus = n;
  });
  return info[dev];
}

thread_local const char* g_last_path = "none";

dppo_status_t check_args(const dppo_args_t* a, bool grad) {
  if (!a) return DPPO_ERR_NULL;
  if (a->T < 0 || a->V < 1 || a->ld < a->V || a->V >= (int64_t(1) << 31) || a->T >= (int64_t(1) << 31)) return DPPO_ERR_SHAPE;
  if (a->variant < DPPO_BINARY_TV || a->variant > DPPO_FULL_KL) return DPPO_ERR_VARIANT;
  if (a->K < 0 || a->K > DPPO_KMAX) return DPPO_ERR_K;
  const bool topk = (a->variant == DPPO_TOPK_TV || a->variant == DPPO_TOPK_KL);
  if (topk && a->K > 0 && (!a->mu_topk_ids || !a->mu_topk_logp)) return DPPO_ERR_K;
  if (!a->loss) return DPPO_ERR_NULL;
  if (std::isnan(a->delta) || std::isnan(a->loss_scale) || std::isnan(a->ratio_cap)) return DPPO_ERR_VALUE;
  if (a->mask_rule < DPPO_MASK_DIVERGENCE || a->mask_rule > DPPO_MASK_NONE) return DPPO_ERR_VALUE;
  if (a->mask_rule == DPPO_MASK_RATIO_CLIP && !(a->eps_low >= 0.f && a->eps_low < 1.f && a->eps_high >= 0.f)) return DPPO_ERR_VALUE;
  if (!a->workspace || a->workspace_bytes < dppo_workspace_bytes(a->T, a->V, a->K)) return DPPO_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(a->workspace) & 7u) return DPPO_ERR_ALIGN;
  if (a->T > 0) {
    if (!a->logits || !a->sampled_ids || !a->mu_logp || !a->advantages || !a->divergence || !a->mask) return DPPO_ERR_NULL;
    if (grad && !a->grad_logits) return DPPO_ERR_NULL;
    if (a->variant == DPPO_FULL_TV || a->variant == DPPO_FULL_KL) {
      if (!a->mu_logits) return DPPO_ERR_NULL;
      if (a->mu_ld < a->V) return DPPO_ERR_SHAPE;
      if (reinterpret_cast<uintptr_t>(a->mu_logits) & 1u) return DPPO_ERR_ALIGN;
    }
    if (reinterpret_cast<uintptr_t>(a->logits) & 1u) return DPPO_ERR_ALIGN;
    if (grad && (reinterpret_cast<uintptr_t>(a->grad_logits) & 1u)) return DPPO_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(a->diagnostics) & 15u) return DPPO_ERR_ALIGN;
  }
  return DPPO_OK;
}

dppo_status_t run(const dppo_args_t* a, void* stream, bool grad) {
  const dppo_status_t st = check_args(a, grad);
  if (st != DPPO_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  double* partial = static_cast<double*>(a->workspace);
  const int max_parts = static_cast<int>(DPPO_WORKSPACE_BYTES / sizeof(double));

  int nparts = 0;
  if (a->T > 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return DPPO_ERR_LAUNCH;
    const int cus = device_info(dev).cus;

    dppo::KParams p;
    p.logits = static_cast<const uint16_t*>(a->logits);
    p.grad = grad ? static_cast<uint16_t*>(a->grad_logits) : nullptr;
    p.sampled = a->sampled_ids;
    p.mu_logp = a->mu_logp;
    const bool topk = (a->variant == DPPO_TOPK_TV || a->variant == DPPO_TOPK_KL);
    p.tk_ids = topk ? a->mu_topk_ids : nullptr;
    p.tk_lp = topk ? a->mu_topk_logp : nullptr;
    p.K = topk ? a->K : 0;
    p.adv = a->advantages;
    p.loss_tok = a->loss_tok;
    p.divergence = a->divergence;
    p.mask = a->mask;
    p.diag = a->diagnostics;
    p.partial = partial;
    p.ld = a->ld;
    p.T = static_cast<int32_t>(a->T);
    p.V = static_cast<int32_t>(a->V);
    p.variant = a->variant;
    p.delta = a->delta;
    p.loss_scale = a->loss_scale;
    p.mask_rule = a->mask_rule;
    p.eps_low = a->eps_low;
    p.eps_high = a->eps_high;
    p.ratio_cap = (a->ratio_cap > 0.f && std::isfinite(a->ratio_cap)) ? a->ratio_cap : 0.f;   // 0: no cap
    const bool full = (a->variant == DPPO_FULL_TV || a->variant == DPPO_FULL_KL);
    p.mu_logits = full ? static_cast<const uint16_t*>(a->mu_logits) : nullptr;
    p.mu_ld = full ? a->mu_ld : 0;

    const uintptr_t lz = reinterpret_cast<uintptr_t>(a->logits), lg = reinterpret_cast<uintptr_t>(a->grad_logits);
    // Register-resident kernel: rows of 8192 .. 155648 entries, a multiple of 8, 16-byte aligned.
    int r_threads = 0, r_chunks = 0;
    const bool resident = !full && !(a->flags & DPPO_FLAG_FORCE_STREAMING) && (a->ld % 8 == 0) && ((lz | (grad ? lg : 0)) & 15u) == 0 &&
                          dppo::resident_shape(a->V, &r_threads, &r_chunks);
    if (full) {
      // Two rows per workgroup in flight: one workgroup of 1024 threads per compute unit keeps the
      // rows that pass 2 and 3 re-read within reach of the caches.
      const int threads = (a->V >= 65536) ? 1024 : (a->V >= 8192 ? 512 : 256);
      int64_t grid = static_cast<int64_t>(cus) * (1024 / threads);
      if (grid > a->T) grid = a->T;
      if (grid > max_parts) grid = max_parts;
      nparts = static_cast<int>(grid);
      if (dppo::launch_fullvocab(p, a->variant == DPPO_FULL_TV, grad, threads, nparts, s) != hipSuccess) return DPPO_ERR_LAUNCH;
      g_last_path = "fullvocab";
    } else if (resident) {
      int64_t grid = static_cast<int64_t>(cus) * dppo::resident_blocks_per_cu(grad, r_threads, r_chunks);
      if (grid > a->T) grid = a->T;
      if (grid > max_parts) grid = max_parts;
      nparts = static_cast<int>(grid);
      if (dppo::launch_resident(p, grad, r_threads, r_chunks, nparts, s) != hipSuccess) return DPPO_ERR_LAUNCH;
      g_last_path = "resident";
    } else {
      // 16-byte vectors need logits and grad rows to share their misalignment.
      const bool vec = !grad || (((lz - lg) & 15u) == 0);
      // Workgroup size by row length; a few rows in flight per compute unit so that the re-read
      // of pass 2 still finds the row in cache.
      const int threads = (a->V >= 65536) ? 1024 : (a->V >= 8192 ? 512 : 256);
      const int per_cu = 2048 / threads;
      int64_t grid = static_cast<int64_t>(cus) * per_cu;
      if (grid > a->T) grid = a->T;
      if (grid > max_parts) grid = max_parts;
      nparts = static_cast<int>(grid);
      if (dppo::launch_streaming(p, vec, grad, threads, nparts, s) != hipSuccess) return DPPO_ERR_LAUNCH;
      g_last_path = "streaming";
    }
  }
  if (dppo::launch_finalize(partial, nparts, a->loss_scale, a->loss, s) != hipSuccess) return DPPO_ERR_LAUNCH;
  return DPPO_OK;
}

}  // namespace

extern "C" {

size_t dppo_workspace_bytes(int64_t, int64_t, int32_t) { return DPPO_WORKSPACE_BYTES; }

dppo_status_t dppo_loss_fwd(const dppo_args_t* args, void* stream) { return run(args, stream, false); }

dppo_status_t dppo_loss_fwd_bwd(const dppo_args_t* args, void* stream) { return run(args, stream, true); }

const char* dppo_status_str(dppo_status_t status) {
  switch (status) {
    case DPPO_OK: return "ok";
    case DPPO_ERR_NULL: return "a required pointer is NULL";
    case DPPO_ERR_SHAPE: return "bad shape: need T >= 0, 1 <= V <= ld (and <= mu_ld for DPPO_FULL_*), T and V below 2^31";
    case DPPO_ERR_ALIGN: return "misaligned pointer: bf16 buffers need 2-byte, workspace 8-byte, diagnostics 16-byte alignment";
    case DPPO_ERR_VARIANT: return "variant is not one of DPPO_BINARY_TV/KL, DPPO_TOPK_TV/KL, DPPO_FULL_TV/KL";
    case DPPO_ERR_K: return "bad K: need 0 <= K <= DPPO_KMAX and top-K pointers when K > 0";
    case DPPO_ERR_WORKSPACE: return "workspace missing or smaller than dppo_workspace_bytes()";
    case DPPO_ERR_LAUNCH: return "HIP kernel launch failed";
    case DPPO_ERR_VALUE: return "bad value: NaN delta / loss_scale / ratio_cap, unknown mask_rule, or clip range outside 0 <= eps_low < 1, eps_high >= 0";
  }
  return "unknown status";
}

int dppo_version(void) { return DPPO_VERSION; }

size_t dppo_args_size(void) { return sizeof(dppo_args_t); }

const char* dppo_last_path(void) { return g_last_path; }

}  // extern "C"
