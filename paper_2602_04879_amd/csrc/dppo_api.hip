// C ABI of the DPPO loss library: argument checks, kernel-path choice, launches.
#include <hip/hip_runtime.h>
#include <cmath>
#include <limits>
#include <atomic>
#include <cstdint>
#include <mutex>

#include "dppo.h"
#include "dppo_common.hpp"
#include "dppo_launch.hpp"

// Scratch of dppo_loss_fwd_bwd_static: the per-workgroup partial sums of the loss, in device memory
// that every GPU the library runs on holds from the moment the library is loaded there.  In host
// code this name is only a handle for hipGetSymbolAddress; the device address it yields (one per
// GPU) is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[DPPO_STATIC_SCRATCH_BYTES];

namespace {

// Device address of `scratch` on device `dev`, which must be the current device; asked of the
// runtime once per device.  nullptr if the runtime refuses.
void* static_scratch(int dev) {
  static void* ptr[64];
  static std::once_flag once[64];
  if (dev < 0 || dev >= 64) return nullptr;
  std::call_once(once[dev], [dev]() {
    void* q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess) q = nullptr;
    ptr[dev] = q;
  });
  return ptr[dev];
}

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

// The device a stream belongs to (NULL: the current device).
bool stream_device(hipStream_t s, int* dev) {
  hipDevice_t d = 0;
  if (s != nullptr && hipStreamGetDevice(s, &d) == hipSuccess) {
    *dev = static_cast<int>(d);
    return true;
  }
  return hipGetDevice(dev) == hipSuccess;
}

// Workgroups per compute unit of a register-resident shape: a constant of (device, shape, form),
// asked of the runtime once and kept.
int resident_blocks_per_cu_cached(int dev, bool grad, bool dyn, bool ragged, int threads, int chunks) {
  static std::atomic<int> cache[64][8][3][41];
  if (dev < 0 || dev >= 64 || chunks < 0 || chunks > 40) return dppo::resident_blocks_per_cu(grad, dyn, ragged, threads, chunks);
  std::atomic<int>& slot = cache[dev][(grad ? 1 : 0) + (dyn ? 2 : 0) + (ragged ? 4 : 0)][threads == 512 ? 2 : threads == 256 ? 1 : 0][chunks];
  int n = slot.load(std::memory_order_relaxed);
  if (n == 0) {
    n = dppo::resident_blocks_per_cu(grad, dyn, ragged, threads, chunks);
    slot.store(n, std::memory_order_relaxed);
  }
  return n;
}

thread_local const char* g_last_path = "none";

dppo_status_t check_args(const dppo_args_t* a, bool grad, bool own_scratch = false) {
  if (!a) return DPPO_ERR_NULL;
  if (a->T < 0 || a->V < 1 || a->ld < a->V || a->V >= (int64_t(1) << 31) || a->T >= (int64_t(1) << 31)) return DPPO_ERR_SHAPE;
  if (a->variant < DPPO_BINARY_TV || a->variant > DPPO_FULL_KL) return DPPO_ERR_VARIANT;
  if (a->K < 0 || a->K > DPPO_KMAX) return DPPO_ERR_K;
  const bool topk = (a->variant == DPPO_TOPK_TV || a->variant == DPPO_TOPK_KL);
  if (topk && a->K > 0 && a->T > 0 && (!a->mu_topk_ids || !a->mu_topk_logp)) return DPPO_ERR_K;
  if (!a->loss) return DPPO_ERR_NULL;
  if (std::isnan(a->delta) || std::isnan(a->loss_scale) || std::isnan(a->ratio_cap)) return DPPO_ERR_VALUE;
  if (a->mask_rule < DPPO_MASK_DIVERGENCE || a->mask_rule > DPPO_MASK_NONE) return DPPO_ERR_VALUE;
  if (a->mask_rule == DPPO_MASK_RATIO_CLIP && !(a->eps_low >= 0.f && a->eps_low < 1.f && a->eps_high >= 0.f)) return DPPO_ERR_VALUE;
  if (!(a->relax_alpha >= 0.f && a->relax_alpha <= 1.f) || (a->relax_sides & ~(DPPO_RELAX_HIGH | DPPO_RELAX_LOW))) return DPPO_ERR_VALUE;
  if (!own_scratch) {
    if (!a->workspace || a->workspace_bytes < DPPO_WORKSPACE_BYTES) return DPPO_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(a->workspace) & 7u) return DPPO_ERR_ALIGN;
  }
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

// The kernel arguments of one (validated) call, scratch pointers left empty.
dppo::KParams make_kparams(const dppo_args_t* a, bool grad) {
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
  p.partial = nullptr;
  p.row_counters = nullptr;
  p.row_loss = nullptr;
  p.gath = nullptr;
  p.anchor_logp = a->anchor_logp;
  const bool relax = a->mask_rule == DPPO_MASK_RATIO_CLIP && a->relax_alpha > 0.f && a->relax_sides != 0;
  p.relax_log_alpha = relax ? std::log(static_cast<double>(a->relax_alpha)) : -std::numeric_limits<double>::infinity();
  p.relax_sides = relax ? static_cast<int32_t>(a->relax_sides) : 0;
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
  return p;
}

// Device scratch of one loss launch.  partial: one loss partial sum per workgroup (max_parts of
// them).  counters / row_loss (both or neither): the row counter and one loss term per row,
// for the kernel form that hands its rows out at run time.
struct LossScratch {
  double* partial = nullptr;
  int max_parts = 0;
  int32_t* counters = nullptr;
  double* row_loss = nullptr;
};
// The layout of a caller's workspace: [partial sums, 32 KiB | counters | unused up to 64 KiB | row loss terms, 8 T bytes]
constexpr size_t kPartialBytes = 32768;
LossScratch scratch_of(void* base, size_t bytes, int64_t T) {
  LossScratch sc;
  char* b = static_cast<char*>(base);
  sc.partial = reinterpret_cast<double*>(b);
  sc.max_parts = static_cast<int>(kPartialBytes / sizeof(double));
  if (bytes >= DPPO_WORKSPACE_BYTES + static_cast<size_t>(T) * sizeof(double)) {
    sc.counters = reinterpret_cast<int32_t*>(b + kPartialBytes);
    sc.row_loss = reinterpret_cast<double*>(b + DPPO_WORKSPACE_BYTES);
  }
  return sc;
}

// Rows handed out at run time (the persistent one-workgroup-per-compute-unit kernels with the
// gradient): possible when the caller's scratch has the counter and the per-row loss terms, the
// grid is a multiple of the eight dies, every workgroup gets a dozen rows or more, and the caller
// did not ask for fixed rows.  (With fewer rows the hand-out costs more than the uneven dies: a
// workgroup commits to two rows ahead, and a counter-clearing kernel precedes the launch.  Measured
// at V = 151936, rows at run time against fixed rows: 4 rows per compute unit 133 / 126 us, 8:
// 250 / 246, 16: 462 / 468, 32: 881 / 913.)
bool rows_at_run_time(const dppo_args_t* a, const LossScratch& sc, int64_t grid) {
  return sc.counters && grid % 8 == 0 && a->T >= 12 * grid && !(a->flags & DPPO_FLAG_STATIC_ROWS);
}
// Points the kernel at the counter (cleared by a small kernel first: no memset, so a call stays
// capturable) and at the per-row loss terms, which the reduction then sums instead of the
// per-workgroup partial sums.
dppo_status_t arm_rows_at_run_time(dppo::KParams& p, const dppo_args_t* a, const LossScratch& sc, const double** fin, int* fin_n, hipStream_t s) {
  p.row_counters = sc.counters;
  p.row_loss = sc.row_loss;
  if (dppo::launch_clear_counters(sc.counters, s) != hipSuccess) return DPPO_ERR_LAUNCH;
  *fin = sc.row_loss;
  *fin_n = static_cast<int>(a->T);
  return DPPO_OK;
}

// Rows of middle length in groups of rows per workgroup: the number of groups per compute unit from
// which that form is taken.  A group is 23 us of a compute unit's time: with few of them a call ends
// sooner on the one-row shapes, whose unit of work is a row.  Measured, per shape: groups of 4
// rows (V up to 32768) gain 1 % at 16 groups per compute unit, 5 % at 32, 7.5 % at 64, and lose
// below; groups of 6 (up to 24576) are even at 16, gain 4 % at 24, 6 % at 32; groups of 2 (up to
// 65536) gain 1.5-7 % from 32 on; groups of 3 (up to 40960 / 49152) are even at 8-12 groups per
// compute unit and gain 0-3 % at 16, 3.5-9 % at 32.
int64_t multi_min_groups(int rows) { return rows == 3 ? 16 : rows == 2 ? 32 : 24; }

// Launch the loss kernel of one (already validated) call.  Afterwards the scalar loss is
// loss_scale times the sum of fin[0 .. *fin_n) (per-workgroup partial sums, or per-row terms).
dppo_status_t launch_loss(const dppo_args_t* a, bool grad, const LossScratch& sc, const double** fin, int* fin_n, hipStream_t s) {
  double* partial = sc.partial;
  const int max_parts = sc.max_parts;
  *fin = partial;
  int nparts = 0;
  if (a->T > 0) {
    int dev = 0;
    if (!stream_device(s, &dev)) return DPPO_ERR_LAUNCH;
    const int cus = device_info(dev).cus;

    dppo::KParams p = make_kparams(a, grad);
    p.partial = partial;
    const bool full = (a->variant == DPPO_FULL_TV || a->variant == DPPO_FULL_KL);

    const uintptr_t lz = reinterpret_cast<uintptr_t>(a->logits), lg = reinterpret_cast<uintptr_t>(a->grad_logits);
    // Register-resident kernel: rows of 1024 .. 155648 entries.  A multiple of 8 and 16-byte aligned:
    // the plain form; else its ragged form, if logits and gradient share their misalignment.
    int r_threads = 0, r_chunks = 0;
    const bool aligned = (a->V % 8 == 0) && (a->ld % 8 == 0) && ((lz | (grad ? lg : 0)) & 15u) == 0;
    const bool ragged_ok = !grad || ((lz - lg) & 15u) == 0;
    // Rows of 16384 entries and more that are 16-byte aligned but do not start on 128-byte lines
    // are faster in the ragged form, whose accesses are whole lines (measured +1.4 % at 20008
    // entries, +5 % at 32008 .. 151944; shorter rows lose 2-10 %), unless the form with several
    // rows per workgroup takes them (decided below).
    const bool on_lines = aligned && (a->ld % 64 == 0) && ((lz | (grad ? lg : 0)) & 127u) == 0;
    int l_threads = 0, l_chunks = 0;
    const bool prefer_lines = aligned && !on_lines && ragged_ok && a->V >= 16384 && dppo::resident_shape(a->V, true, &l_threads, &l_chunks);
    bool ragged = !aligned && ragged_ok;
    bool resident = !full && !(a->flags & DPPO_FLAG_FORCE_STREAMING) && (aligned || ragged) &&
                    dppo::resident_shape(a->V, ragged, &r_threads, &r_chunks);
    // Longer rows, forward + backward: the long-row form of the same kernel, up to 262144 entries.
    const int long_chunks = (!full && grad && !resident && !(a->flags & DPPO_FLAG_FORCE_STREAMING) && aligned)
                                ? dppo::resident_long_chunks(a->V) : 0;
    // Rows of middle length, forward + backward, when rows can be handed out at run time and every
    // compute unit gets several groups of them: several rows per workgroup.
    int m_rows = 0, m_chunks = 0;
    const bool m_ragged = !on_lines;        // (resident and not aligned: the ragged form applies, see above)
    const bool m_shape = resident && grad && ragged_ok && dppo::resident_multi_shape(a->V, m_ragged, &m_rows, &m_chunks);
    const int64_t m_groups = m_shape ? (a->T + m_rows - 1) / m_rows : 0;
    const bool multi = m_shape && sc.counters && !(a->flags & DPPO_FLAG_STATIC_ROWS) && m_groups >= multi_min_groups(m_rows) * cus;
    if (resident && !multi && prefer_lines) {
      ragged = true;
      r_threads = l_threads;
      r_chunks = l_chunks;
    }
    const bool tv_full = a->variant == DPPO_FULL_TV;
    const int fr_chunks = (full && !(a->flags & DPPO_FLAG_FORCE_STREAMING)) ? dppo::fullvocab_resident_chunks(p, tv_full, grad) : 0;
    if (fr_chunks) {
      // long aligned rows (backward, or the TV form): the trainer's row stays in registers, one workgroup per compute unit
      int64_t grid = cus;
      if (grid > a->T) grid = a->T;
      if (grid > max_parts) grid = max_parts;
      nparts = static_cast<int>(grid);
      // with the gradient and several rows per workgroup: rows handed out at run time
      const bool dyn = grad && rows_at_run_time(a, sc, grid);
      if (dyn && arm_rows_at_run_time(p, a, sc, fin, fin_n, s) != DPPO_OK) return DPPO_ERR_LAUNCH;
      if (dppo::launch_fullvocab_resident(p, tv_full, grad, fr_chunks, nparts, s) != hipSuccess) return DPPO_ERR_LAUNCH;
      g_last_path = "fullvocab_resident";
      if (dyn) return DPPO_OK;
    } else if (full) {
      // Two rows per workgroup in flight: one workgroup of 1024 threads per compute unit keeps the
      // rows that pass 2 and 3 re-read within reach of the caches.
      const int threads = (a->V >= 65536) ? 1024 : (a->V >= 8192 ? 512 : 256);
      int64_t grid = static_cast<int64_t>(cus) * (1024 / threads);
      if (grid > a->T) grid = a->T;
      if (grid > max_parts) grid = max_parts;
      nparts = static_cast<int>(grid);
      if (dppo::launch_fullvocab(p, a->variant == DPPO_FULL_TV, grad, threads, nparts, s) != hipSuccess) return DPPO_ERR_LAUNCH;
      g_last_path = "fullvocab";
    } else if (long_chunks) {
      // rows beyond the register file: registers + LDS + a re-read tail, one workgroup per compute unit
      int64_t grid = cus;
      if (grid > a->T) grid = a->T;
      if (grid > max_parts) grid = max_parts;
      nparts = static_cast<int>(grid);
      const bool dyn = rows_at_run_time(a, sc, grid);
      if (dyn && arm_rows_at_run_time(p, a, sc, fin, fin_n, s) != DPPO_OK) return DPPO_ERR_LAUNCH;
      if (dppo::launch_resident_long(p, long_chunks, nparts, s) != hipSuccess) return DPPO_ERR_LAUNCH;
      g_last_path = "resident_long";
      if (dyn) return DPPO_OK;
    } else if (resident && multi) {
      // rows of middle length, forward + backward: groups of rows per workgroup, one workgroup per compute unit
      nparts = static_cast<int>(cus);
      if (arm_rows_at_run_time(p, a, sc, fin, fin_n, s) != DPPO_OK) return DPPO_ERR_LAUNCH;
      if (dppo::launch_resident_multi(p, m_ragged, m_rows, m_chunks, nparts, s) != hipSuccess) return DPPO_ERR_LAUNCH;
      g_last_path = "resident_multi";
      return DPPO_OK;
    } else if (resident) {
      int per_cu = resident_blocks_per_cu_cached(dev, grad, false, ragged, r_threads, r_chunks);
      int64_t grid = static_cast<int64_t>(cus) * per_cu;
      if (grid > a->T) grid = a->T;
      if (grid > max_parts) grid = max_parts;
      // With the gradient and one workgroup per compute unit (the long rows), rows are handed out at
      // run time: the dies do not run at one speed, and the slowest one would end the kernel.  (The
      // forward-only form and the shapes with several workgroups per compute unit measure slower
      // that way: their waves run ahead of wave 0, which would have to wait for the counter.)
      bool dyn = false;
      if (grad && r_threads == 512 && per_cu == 1) {
        // the form that draws its rows has its own register count, so its own occupancy
        const int64_t grid_dyn = static_cast<int64_t>(cus) * resident_blocks_per_cu_cached(dev, grad, true, ragged, r_threads, r_chunks);
        if (grid_dyn <= max_parts && rows_at_run_time(a, sc, grid_dyn)) {
          grid = grid_dyn;
          dyn = true;
        }
      }
      nparts = static_cast<int>(grid);
      if (dyn && arm_rows_at_run_time(p, a, sc, fin, fin_n, s) != DPPO_OK) return DPPO_ERR_LAUNCH;
      if (dppo::launch_resident(p, grad, ragged, r_threads, r_chunks, nparts, s) != hipSuccess) return DPPO_ERR_LAUNCH;
      g_last_path = "resident";
      if (p.row_counters) return DPPO_OK;
    } else {
      // 16-byte vectors need logits and grad rows to share their misalignment.
      const bool vec = !grad || (((lz - lg) & 15u) == 0);
      // Workgroup size by row length: few rows in flight per compute unit, so that the re-read of
      // pass 2 still finds the row in cache.  Forward only there is no second pass, and many short
      // workgroups are better: one row's epilogue then runs while the others' rows stream
      // (V = 256000: 5.5 against 4.6 TB/s with 1024 threads).
      const int threads = !grad ? 256 : (a->V >= 65536) ? 1024 : (a->V >= 8192 ? 512 : 256);
      const int per_cu = 2048 / threads;
      int64_t grid = static_cast<int64_t>(cus) * per_cu;
      if (grid > a->T) grid = a->T;
      if (grid > max_parts) grid = max_parts;
      nparts = static_cast<int>(grid);
      if (dppo::launch_streaming(p, vec, grad, threads, nparts, s) != hipSuccess) return DPPO_ERR_LAUNCH;
      g_last_path = "streaming";
    }
  }
  *fin_n = nparts;
  return DPPO_OK;
}

dppo_status_t run(const dppo_args_t* a, void* stream, bool grad) {
  dppo_status_t st = check_args(a, grad);
  if (st != DPPO_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const LossScratch sc = scratch_of(a->workspace, a->workspace_bytes, a->T);
  const double* fin = nullptr;
  int fin_n = 0;
  st = launch_loss(a, grad, sc, &fin, &fin_n, s);
  if (st != DPPO_OK) return st;
  if (dppo::launch_finalize(fin, fin_n, a->loss_scale, a->loss, s) != hipSuccess) return DPPO_ERR_LAUNCH;
  return DPPO_OK;
}

// The same call with the partial sums in the library's own static device array instead of the
// caller's workspace: nothing is allocated, here or by the caller.
dppo_status_t run_static(const dppo_args_t* a, void* stream) {
  dppo_status_t st = check_args(a, true, true);
  if (st != DPPO_OK) return st;
  if (a->T > DPPO_STATIC_MAX_T) return DPPO_ERR_SHAPE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int cur = 0, dev = 0;
  if (hipGetDevice(&cur) != hipSuccess || !stream_device(s, &dev)) return DPPO_ERR_LAUNCH;
  if (dev != cur) return DPPO_ERR_LAUNCH;          // each GPU has its own copy of the array: the current one's is used
  void* base = static_scratch(cur);
  if (!base) return DPPO_ERR_WORKSPACE;
  // (with 64 KiB there is no room for per-row loss terms: every workgroup takes the rows its index fixes)
  const LossScratch sc = scratch_of(base, DPPO_STATIC_SCRATCH_BYTES, a->T);
  const double* fin = nullptr;
  int fin_n = 0;
  st = launch_loss(a, true, sc, &fin, &fin_n, s);
  if (st != DPPO_OK) return st;
  if (dppo::launch_finalize(fin, fin_n, a->loss_scale, a->loss, s) != hipSuccess) return DPPO_ERR_LAUNCH;
  return DPPO_OK;
}

// ---- the logits-free path: hidden states and lm_head weight in, gradient of the hidden states out

constexpr int64_t kLmheadDefaultChunk = 8192;

int64_t lmhead_chunk_rows(const dppo_lmhead_args_t* a) {
  int64_t c = a->chunk_rows > 0 ? a->chunk_rows : kLmheadDefaultChunk;
  if (c > a->loss.T) c = a->loss.T;
  return c < 1 ? 1 : c;
}

size_t align256(size_t n) { return (n + 255u) & ~static_cast<size_t>(255u); }

// Forward only: [64 KiB | one loss term per row | per chunk: tile statistics, 16 bytes per row and
// 256-column tile | per chunk: the logits at the sampled and top-K ids, 4 (K + 1) bytes per row]
size_t lmhead_fwd_workspace(int64_t T, int64_t V, int32_t K, int64_t chunk_rows) {
  int64_t c = chunk_rows > 0 ? chunk_rows : kLmheadDefaultChunk;
  if (c > T) c = T;
  if (c < 1) c = 1;
  const size_t tiles_n = static_cast<size_t>((V + dppo::kGemmTileN - 1) / dppo::kGemmTileN);
  return DPPO_WORKSPACE_BYTES + align256(static_cast<size_t>(T > 0 ? T : 0) * sizeof(double)) +
         align256(static_cast<size_t>(c) * tiles_n * 16) + align256(static_cast<size_t>(c) * static_cast<size_t>(K + 1) * 4);
}

// Forward + backward: [partial sums | one chunk of logits, which becomes the chunk's logit gradient
// in place]; never less than the forward-only call needs with the largest K.
size_t lmhead_workspace(int64_t T, int64_t V, int64_t chunk_rows) {
  int64_t c = chunk_rows > 0 ? chunk_rows : kLmheadDefaultChunk;
  if (c > T) c = T;
  if (c < 1) c = 1;
  size_t b = DPPO_WORKSPACE_BYTES;
  b += static_cast<size_t>(c) * static_cast<size_t>(V) * 2;
  const size_t f = lmhead_fwd_workspace(T, V, DPPO_KMAX, chunk_rows);
  return b > f ? b : f;
}

dppo_status_t run_lmhead(const dppo_lmhead_args_t* a, void* stream, bool grad) {
  if (!a) return DPPO_ERR_NULL;
  const int64_t T = a->loss.T, V = a->loss.V, d = a->d;
  if (T < 0 || V < 64 || V % 64 != 0 || d < 64 || d % 64 != 0 || a->ld_hidden < d || a->ld_weight < d ||
      a->ld_hidden % 8 != 0 || a->ld_weight % 8 != 0 || V >= (int64_t(1) << 22) || d >= (int64_t(1) << 22))
    return DPPO_ERR_SHAPE;
  if (a->loss.variant == DPPO_FULL_TV || a->loss.variant == DPPO_FULL_KL) return DPPO_ERR_VARIANT;
  if (grad && (a->ld_grad_hidden < d)) return DPPO_ERR_SHAPE;
  const int64_t chunk = lmhead_chunk_rows(a);
  const bool want_gw = grad && a->grad_weight != nullptr;
  if (want_gw && (a->ld_grad_weight < d || a->ld_grad_weight % 4 != 0)) return DPPO_ERR_SHAPE;
  if (want_gw && (reinterpret_cast<uintptr_t>(a->grad_weight) & 15u)) return DPPO_ERR_ALIGN;
  // Forward only, nothing of size [chunk, V] is needed: the first product leaves softmax statistics
  // instead of logits (unless the caller asks for the general kernels, for comparison).
  const bool fused_fwd = !grad && !(a->loss.flags & DPPO_FLAG_FORCE_STREAMING);
  if (a->loss.K < 0 || a->loss.K > DPPO_KMAX) return DPPO_ERR_K;
  const bool topk_variant = (a->loss.variant == DPPO_TOPK_TV || a->loss.variant == DPPO_TOPK_KL);
  const int32_t Ktop = topk_variant ? a->loss.K : 0;
  if (!a->workspace || a->workspace_bytes < (fused_fwd ? lmhead_fwd_workspace(T, V, Ktop, a->chunk_rows) : lmhead_workspace(T, V, a->chunk_rows)))
    return DPPO_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(a->workspace) & 255u) return DPPO_ERR_ALIGN;
  if (T > 0) {
    if (!a->hidden || !a->weight || (grad && !a->grad_hidden)) return DPPO_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(a->hidden) | reinterpret_cast<uintptr_t>(a->weight)) & 15u)
      return DPPO_ERR_ALIGN;
    if (grad && (reinterpret_cast<uintptr_t>(a->grad_hidden) & 1u)) return DPPO_ERR_ALIGN;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(a->workspace);
  double* partial = reinterpret_cast<double*>(ws);
  uint16_t* zbuf = reinterpret_cast<uint16_t*>(ws + DPPO_WORKSPACE_BYTES);

  // validate the loss arguments on the first chunk's view before anything is launched
  dppo_args_t c = a->loss;
  c.logits = zbuf;
  c.grad_logits = zbuf;
  c.ld = V;
  c.workspace = ws;
  c.workspace_bytes = DPPO_WORKSPACE_BYTES;
  const dppo_status_t st0 = check_args(&c, grad);
  if (st0 != DPPO_OK) return st0;

  if (fused_fwd) {
    const int tiles_n = static_cast<int>((V + dppo::kGemmTileN - 1) / dppo::kGemmTileN);
    double* row_loss = reinterpret_cast<double*>(ws + DPPO_WORKSPACE_BYTES);
    char* part = ws + DPPO_WORKSPACE_BYTES + align256(static_cast<size_t>(T) * sizeof(double));
    char* gath = part + align256(static_cast<size_t>(chunk) * static_cast<size_t>(tiles_n) * 16);
    for (int64_t r0 = 0; r0 < T; r0 += chunk) {
      const int64_t rows = (T - r0 < chunk) ? (T - r0) : chunk;
      c.T = rows;
      c.sampled_ids = a->loss.sampled_ids + r0;
      c.mu_logp = a->loss.mu_logp + r0;
      c.advantages = a->loss.advantages + r0;
      c.anchor_logp = a->loss.anchor_logp ? a->loss.anchor_logp + r0 : nullptr;
      c.mu_topk_ids = a->loss.mu_topk_ids ? a->loss.mu_topk_ids + r0 * a->loss.K : nullptr;
      c.mu_topk_logp = a->loss.mu_topk_logp ? a->loss.mu_topk_logp + r0 * a->loss.K : nullptr;
      c.loss_tok = a->loss.loss_tok ? a->loss.loss_tok + r0 : nullptr;
      c.divergence = a->loss.divergence + r0;
      c.mask = a->loss.mask + r0;
      c.diagnostics = a->loss.diagnostics ? a->loss.diagnostics + r0 * DPPO_NDIAG : nullptr;
      dppo::KParams p = make_kparams(&c, false);
      p.logits = nullptr;
      dppo::GemmStats gs;
      gs.part = reinterpret_cast<dppo::gemm_f32x4*>(part);
      gs.gath = reinterpret_cast<float*>(gath);
      gs.sampled = p.sampled;
      gs.tk_ids = p.tk_ids;
      gs.Ktop = p.K;
      gs.tiles_n = tiles_n;
      p.gath = gs.gath;
      const uint16_t* h = static_cast<const uint16_t*>(a->hidden) + r0 * a->ld_hidden;
      if (dppo::launch_gemm_stats(h, a->ld_hidden, static_cast<const uint16_t*>(a->weight), a->ld_weight, static_cast<int>(rows),
                                  static_cast<int>(V), static_cast<int>(d), gs, s) != hipSuccess)
        return DPPO_ERR_LAUNCH;
      if (dppo::launch_lmhead_rows(p, gs, row_loss + r0, s) != hipSuccess) return DPPO_ERR_LAUNCH;
    }
    if (dppo::launch_finalize(row_loss, static_cast<int>(T), a->loss.loss_scale, a->loss.loss, s) != hipSuccess) return DPPO_ERR_LAUNCH;
    if (T > 0) g_last_path = "lmhead_fused";
    return DPPO_OK;
  }
  const int max_parts = static_cast<int>(kPartialBytes / sizeof(double));
  const int64_t nchunks = T > 0 ? (T + chunk - 1) / chunk : 0;
  const int parts_per_chunk = nchunks > 0 ? static_cast<int>(max_parts / nchunks) : max_parts;
  if (nchunks > 0 && parts_per_chunk < 1) return DPPO_ERR_SHAPE;
  int used = 0;
  for (int64_t r0 = 0; r0 < T; r0 += chunk) {
    const int64_t rows = (T - r0 < chunk) ? (T - r0) : chunk;
    const uint16_t* h = static_cast<const uint16_t*>(a->hidden) + r0 * a->ld_hidden;
    // logits of the chunk (bf16, as a trainer's lm_head produces them)
    if (dppo::launch_gemm_nt(h, a->ld_hidden, static_cast<const uint16_t*>(a->weight), a->ld_weight, zbuf, V,
                             static_cast<int>(rows), static_cast<int>(V), static_cast<int>(d), 0, s) != hipSuccess)
      return DPPO_ERR_LAUNCH;
    c.T = rows;
    c.sampled_ids = a->loss.sampled_ids + r0;
    c.mu_logp = a->loss.mu_logp + r0;
    c.advantages = a->loss.advantages + r0;
    c.anchor_logp = a->loss.anchor_logp ? a->loss.anchor_logp + r0 : nullptr;
    c.mu_topk_ids = a->loss.mu_topk_ids ? a->loss.mu_topk_ids + r0 * a->loss.K : nullptr;
    c.mu_topk_logp = a->loss.mu_topk_logp ? a->loss.mu_topk_logp + r0 * a->loss.K : nullptr;
    c.loss_tok = a->loss.loss_tok ? a->loss.loss_tok + r0 : nullptr;
    c.divergence = a->loss.divergence + r0;
    c.mask = a->loss.mask + r0;
    c.diagnostics = a->loss.diagnostics ? a->loss.diagnostics + r0 * DPPO_NDIAG : nullptr;
    int np = 0;
    LossScratch sc;                   // per-workgroup partial sums only: the chunks of one call share the scratch
    sc.partial = partial + used;
    sc.max_parts = parts_per_chunk;
    const double* fin = nullptr;
    const dppo_status_t st = launch_loss(&c, grad, sc, &fin, &np, s);   // gradient in place
    if (st != DPPO_OK) return st;
    used += np;
    if (grad) {
      // gradient of the chunk's hidden states: g [rows, V] times W [V, d], the weight as it lies
      uint16_t* gh = static_cast<uint16_t*>(a->grad_hidden) + r0 * a->ld_grad_hidden;
      if (dppo::launch_gemm_nn(zbuf, V, static_cast<const uint16_t*>(a->weight), a->ld_weight, gh, a->ld_grad_hidden, static_cast<int>(rows),
                               static_cast<int>(d), static_cast<int>(V), s) != hipSuccess)
        return DPPO_ERR_LAUNCH;
    }
    if (want_gw) {
      // gradient of the lm_head weight: g_c^T h_c with g_c [rows, V] and h_c [rows, d] as they lie
      // (the token index is the row index of both); fp32, summed over the chunks (and onto the
      // caller's buffer if asked to accumulate)
      const int out = (r0 == 0 && !a->grad_weight_accumulate) ? 1 : 2;
      if (dppo::launch_gemm_tn(zbuf, V, h, a->ld_hidden, a->grad_weight, a->ld_grad_weight, static_cast<int>(V), static_cast<int>(d),
                               static_cast<int>(rows), out, s) != hipSuccess)
        return DPPO_ERR_LAUNCH;
    }
  }
  if (dppo::launch_finalize(partial, used, a->loss.loss_scale, a->loss.loss, s) != hipSuccess) return DPPO_ERR_LAUNCH;
  if (T > 0) g_last_path = "lmhead";
  return DPPO_OK;
}

}  // namespace

extern "C" {

size_t dppo_workspace_bytes(int64_t T, int64_t, int32_t) {
  return DPPO_WORKSPACE_BYTES + (T > 0 ? static_cast<size_t>(T) * sizeof(double) : 0);
}

dppo_status_t dppo_loss_fwd(const dppo_args_t* args, void* stream) { return run(args, stream, false); }

dppo_status_t dppo_loss_fwd_bwd(const dppo_args_t* args, void* stream) { return run(args, stream, true); }

dppo_status_t dppo_loss_fwd_bwd_static(const dppo_args_t* args, void* stream) { return run_static(args, stream); }

dppo_status_t dppo_static_init(void) {
  int cur = 0;
  if (hipGetDevice(&cur) != hipSuccess) return DPPO_ERR_LAUNCH;
  return static_scratch(cur) ? DPPO_OK : DPPO_ERR_WORKSPACE;
}

const char* dppo_status_str(dppo_status_t status) {
  switch (status) {
    case DPPO_OK: return "ok";
    case DPPO_ERR_NULL: return "a required pointer is NULL";
    case DPPO_ERR_SHAPE: return "bad shape: need T >= 0, 1 <= V <= ld (and <= mu_ld for DPPO_FULL_*), T and V below 2^31 (T <= DPPO_STATIC_MAX_T for dppo_loss_fwd_bwd_static)";
    case DPPO_ERR_ALIGN: return "misaligned pointer: bf16 buffers need 2-byte, workspace 8-byte, diagnostics 16-byte alignment";
    case DPPO_ERR_VARIANT: return "variant is not one of DPPO_BINARY_TV/KL, DPPO_TOPK_TV/KL, DPPO_FULL_TV/KL";
    case DPPO_ERR_K: return "bad K: need 0 <= K <= DPPO_KMAX and top-K pointers when K > 0";
    case DPPO_ERR_WORKSPACE: return "workspace missing or smaller than dppo_workspace_bytes() (dppo_loss_fwd_bwd_static: the static scratch array has no device address)";
    case DPPO_ERR_LAUNCH: return "HIP kernel launch failed (or the stream does not belong to the current device)";
    case DPPO_ERR_VALUE: return "bad value: NaN delta / loss_scale / ratio_cap, unknown mask_rule, or clip range outside 0 <= eps_low < 1, eps_high >= 0, relax_alpha outside [0, 1] or unknown relax_sides";
  }
  return "unknown status";
}

int dppo_version(void) { return DPPO_VERSION; }

size_t dppo_args_size(void) { return sizeof(dppo_args_t); }

const char* dppo_last_path(void) { return g_last_path; }

size_t dppo_lmhead_workspace_bytes(int64_t T, int64_t V, int64_t chunk_rows) {
  return lmhead_workspace(T, V, chunk_rows);
}

dppo_status_t dppo_lmhead_loss_fwd(const dppo_lmhead_args_t* args, void* stream) { return run_lmhead(args, stream, false); }

dppo_status_t dppo_lmhead_loss_fwd_bwd(const dppo_lmhead_args_t* args, void* stream) { return run_lmhead(args, stream, true); }

size_t dppo_lmhead_args_size(void) { return sizeof(dppo_lmhead_args_t); }

size_t dppo_lmhead_fwd_workspace_bytes(int64_t T, int64_t V, int32_t K, int64_t chunk_rows) {
  return lmhead_fwd_workspace(T, V, K < 0 ? 0 : K, chunk_rows);
}

dppo_status_t dppo_gemm_nt(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                           int64_t M, int64_t N, int64_t K, void* stream) {
  if (M < 0 || N < 0 || K < 64 || K % 64 != 0 || M >= (int64_t(1) << 31) || N >= (int64_t(1) << 31) || K >= (int64_t(1) << 31)) return DPPO_ERR_SHAPE;
  if (lda < K || ldb < K || ldc < N || lda % 8 != 0 || ldb % 8 != 0 || lda >= (int64_t(1) << 22) || ldb >= (int64_t(1) << 22)) return DPPO_ERR_SHAPE;
  if (M == 0 || N == 0) return DPPO_OK;
  if (!A || !B || !C) return DPPO_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 15u) return DPPO_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(C) & 1u) return DPPO_ERR_ALIGN;
  const hipError_t e = dppo::launch_gemm_nt(static_cast<const uint16_t*>(A), lda, static_cast<const uint16_t*>(B), ldb,
                                            C, ldc, static_cast<int>(M), static_cast<int>(N),
                                            static_cast<int>(K), 0, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DPPO_OK : DPPO_ERR_LAUNCH;
}

dppo_status_t dppo_gemm_nt_f32(const void* A, int64_t lda, const void* B, int64_t ldb, float* C, int64_t ldc,
                               int64_t M, int64_t N, int64_t K, int accumulate, void* stream) {
  if (M < 0 || N < 0 || K < 64 || K % 64 != 0 || M >= (int64_t(1) << 31) || N >= (int64_t(1) << 31) || K >= (int64_t(1) << 31)) return DPPO_ERR_SHAPE;
  if (lda < K || ldb < K || ldc < N || lda % 8 != 0 || ldb % 8 != 0 || ldc % 4 != 0 || lda >= (int64_t(1) << 22) || ldb >= (int64_t(1) << 22)) return DPPO_ERR_SHAPE;
  if (M == 0 || N == 0) return DPPO_OK;
  if (!A || !B || !C) return DPPO_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B) | reinterpret_cast<uintptr_t>(C)) & 15u) return DPPO_ERR_ALIGN;
  const hipError_t e = dppo::launch_gemm_nt(static_cast<const uint16_t*>(A), lda, static_cast<const uint16_t*>(B), ldb,
                                            C, ldc, static_cast<int>(M), static_cast<int>(N), static_cast<int>(K),
                                            accumulate ? 2 : 1, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DPPO_OK : DPPO_ERR_LAUNCH;
}

dppo_status_t dppo_gemm_nn(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                           int64_t M, int64_t N, int64_t K, void* stream) {
  if (M < 0 || N < 0 || K < 64 || K % 64 != 0 || M >= (int64_t(1) << 31) || N >= (int64_t(1) << 31) || K >= (int64_t(1) << 31)) return DPPO_ERR_SHAPE;
  if (lda < K || ldb < N || ldc < N || lda % 8 != 0 || ldb % 8 != 0 || lda >= (int64_t(1) << 22) || ldb >= (int64_t(1) << 22)) return DPPO_ERR_SHAPE;
  if (M == 0 || N == 0) return DPPO_OK;
  if (!A || !B || !C) return DPPO_ERR_NULL;
  if (((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 15u) || (reinterpret_cast<uintptr_t>(C) & 1u)) return DPPO_ERR_ALIGN;
  const hipError_t e = dppo::launch_gemm_nn(static_cast<const uint16_t*>(A), lda, static_cast<const uint16_t*>(B), ldb,
                                            C, ldc, static_cast<int>(M), static_cast<int>(N), static_cast<int>(K),
                                            static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DPPO_OK : DPPO_ERR_LAUNCH;
}

dppo_status_t dppo_gemm_tn_f32(const void* A, int64_t lda, const void* B, int64_t ldb, float* C, int64_t ldc,
                               int64_t M, int64_t N, int64_t K, int accumulate, void* stream) {
  if (M < 0 || N < 0 || K < 1 || M >= (int64_t(1) << 31) || N >= (int64_t(1) << 31) || K >= (int64_t(1) << 31)) return DPPO_ERR_SHAPE;
  if (lda < M || ldb < N || ldc < N || lda % 8 != 0 || ldb % 8 != 0 || ldc % 4 != 0 || lda >= (int64_t(1) << 22) || ldb >= (int64_t(1) << 22)) return DPPO_ERR_SHAPE;
  if (M == 0 || N == 0) return DPPO_OK;
  if (!A || !B || !C) return DPPO_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B) | reinterpret_cast<uintptr_t>(C)) & 15u) return DPPO_ERR_ALIGN;
  const hipError_t e = dppo::launch_gemm_tn(static_cast<const uint16_t*>(A), lda, static_cast<const uint16_t*>(B), ldb,
                                            C, ldc, static_cast<int>(M), static_cast<int>(N), static_cast<int>(K),
                                            accumulate ? 2 : 1, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? DPPO_OK : DPPO_ERR_LAUNCH;
}

}  // extern "C"
