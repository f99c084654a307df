// General two-pass kernel: one workgroup per row, any V, any row pitch, any alignment.
//
// Pass 1 streams the row once from HBM with 16-byte loads (per-thread online max / sum of
// exponentials in fp32), the workgroup combines the statistics, one wave evaluates the
// per-token epilogue, and pass 2 re-reads the row (normally still in L2 / Infinity Cache),
// from its end backwards (what pass 1 read last is what the L2 still holds), and writes the bf16
// gradient with non-temporal 16-byte stores.  Rows whose gradient
// coefficient is zero (masked, zero advantage, ignored) are zero-filled without the re-read.
#include "dppo_common.hpp"
#include "dppo_launch.hpp"

namespace dppo {
namespace {

template <int THREADS, bool VEC, bool GRAD>
__global__ __launch_bounds__(THREADS) void dppo_streaming_kernel(const KParams p) {
  constexpr int NW = THREADS / kWave;
  __shared__ float sh_max[NW];
  __shared__ double sh_sum[NW], sh_tsum[NW];
  __shared__ RowCoef sh_rc;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wid = tid / kWave;
  const EpiParams ep = epi_params(p);
  double loss_acc = 0.0;   // meaningful in wave 0 only

  for (int row = blockIdx.x; row < p.T; row += gridDim.x) {
    const int a = p.sampled[row];
    const uint16_t* zrow = p.logits + static_cast<int64_t>(row) * p.ld;
    uint16_t* grow = GRAD ? p.grad + static_cast<int64_t>(row) * p.ld : nullptr;
    // Split the row into [head | 16-byte vectors | tail]; VEC=false makes everything "head".
    int head = p.V, nvec = 0;
    if (VEC) {
      const int mis = static_cast<int>((reinterpret_cast<uintptr_t>(zrow) & 15u) >> 1);
      head = min((8 - mis) & 7, p.V);
      nvec = (p.V - head) >> 3;
    }
    const int tail0 = head + (nvec << 3);       // first tail element
    const int nscalar = head + (p.V - tail0);   // head + tail element count
    const bool live = (a >= 0 && a < p.V);

    RowCoef rc;
    rc.coef = 0.f; rc.kexp = 0.f; rc.g_a = 0.f;
    const int av = (live && a >= head && a < tail0) ? ((a - head) >> 3) : -1;   // vector holding a_t
    if (live) {
      // ---- pass 1: online max / sum-exp over j != a_t -----------------------------------
      OnlineStat st;
      st.cover(fmaxf(kNegBig, bf16_bits_to_float(zrow[a])));   // the offset must cover z[a_t]
      const u32x4* zv = reinterpret_cast<const u32x4*>(zrow + head);
      auto add_vec = [&](const u32x4& q, int v) {
        float z[8];
        unpack8(q, z);
        if (v == av) {
          const int sub = (a - head) & 7;
#pragma unroll
          for (int i = 0; i < 8; ++i) z[i] = (i == sub) ? -INFINITY : z[i];
        }
        st.add8(z);
      };
      int v = tid;
      for (; v + 3 * THREADS < nvec; v += 4 * THREADS) {     // four 16-byte loads in flight per thread
        const u32x4 q0 = zv[v], q1 = zv[v + THREADS], q2 = zv[v + 2 * THREADS], q3 = zv[v + 3 * THREADS];
        add_vec(q0, v);
        add_vec(q1, v + THREADS);
        add_vec(q2, v + 2 * THREADS);
        add_vec(q3, v + 3 * THREADS);
      }
      for (; v < nvec; v += THREADS) add_vec(zv[v], v);
      for (int e = tid; e < nscalar; e += THREADS) {
        const int j = (e < head) ? e : tail0 + (e - head);
        if (j != a) st.add1(bf16_bits_to_float(zrow[j]));
      }
      // workgroup-wide offset = the smallest one; rescaling to it is exact
      float wb = -wave_max(-st.b);
      if (lane == 0) sh_max[wid] = wb;
      __syncthreads();
      float b = sh_max[0];
#pragma unroll
      for (int w = 1; w < NW; ++w) b = fminf(b, sh_max[w]);
      const double dd = static_cast<double>(b - st.b), sc = static_cast<double>(fast_exp2(b - st.b));
      const double sd = wave_sum(st.s * sc);
      const double td = wave_sum(sc * (static_cast<double>(st.t) + dd * st.s));
      if (lane == 0) { sh_sum[wid] = sd; sh_tsum[wid] = td; }
      __syncthreads();
      // ---- epilogue on wave 0 -----------------------------------------------------------
      if (wid == 0) {
        double S_rest = 0.0, T_rest = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w) { S_rest += sh_sum[w]; T_rest += sh_tsum[w]; }
        RowScalars rs;
        rs.a = a;
        rs.za = bf16_bits_to_float(zrow[a]);
        rs.lmu = p.mu_logp[row];
        rs.lanc = anchor_or(p, row, rs.lmu);
        rs.adv = p.adv[row];
        const TopkLane tk = load_topk_lane(p, row, a, zrow, lane);
        const RowResult res = row_epilogue_call(ep, row, rs, tk, zrow, b, S_rest, T_rest, lane);
        rc = res.rc;
        loss_acc += res.loss_term;
        if (GRAD && lane == 0) sh_rc = rc;
      }
      if (GRAD) {
        __syncthreads();
        rc = sh_rc;
      }
    } else if (tid == 0) {
      p.divergence[row] = 0.f;
      p.mask[row] = 0;
      if (p.loss_tok) p.loss_tok[row] = 0.f;
      if (p.diag) {
        for (int k = 0; k < 8; ++k) p.diag[static_cast<int64_t>(row) * 8 + k] = 0.f;
      }
    }

    if (GRAD) {
      // ---- pass 2: gradient --------------------------------------------------------------
      u32x4* gv = reinterpret_cast<u32x4*>(grow + head);
      if (rc.coef == 0.f) {
        const u32x4 zero = {0u, 0u, 0u, 0u};
        for (int v = tid; v < nvec; v += THREADS) __builtin_nontemporal_store(zero, gv + v);
        for (int e = tid; e < nscalar; e += THREADS) grow[(e < head) ? e : tail0 + (e - head)] = 0;
      } else {
        const uint32_t sgn = (rc.coef < 0.f) ? 0x80008000u : 0u;
        const float kexp = rc.kexp;
        const u32x4* zv = reinterpret_cast<const u32x4*>(zrow + head);
        auto grad_vec = [&](const u32x4& q, int v) {
          float z[8];
          unpack8(q, z);
#pragma unroll
          for (int i = 0; i < 8; ++i) z[i] = fast_exp2(fmaf(z[i], kLog2e, kexp));
          uint32_t w[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(z[2 * i], z[2 * i + 1]) ^ sgn;
          if (v == av) {   // the vector holding a_t: overwrite that one entry
            const int sub = (a - head) & 7;
            const uint32_t ga = float_to_bf16_bits(rc.g_a);
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if ((sub >> 1) == i) w[i] = (sub & 1) ? ((w[i] & 0x0000ffffu) | (ga << 16)) : ((w[i] & 0xffff0000u) | ga);
          }
          const u32x4 o = {w[0], w[1], w[2], w[3]};
          __builtin_nontemporal_store(o, gv + v);
        };
        // From the END of the row backwards: what pass 1 read last is what the L2 still holds.
        // Four loads in flight, then four stores; the row is not needed again: non-temporal loads (2 % faster).
        const int nfull = nvec / (4 * THREADS);                   // blocks of 4 * THREADS vectors
        for (int v = nfull * 4 * THREADS + tid; v < nvec; v += THREADS) grad_vec(zv[v], v);   // the ragged end first
        for (int blk = nfull - 1; blk >= 0; --blk) {
          const int v = blk * 4 * THREADS + tid;
          const u32x4 q3 = __builtin_nontemporal_load(zv + v + 3 * THREADS), q2 = __builtin_nontemporal_load(zv + v + 2 * THREADS);
          const u32x4 q1 = __builtin_nontemporal_load(zv + v + THREADS), q0 = __builtin_nontemporal_load(zv + v);
          grad_vec(q3, v + 3 * THREADS);
          grad_vec(q2, v + 2 * THREADS);
          grad_vec(q1, v + THREADS);
          grad_vec(q0, v);
        }
        for (int e = tid; e < nscalar; e += THREADS) {
          const int j = (e < head) ? e : tail0 + (e - head);
          float g = fast_exp2(fmaf(bf16_bits_to_float(zrow[j]), kLog2e, kexp));
          g = (rc.coef < 0.f) ? -g : g;
          if (j == a) g = rc.g_a;
          grow[j] = float_to_bf16_bits(g);
        }
      }
    }
    // The shared statistics are rewritten by the next row: make sure everyone has read them.
    __syncthreads();
  }
  if (tid == 0) p.partial[blockIdx.x] = loss_acc;
}

}  // namespace

template <int THREADS>
static hipError_t launch_streaming_t(const KParams& p, bool vec, bool grad, int grid, hipStream_t s) {
  if (vec) {
    if (grad) hipLaunchKernelGGL((dppo_streaming_kernel<THREADS, true, true>), dim3(grid), dim3(THREADS), 0, s, p);
    else      hipLaunchKernelGGL((dppo_streaming_kernel<THREADS, true, false>), dim3(grid), dim3(THREADS), 0, s, p);
  } else {
    if (grad) hipLaunchKernelGGL((dppo_streaming_kernel<THREADS, false, true>), dim3(grid), dim3(THREADS), 0, s, p);
    else      hipLaunchKernelGGL((dppo_streaming_kernel<THREADS, false, false>), dim3(grid), dim3(THREADS), 0, s, p);
  }
  return hipGetLastError();
}

hipError_t launch_streaming(const KParams& p, bool vec, bool grad, int threads, int grid, hipStream_t s) {
  switch (threads) {
    case 256: return launch_streaming_t<256>(p, vec, grad, grid, s);
    case 512: return launch_streaming_t<512>(p, vec, grad, grid, s);
    default:  return launch_streaming_t<1024>(p, vec, grad, grid, s);
  }
}

// Sum the n terms (per-workgroup partial sums, or one term per row) in a fixed order and store
// loss = loss_scale * sum.  One workgroup of 1024 threads: thread i takes terms i, i + 1024, ...
// into eight accumulators (so that eight loads are in flight; term k goes to accumulator
// (k / 1024) % 8), which are then added in a fixed order, and a tree over the threads follows.
__global__ __launch_bounds__(1024) void dppo_finalize_kernel(const double* partial, int n, float loss_scale, float* loss) {
  __shared__ double sh[1024];
  double acc[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
  int i = threadIdx.x;
  for (; i + 7 * 1024 < n; i += 8 * 1024) {
    double v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = partial[i + u * 1024];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] += v[u];
  }
#pragma unroll
  for (int u = 0; u < 8; ++u)
    if (i + u * 1024 < n) acc[u] += partial[i + u * 1024];
  sh[threadIdx.x] = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if (static_cast<int>(threadIdx.x) < o) sh[threadIdx.x] += sh[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = static_cast<float>(static_cast<double>(loss_scale) * sh[0]);
}

__global__ __launch_bounds__(64) void dppo_clear_counters_kernel(int32_t* counters) {
  if (threadIdx.x < 8) counters[threadIdx.x] = 0;
}

hipError_t launch_clear_counters(int32_t* counters, hipStream_t s) {
  hipLaunchKernelGGL(dppo_clear_counters_kernel, dim3(1), dim3(64), 0, s, counters);
  return hipGetLastError();
}

hipError_t launch_finalize(const double* partial, int n, float loss_scale, float* loss, hipStream_t s) {
  hipLaunchKernelGGL(dppo_finalize_kernel, dim3(1), dim3(1024), 0, s, partial, n, loss_scale, loss);
  return hipGetLastError();
}

}  // namespace dppo
