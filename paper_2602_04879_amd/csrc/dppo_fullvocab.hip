// Trust region on the EXACT full-vocabulary divergence (App. B): total variation
// 1/2 sum_j |mu_j - pi_j| or KL(mu || pi) = sum_j mu_j ln(mu_j / pi_j) between the rollout policy's
// and the trainer's next-token distributions, both given as rows of bf16 logits.  These are the
// quantities the Binary and Top-K forms of Sec. 4.4 lower-bound.
//
// One workgroup per row, any V, any pitch, any alignment:
//   pass 1  streams both rows once: online sum of exponentials of the trainer row z (sampled
//           token left out, as in the other kernels), of the rollout row y, and the cross term
//           sum_j 2^(y_j..) (y_j - z_j).  With both normalisers known this already gives
//           KL = E_mu[y - z] - lse(y) + lse(z).
//   pass 2  (TV only) re-reads both rows and sums min(pi_j, mu_j): TV = 1 - that sum; with the
//           backward it also writes the gradient row, as if the divergence did not mask it.
//   epilogue on one wave: mask, loss term, gradient coefficient.
//   pass 3  (backward, KL form) re-reads z and writes the bf16 gradient row; in the TV form
//           only the rows the divergence masked are zero-filled.
// The re-reads come right after the first read of the same row and are normally served by the
// L2 / Infinity Cache.
#include "dppo_common.hpp"
#include "dppo_launch.hpp"

namespace dppo {
namespace {

template <int THREADS, bool TV, bool GRAD>
__global__ __launch_bounds__(THREADS) void dppo_fullvocab_kernel(const KParams p) {
  constexpr int NW = THREADS / kWave;
  __shared__ float sh_bz[NW], sh_by[NW];
  __shared__ double sh_sz[NW], sh_tz[NW], sh_sy[NW], sh_uy[NW], sh_acc[NW];
  __shared__ RowCoef sh_rc;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wid = tid / kWave;
  const EpiParams ep = epi_params(p);
  double loss_acc = 0.0;   // meaningful in wave 0 only

  for (int row = blockIdx.x; row < p.T; row += gridDim.x) {
    const int a = p.sampled[row];
    const uint16_t* zrow = p.logits + static_cast<int64_t>(row) * p.ld;
    const uint16_t* yrow = p.mu_logits + static_cast<int64_t>(row) * p.mu_ld;
    uint16_t* grow = GRAD ? p.grad + static_cast<int64_t>(row) * p.ld : nullptr;
    // [head | 16-byte vectors | tail], when the rows share their 16-byte misalignment;
    // otherwise everything is "head" (element-wise).
    const uintptr_t za = reinterpret_cast<uintptr_t>(zrow);
    bool vec = ((za ^ reinterpret_cast<uintptr_t>(yrow)) & 15u) == 0;
    if (GRAD) vec = vec && ((za ^ reinterpret_cast<uintptr_t>(grow)) & 15u) == 0;
    int head = p.V, nvec = 0;
    if (vec) {
      head = min((8 - static_cast<int>((za & 15u) >> 1)) & 7, p.V);
      nvec = (p.V - head) >> 3;
    }
    const int tail0 = head + (nvec << 3);
    const int nscalar = head + (p.V - tail0);
    const bool live = (a >= 0 && a < p.V);
    const int av = (live && a >= head && a < tail0) ? ((a - head) >> 3) : -1;   // vector holding a_t
    const int sub = (a - head) & 7;

    RowCoef rc;
    rc.coef = 0.f; rc.kexp = 0.f; rc.g_a = 0.f;
    u32x4* gv = reinterpret_cast<u32x4*>(grow + head);
    // gradient of the eight entries of vector v of the row, given the row's coefficient
    auto grad_vec = [&](const u32x4& q, int v, const RowCoef& c) {
      float z[8];
      unpack8(q, z);
#pragma unroll
      for (int i = 0; i < 8; ++i) z[i] = fast_exp2(fmaf(z[i], kLog2e, c.kexp));
      const uint32_t sgn = (c.coef < 0.f) ? 0x80008000u : 0u;
      uint32_t w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(z[2 * i], z[2 * i + 1]) ^ sgn;
      if (v == av) {   // the vector holding a_t: overwrite that one entry
        const uint32_t ga = float_to_bf16_bits(c.g_a);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if ((sub >> 1) == i) w[i] = (sub & 1) ? ((w[i] & 0x0000ffffu) | (ga << 16)) : ((w[i] & 0xffff0000u) | ga);
      }
      const u32x4 o = {w[0], w[1], w[2], w[3]};
      __builtin_nontemporal_store(o, gv + v);
    };
    auto grad_scalar = [&](int j, const RowCoef& c) {
      float g = fast_exp2(fmaf(bf16_bits_to_float(zrow[j]), kLog2e, c.kexp));
      g = (c.coef < 0.f) ? -g : g;
      if (j == a) g = c.g_a;
      grow[j] = float_to_bf16_bits(g);
    };
    auto zero_row = [&]() {
      const u32x4 zero = {0u, 0u, 0u, 0u};
      for (int v = tid; v < nvec; v += THREADS) __builtin_nontemporal_store(zero, gv + v);
      for (int e = tid; e < nscalar; e += THREADS) grow[(e < head) ? e : tail0 + (e - head)] = 0;
    };
    bool grad_written = false;      // the TV form writes the gradient during its second pass ...
    RowCoef rc1;                    // ... with this coefficient: the row's if the divergence does not mask it
    rc1.coef = 0.f; rc1.kexp = 0.f; rc1.g_a = 0.f;
    if (live) {
      const float z_a = bf16_bits_to_float(zrow[a]);
      // ---- pass 1 --------------------------------------------------------------------------
      OnlineStat st;       // z, without a_t
      CrossStat cs;        // y, and y - z
      st.cover(fmaxf(kNegBig, z_a));   // the offset must cover z[a_t]
      const u32x4* zv = reinterpret_cast<const u32x4*>(zrow + head);
      const u32x4* yv = reinterpret_cast<const u32x4*>(yrow + head);
      auto both = [&](const u32x4& zq, const u32x4& yq, int v) {
        float z[8], y[8];
        unpack8(zq, z);
        unpack8(yq, y);
        cs.add8(y, z);
        if (v == av) {
#pragma unroll
          for (int i = 0; i < 8; ++i) z[i] = (i == sub) ? -INFINITY : z[i];
        }
        st.add8(z);
      };
      int v = tid;
      for (; v + THREADS < nvec; v += 2 * THREADS) {     // two vectors of each row in flight
        // the KL form reads the rollout row only here: marked non-temporal (1-2 % faster)
        const u32x4 z0 = zv[v], y0 = TV ? yv[v] : __builtin_nontemporal_load(yv + v);
        const u32x4 z1 = zv[v + THREADS], y1 = TV ? yv[v + THREADS] : __builtin_nontemporal_load(yv + v + THREADS);
        both(z0, y0, v);
        both(z1, y1, v + THREADS);
      }
      if (v < nvec) both(zv[v], yv[v], v);
      for (int e = tid; e < nscalar; e += THREADS) {
        const int j = (e < head) ? e : tail0 + (e - head);
        const float zj = bf16_bits_to_float(zrow[j]);
        cs.add1(bf16_bits_to_float(yrow[j]), zj);
        if (j != a) st.add1(zj);
      }
      // workgroup-wide offsets = the smallest ones; rescaling to them is exact
      const float wbz = -wave_max(-st.b), wby = -wave_max(-cs.b);
      if (lane == 0) { sh_bz[wid] = wbz; sh_by[wid] = wby; }
      __syncthreads();
      float bz = sh_bz[0], by = sh_by[0];
#pragma unroll
      for (int w = 1; w < NW; ++w) { bz = fminf(bz, sh_bz[w]); by = fminf(by, sh_by[w]); }
      {
        const double dd = static_cast<double>(bz - st.b), sc = static_cast<double>(fast_exp2(bz - st.b));
        const double scy = static_cast<double>(fast_exp2(by - cs.b));
        const double sd = wave_sum(st.s * sc);
        const double td = wave_sum(sc * (static_cast<double>(st.t) + dd * st.s));
        const double sy = wave_sum(cs.s * scy);
        const double uy = wave_sum(static_cast<double>(cs.u) * scy);
        if (lane == 0) { sh_sz[wid] = sd; sh_tz[wid] = td; sh_sy[wid] = sy; sh_uy[wid] = uy; }
      }
      __syncthreads();
      // Every thread forms the two normalisers (pass 2 needs them everywhere).
      double S_rest = 0.0, T_rest = 0.0, Sy = 0.0, Uy = 0.0;
#pragma unroll
      for (int w = 0; w < NW; ++w) { S_rest += sh_sz[w]; T_rest += sh_tz[w]; Sy += sh_sy[w]; Uy += sh_uy[w]; }
      const double xa = static_cast<double>(z_a) * static_cast<double>(kLog2e) + static_cast<double>(bz);
      const double S = S_rest + exp2_d(xa);
      double D;
      if (TV) {
        // ---- pass 2: TV = 1/2 sum |pi_j - mu_j| = 1 - sum_j min(pi_j, mu_j) -------------------
        // One exponential per entry: the minimum is taken on the base-2 log-probabilities
        // z_j*log2e + b - log2 S.  The integer part of log2 S goes into the (integer) offset, which
        // stays exact, and only the fraction in [0, 1) is subtracted in fp32, so a probability
        // keeps a relative error of about 1e-7 however large the offset is.
        const double l2z = log2_d(S), l2y = log2_d(Sy);
        const double nz = floor(l2z), ny = floor(l2y);
        const float bz2 = bz - static_cast<float>(nz), by2 = by - static_cast<float>(ny);
        const float fz = static_cast<float>(l2z - nz), fy = static_cast<float>(l2y - ny);
        // Backward: the row's gradient is written in this same pass, with the coefficient the row
        // has if the divergence does not mask it (everything else that decides it is known); the
        // few rows the exact divergence then masks are zero-filled afterwards.  That saves the
        // third read of z for all the others.
        if (GRAD) {
          if (wid == 0) {
            RowScalars rs;
            rs.a = a; rs.za = z_a; rs.lmu = p.mu_logp[row]; rs.adv = p.adv[row]; rs.lanc = anchor_or(p, row, rs.lmu);
            TopkLane tk;
            tk.id = -1; tk.lp = 0.f; tk.z = 0.f;
            const RowResult res = row_epilogue_call(ep, row, rs, tk, zrow, bz, S_rest, T_rest, lane, 0.0);   // D = 0: not masked by it
            if (lane == 0) sh_rc = res.rc;
          }
          __syncthreads();
          rc1 = sh_rc;
        }
        double acc0 = 0.0, acc1 = 0.0;
        auto min8 = [&](const u32x4& zq, const u32x4& yq, double& acc) {
          float z[8], y[8], m[8];
          unpack8(zq, z);
          unpack8(yq, y);
#pragma unroll
          for (int i = 0; i < 8; ++i) m[i] = fast_exp2(fminf(fmaf(z[i], kLog2e, bz2) - fz, fmaf(y[i], kLog2e, by2) - fy));
          acc += static_cast<double>(sum8(m));      // eight entries among themselves, then into float64
        };
        const bool write_grad = GRAD && rc1.coef != 0.f;
        int v2 = tid;
        for (; v2 + THREADS < nvec; v2 += 2 * THREADS) {
          // last use of both rows: non-temporal loads (7 % faster on the headline shape)
          const u32x4 z0 = __builtin_nontemporal_load(zv + v2), y0 = __builtin_nontemporal_load(yv + v2);
          const u32x4 z1 = __builtin_nontemporal_load(zv + v2 + THREADS), y1 = __builtin_nontemporal_load(yv + v2 + THREADS);
          min8(z0, y0, acc0);
          min8(z1, y1, acc1);
          if (write_grad) {
            grad_vec(z0, v2, rc1);
            grad_vec(z1, v2 + THREADS, rc1);
          }
        }
        if (v2 < nvec) {
          const u32x4 z0 = zv[v2];
          min8(z0, yv[v2], acc0);
          if (write_grad) grad_vec(z0, v2, rc1);
        }
        for (int e = tid; e < nscalar; e += THREADS) {
          const int j = (e < head) ? e : tail0 + (e - head);
          acc1 += static_cast<double>(fast_exp2(fminf(fmaf(bf16_bits_to_float(zrow[j]), kLog2e, bz2) - fz, fmaf(bf16_bits_to_float(yrow[j]), kLog2e, by2) - fy)));
          if (write_grad) grad_scalar(j, rc1);
        }
        if (GRAD) {
          if (!write_grad) zero_row();
          grad_written = true;
        }
        const double wa = wave_sum(acc0 + acc1);
        if (lane == 0) sh_acc[wid] = wa;
        __syncthreads();
        double tot = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w) tot += sh_acc[w];
        D = fmax(1.0 - tot, 0.0);
        if (tot != tot) D = tot;                  // NaN logits propagate
      } else {
        // KL = E_mu[y - z] - lse(y) + lse(z), the log-sum-exps in base 2 against their offsets
        const double lse2_z = log2_d(S) - static_cast<double>(bz), lse2_y = log2_d(Sy) - static_cast<double>(by);
        D = Uy / Sy + kLn2 * (lse2_z - lse2_y);
        D = (D > 0.0 || D != D) ? D : 0.0;       // rounding can leave -1e-8 for identical rows
      }
      // ---- epilogue on wave 0 ----------------------------------------------------------------
      if (wid == 0) {
        RowScalars rs;
        rs.a = a;
        rs.za = z_a;
        rs.lmu = p.mu_logp[row];
        rs.lanc = anchor_or(p, row, rs.lmu);
        rs.adv = p.adv[row];
        TopkLane tk;
        tk.id = -1; tk.lp = 0.f; tk.z = 0.f;
        const RowResult res = row_epilogue_call(ep, row, rs, tk, zrow, bz, S_rest, T_rest, lane, D);
        rc = res.rc;
        loss_acc += res.loss_term;
        if (GRAD && lane == 0) sh_rc = rc;
      }
      if (GRAD) {
        __syncthreads();
        rc = sh_rc;
        // TV form: the row was written as if unmasked; the exact divergence has now masked it
        if (TV && grad_written && rc1.coef != 0.f && rc.coef == 0.f) zero_row();
      }
    } else if (tid == 0) {
      p.divergence[row] = 0.f;
      p.mask[row] = 0;
      if (p.loss_tok) p.loss_tok[row] = 0.f;
      if (p.diag) {
        for (int k = 0; k < 8; ++k) p.diag[static_cast<int64_t>(row) * 8 + k] = 0.f;
      }
    }

    if (GRAD && !grad_written) {
      // ---- pass 3: gradient (KL form, and rows that were never live) ---------------------------
      if (rc.coef == 0.f) {
        zero_row();
      } else {
        const u32x4* zv = reinterpret_cast<const u32x4*>(zrow + head);
        int v = tid;
        for (; v + 3 * THREADS < nvec; v += 4 * THREADS) {     // four loads in flight, then four stores
          const u32x4 q0 = __builtin_nontemporal_load(zv + v), q1 = __builtin_nontemporal_load(zv + v + THREADS);   // last use of the row
          const u32x4 q2 = __builtin_nontemporal_load(zv + v + 2 * THREADS), q3 = __builtin_nontemporal_load(zv + v + 3 * THREADS);
          grad_vec(q0, v, rc);
          grad_vec(q1, v + THREADS, rc);
          grad_vec(q2, v + 2 * THREADS, rc);
          grad_vec(q3, v + 3 * THREADS, rc);
        }
        for (; v < nvec; v += THREADS) grad_vec(zv[v], v, rc);
        for (int e = tid; e < nscalar; e += THREADS) grad_scalar((e < head) ? e : tail0 + (e - head), rc);
      }
    }
    // The shared statistics are rewritten by the next row: make sure everyone has read them.
    __syncthreads();
  }
  if (tid == 0) p.partial[blockIdx.x] = loss_acc;
}

template <int THREADS>
hipError_t launch_fullvocab_t(const KParams& p, bool tv, bool grad, int grid, hipStream_t s) {
  const dim3 g(grid), b(THREADS);
  if (tv) {
    if (grad) hipLaunchKernelGGL((dppo_fullvocab_kernel<THREADS, true, true>), g, b, 0, s, p);
    else      hipLaunchKernelGGL((dppo_fullvocab_kernel<THREADS, true, false>), g, b, 0, s, p);
  } else {
    if (grad) hipLaunchKernelGGL((dppo_fullvocab_kernel<THREADS, false, true>), g, b, 0, s, p);
    else      hipLaunchKernelGGL((dppo_fullvocab_kernel<THREADS, false, false>), g, b, 0, s, p);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fullvocab(const KParams& p, bool tv, bool grad, int threads, int grid, hipStream_t s) {
  switch (threads) {
    case 256: return launch_fullvocab_t<256>(p, tv, grad, grid, s);
    case 512: return launch_fullvocab_t<512>(p, tv, grad, grid, s);
    default:  return launch_fullvocab_t<1024>(p, tv, grad, grid, s);
  }
}

}  // namespace dppo
