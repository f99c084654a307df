// Hidden-state path, forward only: the rows' side of it.  The first product left, per row and
// 256-column tile of the vocabulary, the statistics of that tile's bf16-rounded logits and the
// logits at the row's sampled and top-K ids (GemmStats); here one wave per row combines the tiles
// and runs the per-row epilogue.  No logit was ever written to memory.
#include "dppo_common.hpp"
#include "dppo_launch.hpp"

namespace dppo {
namespace {

__global__ __launch_bounds__(256) void dppo_lmhead_rows_kernel(const KParams p, const GemmStats gs, double* __restrict__ row_loss) {
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wid = uniform_i(tid / kWave);
  const int row = static_cast<int>(blockIdx.x) * 4 + wid;
  if (row >= p.T) return;
  const int a = p.sampled[row];
  if (!(a >= 0 && a < p.V)) {        // ignored row
    if (lane == 0) {
      p.divergence[row] = 0.f;
      p.mask[row] = 0;
      if (p.loss_tok) p.loss_tok[row] = 0.f;
      if (p.diag) {
        for (int k = 0; k < 8; ++k) p.diag[static_cast<int64_t>(row) * 8 + k] = 0.f;
      }
      row_loss[row] = 0.0;
    }
    return;
  }
  // The tiles of the row, lane l those numbered l, l + 64, ...: every offset is an integer, so
  // bringing two sums to the smaller offset is exact.
  float b = 3.0e38f;
  double s = 0.0, t = 0.0;
  const gemm_f32x4* part = gs.part + static_cast<int64_t>(row) * gs.tiles_n;
  for (int j = lane; j < gs.tiles_n; j += kWave) {
    const gemm_f32x4 v = part[j];
    const float bn = fminf(b, v[0]);
    const float d0 = bn - b, d1 = bn - v[0];
    const double c0 = static_cast<double>(fast_exp2(d0)), c1 = static_cast<double>(fast_exp2(d1));
    t = c0 * (t + static_cast<double>(d0) * s) + c1 * (static_cast<double>(v[2]) + static_cast<double>(d1) * static_cast<double>(v[1]));
    s = c0 * s + c1 * static_cast<double>(v[1]);
    b = bn;
  }
  const float za = gs.gath[static_cast<int64_t>(row) * (p.K + 1)];
  // common offset: the smallest one, which must also cover z[a_t] (the epilogue adds its term)
  const float bb = fminf(-wave_max(-b), -ceilf(fmaxf(za, kNegBig) * kLog2e));
  const double dw = static_cast<double>(bb - b), cw = static_cast<double>(fast_exp2(bb - b));
  const double T_rest = wave_sum(cw * (t + dw * s));
  const double S_rest = wave_sum(cw * s);
  RowScalars rs;
  rs.a = a;
  rs.za = za;
  rs.lmu = p.mu_logp[row];
  rs.lanc = anchor_or(p, row, rs.lmu);
  rs.adv = p.adv[row];
  const TopkLane tk = load_topk_lane(p, row, a, nullptr, lane);
  const EpiParams ep = epi_params(p);
  const RowResult res = row_epilogue(ep, row, rs, tk, nullptr, bb, S_rest, T_rest, lane);
  if (lane == 0) row_loss[row] = res.loss_term;
}

}  // namespace

hipError_t launch_lmhead_rows(const KParams& p, const GemmStats& gs, double* row_loss, hipStream_t s) {
  if (p.T <= 0) return hipSuccess;
  hipLaunchKernelGGL(dppo_lmhead_rows_kernel, dim3((p.T + 3) / 4), dim3(256), 0, s, p, gs, row_loss);
  return hipGetLastError();
}

}  // namespace dppo
