// Launchers of the two big kernel families.  Their template instances are compiled in separate
// translation units (ppd_inst.hip with -DPPD_INST=n) so that the library builds in parallel.
#pragma once
#include "ppd_kernels.h"

namespace ppd {

template <typename WT, bool PAIRED, int WR>
hipError_t launch_gemm_t(hipStream_t stream, const GemmArgs& a, int MA, int MB, dim3 grid, size_t lds);

template <int HD>
hipError_t launch_attn_t(hipStream_t stream, const AttnArgs& a, int mmax, dim3 grid, bool causal);

// Workgroups per group for a GEMM with `nsets` row sets (gemm_kernel): each workgroup has four waves and
// every wave takes ceil(nsets / waves) sets, so pick the count in [gmax/2, gmax] that wastes the fewest
// wave slots (ties: the larger grid).
inline int pick_grid(int nsets, int gmax) {
  int need = (nsets + GEMM_WAVES - 1) / GEMM_WAVES;
  if (need <= gmax) return need < 1 ? 1 : need;
  int best = gmax; double best_eff = 0.0;
  for (int g = gmax; g >= gmax / 2 && g >= 1; --g) {
    int nw = g * GEMM_WAVES, nit = (nsets + nw - 1) / nw;
    double eff = (double)nsets / ((double)nit * nw);
    if (eff > best_eff + 1e-9) { best_eff = eff; best = g; }
  }
  return best;
}

// LM-head launch of gemm_kernel (one row, four weight rows per wave): as many workgroups as a plain GEMM,
// more if a workgroup would otherwise produce over HEAD_MAX_ROWS logits
inline int head_grid_valu(int vocab, int gmax) {
  const int nsets = (vocab + 3) / 4;
  int g = pick_grid(nsets, gmax);
  const int sets_per_wg_cap = HEAD_MAX_ROWS / 4;               // per workgroup, all four waves together
  while (((nsets + g * GEMM_WAVES - 1) / (g * GEMM_WAVES)) * GEMM_WAVES > sets_per_wg_cap) ++g;
  return g;
}

// hipError_t of the last failing HIP call made outside any context (ppd_last_hip_error(NULL) reports it)
void set_global_hip_error(int e);

}  // namespace ppd
