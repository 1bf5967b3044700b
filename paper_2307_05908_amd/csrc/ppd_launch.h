// Launchers of the two big kernel families.  Their template instances are compiled in separate
// translation units (ppd_inst.hip with -DPPD_INST=n) so that the library builds in parallel.
#pragma once
#include "ppd_kernels.h"

namespace ppd {

template <typename WT, bool PAIRED, int WR>
hipError_t launch_gemm_t(hipStream_t stream, const GemmArgs& a, int MA, int MB, dim3 grid, size_t lds);

template <int HD>
hipError_t launch_attn_t(hipStream_t stream, const AttnArgs& a, int mmax, dim3 grid, bool causal);

}  // namespace ppd
