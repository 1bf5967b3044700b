// One slice of the kernel template instances, selected by -DPPD_INST=n (see build.py).
#include "ppd_launch.h"

namespace ppd {

#if PPD_INST < 4 || PPD_INST == 6
// MA rows in group 0; MB rows in group 1 (0: single-group launch).  Launch shapes in use:
// (1, 0) main token alone, (k, 0) the candidates alone, (1, k) both in one launch.
template <typename WT, bool PAIRED, int WR>
hipError_t launch_gemm_t(hipStream_t stream, const GemmArgs& a, int MA, int MB, dim3 grid, size_t lds) {
#define GO(ma, mb) hipLaunchKernelGGL((gemm_kernel<WT, ma, mb, PAIRED, WR>), grid, dim3(GEMM_THREADS), lds, stream, a)
  if (MB == 0) {
    switch (MA) {
      case 1: GO(1, 0); break; case 2: GO(2, 0); break; case 3: GO(3, 0); break; case 4: GO(4, 0); break;
      case 5: GO(5, 0); break; case 6: GO(6, 0); break; case 7: GO(7, 0); break; case 8: GO(8, 0); break;
      default: return hipErrorInvalidValue;
    }
  } else {
    if (MA != 1) return hipErrorInvalidValue;
    switch (MB) {
      case 1: GO(1, 1); break; case 2: GO(1, 2); break; case 3: GO(1, 3); break; case 4: GO(1, 4); break;
      case 5: GO(1, 5); break; case 6: GO(1, 6); break; case 7: GO(1, 7); break; case 8: GO(1, 8); break;
      default: return hipErrorInvalidValue;
    }
  }
#undef GO
  return hipGetLastError();
}


// (fp32 weights, and one instance for row-major bf16: inside a context bf16 models run every GEMM on the MFMA kernel)
#if PPD_INST == 0
template hipError_t launch_gemm_t<float, false, 4>(hipStream_t, const GemmArgs&, int, int, dim3, size_t);
#elif PPD_INST == 1
template hipError_t launch_gemm_t<float, true, 4>(hipStream_t, const GemmArgs&, int, int, dim3, size_t);
#elif PPD_INST == 2
template hipError_t launch_gemm_t<float, false, 2>(hipStream_t, const GemmArgs&, int, int, dim3, size_t);
#elif PPD_INST == 3
template hipError_t launch_gemm_t<float, true, 2>(hipStream_t, const GemmArgs&, int, int, dim3, size_t);
#elif PPD_INST == 6
// bf16 weights as the caller holds them (row-major, not repacked): the stand-alone early prediction
template hipError_t launch_gemm_t<bf16_t, false, 4>(hipStream_t, const GemmArgs&, int, int, dim3, size_t);
#endif
#else
// mmax: the largest row count of the launch's groups (sizes LDS); causal: the prompt-chunk instance
template <int HD>
hipError_t launch_attn_t(hipStream_t stream, const AttnArgs& a, int mmax, dim3 grid, bool causal) {
  if (mmax < 1 || mmax > 16) return hipErrorInvalidValue;
  const size_t lds = sizeof(float) * (size_t)attn_lds_floats<HD>(mmax);
  static_assert(sizeof(float) * attn_lds_floats<HD>(16) <= 64 * 1024, "16 rows fit the default dynamic LDS limit");
  if (lds > 64 * 1024) return hipErrorInvalidValue;
  if (causal) attn_kernel<HD, true><<<grid, dim3(ATT_THREADS), lds, stream>>>(a);
  else attn_kernel<HD, false><<<grid, dim3(ATT_THREADS), lds, stream>>>(a);
  return hipGetLastError();
}

#if PPD_INST == 4
template hipError_t launch_attn_t<128>(hipStream_t, const AttnArgs&, int, dim3, bool);
#elif PPD_INST == 5
template hipError_t launch_attn_t<64>(hipStream_t, const AttnArgs&, int, dim3, bool);
#endif
#endif

}  // namespace ppd
