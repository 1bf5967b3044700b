// Kernel instances and launchers of the compute-bound prompt pass (ppd_prefill.h).
#define PPD_PREFILL_TU 1
#include "ppd_prefill.h"

namespace ppd {

hipError_t launch_pack_rows(hipStream_t stream, const PackArgs& a) {
  if (a.M < 1 || a.K < 8 || (a.K & 7) || (a.ld & 3) || a.MT != (a.M + 15) / 16 || a.KT != (a.K + 31) / 32) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pack_rows_kernel, dim3(a.MT * 16), dim3(MG_THREADS), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_pgemm(hipStream_t stream, PGemmArgs a, bool paired) {
  if (a.M < 1 || a.MT != (a.M + 15) / 16 || a.KT < 1 || a.NT < 1) return hipErrorInvalidValue;
  // narrow matrices take two tiles per wave so that the grid still fills the machine
  const int mb = (a.MT + PG_TM - 1) / PG_TM;
  const int tn = ((a.NT + PG_WAVES * 4 - 1) / (PG_WAVES * 4)) * mb >= 384 ? 4 : 2;
  a.MB = mb;
  a.NB = (a.NT + PG_WAVES * tn - 1) / (PG_WAVES * tn);
  const dim3 grid(8 * ((a.NB + 7) / 8) * a.MB);
  if (paired) {
    if (tn == 4) hipLaunchKernelGGL((pgemm_kernel<true, 4>), grid, dim3(PG_THREADS), 0, stream, a);
    else hipLaunchKernelGGL((pgemm_kernel<true, 2>), grid, dim3(PG_THREADS), 0, stream, a);
  } else {
    if (tn == 4) hipLaunchKernelGGL((pgemm_kernel<false, 4>), grid, dim3(PG_THREADS), 0, stream, a);
    else hipLaunchKernelGGL((pgemm_kernel<false, 2>), grid, dim3(PG_THREADS), 0, stream, a);
  }
  return hipGetLastError();
}

hipError_t launch_pattn(hipStream_t stream, const PAttnArgs& a, int head_dim) {
  if (a.M < 1 || (head_dim != 64 && head_dim != 128)) return hipErrorInvalidValue;
  const dim3 grid((a.M + 63) / 64, a.H);
  if (head_dim == 128) hipLaunchKernelGGL(pattn_kernel<128>, grid, dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(pattn_kernel<64>, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace ppd
