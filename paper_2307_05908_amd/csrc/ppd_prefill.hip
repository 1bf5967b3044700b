// Kernel instances and launchers of the compute-bound prompt pass (ppd_prefill.h).
#define PPD_PREFILL_TU 1
#include "ppd_prefill.h"


namespace ppd {

hipError_t launch_pack_rows(hipStream_t stream, const PackArgs& a) {
  if (a.M < 1 || a.K < 8 || (a.K & 7) || (a.ld & 3) || a.MT != (a.M + 15) / 16 || a.KT != (a.K + 31) / 32) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pack_rows_kernel, dim3(a.MT * 16), dim3(MG_THREADS), 0, stream, a);
  return hipGetLastError();
}

template <bool PAIRED, int TN, int TMB>
static hipError_t launch_pgemm_t(hipStream_t stream, PGemmArgs a) {
  a.MB = (a.MT + TMB - 1) / TMB;
  a.NB = (a.NT + PG_WAVES * TN - 1) / (PG_WAVES * TN);
  a.GM = a.MB < PG_GROUP_M ? a.MB : PG_GROUP_M;
  a.GQ = PG_GROUP_Q;
  a.MBG = (a.MB + a.GM - 1) / a.GM;
  const int nbq = (a.NB + 7) / 8;
  const dim3 grid(8 * ((nbq + a.GQ - 1) / a.GQ) * a.GQ * a.MBG * a.GM);
  hipLaunchKernelGGL((pgemm_kernel<PAIRED, TN, TMB>), grid, dim3(PG_THREADS), (size_t)PG_R * PG_STAGE_BLKS * 1024, stream, a);
  return hipGetLastError();
}

hipError_t launch_pgemm(hipStream_t stream, PGemmArgs a, bool paired) {
  if (a.M < 1 || a.MT != (a.M + 15) / 16 || a.KT < 1 || a.NT < 1) return hipErrorInvalidValue;
  // narrow matrices take two blocks per wave so that the grid still fills the machine
  const int mb = (a.MT + 3) / 4;
  const int tn = ((a.NT + PG_WAVES * 4 - 1) / (PG_WAVES * 4)) * mb >= 384 ? 4 : 2;
  if (paired) return tn == 4 ? launch_pgemm_t<true, 4, 4>(stream, a) : launch_pgemm_t<true, 2, 4>(stream, a);
  return tn == 4 ? launch_pgemm_t<false, 4, 4>(stream, a) : launch_pgemm_t<false, 2, 4>(stream, a);
}

hipError_t launch_pkv_pack(hipStream_t stream, const PKvPackArgs& a, int head_dim) {
  if (a.M < 1 || a.JP != (a.M + 31) / 32 || (head_dim != 64 && head_dim != 128) || (a.d_model & 3)) return hipErrorInvalidValue;
  const dim3 grid(a.JP, a.H);
  if (head_dim == 128) hipLaunchKernelGGL(pkv_pack_kernel<128>, grid, dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(pkv_pack_kernel<64>, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

template <int HD, int QT>
static hipError_t launch_pattn_t(hipStream_t stream, const PAttnArgs& a) {
  const int MT = (a.M + 15) / 16;
  const dim3 grid((MT + 4 * QT - 1) / (4 * QT), a.H);
  const size_t lds = (size_t)2 * (4 * (HD / 32) + 2 * (HD / 16)) * 1024;
  hipLaunchKernelGGL((pattn_kernel<HD, QT>), grid, dim3(256), lds, stream, a);
  return hipGetLastError();
}

hipError_t launch_pattn(hipStream_t stream, const PAttnArgs& a, int head_dim) {
  if (a.M < 1 || a.JP != (a.M + 31) / 32 || (head_dim != 64 && head_dim != 128) || a.d_model % 32) return hipErrorInvalidValue;
  // rows per workgroup (64 QT): two query tiles per wave once the prompt gives enough workgroups (four would leave
  // one wave per SIMD: measured slower)
  const bool two = a.M >= 1024;
  if (head_dim == 128) return two ? launch_pattn_t<128, 2>(stream, a) : launch_pattn_t<128, 1>(stream, a);
  return two ? launch_pattn_t<64, 2>(stream, a) : launch_pattn_t<64, 1>(stream, a);
}

}  // namespace ppd
