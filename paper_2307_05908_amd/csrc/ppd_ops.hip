// Stand-alone early prediction (Sec. 3: the LM classifier applied to an intermediate hidden state, then the
// top-k of its output): one call outside any decoding context, for callers that run the transformer layers
// themselves.  Same kernels as a context's early head on row-major weights: final norm fused into the GEMM's
// prologue, every workgroup leaves its own top-k, one small kernel merges the lists.
#include "../../include/ppd.h"
#include "ppd_kernels.h"
#include "ppd_launch.h"

#include <string.h>

#include <mutex>

using namespace ppd;

namespace ppd {

__global__ __launch_bounds__(SEL_THREADS) void topk_merge_kernel(TopkMergeArgs a) {
  __shared__ float wv[SEL_THREADS / WAVE];
  __shared__ int wi[SEL_THREADS / WAVE];
  __shared__ int win[MAXM];
  __shared__ float winv[MAXM];
  merge_block_lists(a.pk_val, a.pk_idx, a.nblk, a.kk, a.k, wv, wi, win, winv);
  if ((int)threadIdx.x < a.k) {
    a.ids[threadIdx.x] = win[threadIdx.x];
    if (a.vals) a.vals[threadIdx.x] = winv[threadIdx.x];
  }
}

}  // namespace ppd

namespace {

constexpr int OPS_GMAX = 512;   // workgroup budget of the head GEMM (as in a context)

struct EarlyTopkPlan {
  int grid, KC;
  size_t lds;
  size_t logits_bytes, pk_bytes;   // scratch: logits [vocab] (when the caller takes none), block lists [grid][MAXM] twice
};

// argument checks shared by the variants; fills the launch plan
int early_topk_plan(int d_model, int vocab, int norm, int wdtype, const void* norm_g, const void* norm_b,
                    const void* head, const float* h, int k, const int32_t* ids_out, EarlyTopkPlan* p) {
  if (d_model < 8 || d_model % 8 || vocab < 1 || norm < 0 || norm > 1 || wdtype < 0 || wdtype > 1) return PPD_EINVAL;
  if (!norm_g || (norm == 0 && !norm_b) || !head || !h || !ids_out) return PPD_EINVAL;
  if (k < 1 || k > PPD_MAX_K || k > vocab) return PPD_EINVAL;
  if (((uintptr_t)h | (uintptr_t)head) & 15) return PPD_EINVAL;
  // one row, four weight rows per wave: the x tile holds the whole reduction length, or chunks of it
  const int span = 1024;   // staged k elements come in multiples of this (a float4 per thread; two k-blocks of 8 bf16 x 64 lanes)
  const int kpad = (d_model + span - 1) / span * span;
  const int kc_cap = GEMM_X_FLOATS / span * span;
  p->KC = kpad < kc_cap ? kpad : kc_cap;
  p->grid = head_grid_valu(vocab, OPS_GMAX);
  p->lds = (GEMM_LDS_HDR + (size_t)p->KC + HEAD_MAX_ROWS) * sizeof(float);
  p->logits_bytes = ((size_t)vocab * sizeof(float) + 255) & ~(size_t)255;
  p->pk_bytes = (size_t)p->grid * MAXM * sizeof(float);
  return PPD_OK;
}

// the two launches; logits, pk_val, pk_idx: DEVICE scratch (or the caller's logits buffer)
hipError_t early_topk_launch(const EarlyTopkPlan& p, int d_model, int vocab, int norm, float norm_eps, int wdtype,
                             const void* norm_g, const void* norm_b, const void* head, const float* h, int k,
                             float* logits, float* pk_val, int32_t* pk_idx, int32_t* ids_out, float* vals_out,
                             hipStream_t stream) {
  GemmArgs a; memset(&a, 0, sizeof a);
  GemmGroup& G = a.g[0];
  G.X = h; G.Rsd = nullptr; G.Y = logits; G.W[0] = head;
  G.ng = norm_g; G.nb = norm == 0 ? norm_b : nullptr; G.M = 1;
  a.K = d_model; a.N[0] = vocab; a.ntot = vocab; a.ldx = d_model; a.ldy = vocab;
  a.norm = norm; a.eps = norm_eps; a.act = 0; a.KC = p.KC;
  a.topk = k; a.pk_val = pk_val; a.pk_idx = pk_idx;
  hipError_t e = wdtype == 0 ? launch_gemm_t<float, false, 4>(stream, a, 1, 0, dim3(p.grid, 1), p.lds)
                             : launch_gemm_t<bf16_t, false, 4>(stream, a, 1, 0, dim3(p.grid, 1), p.lds);
  if (e != hipSuccess) return e;
  TopkMergeArgs t;
  t.pk_val = pk_val; t.pk_idx = pk_idx; t.nblk = p.grid; t.kk = k; t.k = k; t.ids = ids_out; t.vals = vals_out;
  hipLaunchKernelGGL(topk_merge_kernel, dim3(1), dim3(SEL_THREADS), 0, stream, t);
  return hipGetLastError();
}

// ---- the variant that allocates nothing: its scratch is this array (one copy per GPU, held until the process ends)
constexpr int NOALLOC_MAX_VOCAB = 65536;      // logits the array holds
constexpr int NOALLOC_MAX_GRID = 512;         // per-workgroup top-k lists it holds (OPS_GMAX workgroups at most for such vocabularies)
constexpr size_t NOALLOC_LOGITS_BYTES = (size_t)NOALLOC_MAX_VOCAB * sizeof(float);
constexpr size_t NOALLOC_PK_BYTES = (size_t)NOALLOC_MAX_GRID * MAXM * sizeof(float);
constexpr size_t NOALLOC_SCRATCH_BYTES = NOALLOC_LOGITS_BYTES + 2 * NOALLOC_PK_BYTES;   // 288 KiB
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

constexpr int NOALLOC_MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[NOALLOC_MAX_DEVICES];     // device address of `scratch` on each GPU, looked up at the first call there

// Device address of the current GPU's copy of the array (in host code the array's name is only a handle for this
// lookup, never an address to pass on).
hipError_t scratch_of_current_device(char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = (char*)g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" {

int ppd_early_topk(int d_model, int vocab, int norm, float norm_eps, int wdtype, const void* norm_g,
                   const void* norm_b, const void* head, const float* h, int k, int32_t* ids_out,
                   float* vals_out, float* logits_out, void* hip_stream) {
  EarlyTopkPlan p;
  int rc = early_topk_plan(d_model, vocab, norm, wdtype, norm_g, norm_b, head, h, k, ids_out, &p);
  if (rc) return rc;
  hipStream_t stream = (hipStream_t)hip_stream;
  char* buf = nullptr;
  const size_t lb = logits_out ? 0 : p.logits_bytes;
  hipError_t e = hipMalloc((void**)&buf, lb + 2 * p.pk_bytes);
  if (e != hipSuccess) { set_global_hip_error((int)e); (void)hipGetLastError(); return e == hipErrorOutOfMemory ? PPD_ENOMEM : PPD_EHIP; }
  float* logits = logits_out ? logits_out : (float*)buf;
  e = early_topk_launch(p, d_model, vocab, norm, norm_eps, wdtype, norm_g, norm_b, head, h, k, logits,
                        (float*)(buf + lb), (int32_t*)(buf + lb + p.pk_bytes), ids_out, vals_out, stream);
  const hipError_t es = hipStreamSynchronize(stream);   // the buffer is freed below: the launches must be done with it
  if (e == hipSuccess) e = es;
  (void)hipFree(buf);
  if (e != hipSuccess) { set_global_hip_error((int)e); (void)hipGetLastError(); return PPD_EHIP; }
  return PPD_OK;
}

int ppd_early_topk_noalloc(int d_model, int vocab, int norm, float norm_eps, int wdtype, const void* norm_g,
                           const void* norm_b, const void* head, const float* h, int k, int32_t* ids_out,
                           float* vals_out, float* logits_out, void* hip_stream) {
  EarlyTopkPlan p;
  int rc = early_topk_plan(d_model, vocab, norm, wdtype, norm_g, norm_b, head, h, k, ids_out, &p);
  if (rc) return rc;
  if (vocab > NOALLOC_MAX_VOCAB || p.grid > NOALLOC_MAX_GRID) return PPD_ELIMIT;
  char* sp = nullptr;
  hipError_t e = scratch_of_current_device(&sp);
  if (e == hipSuccess) {
    // nothing in the array has to start at zero: the GEMM writes every logit and the first k entries of every
    // workgroup's list, and the merge reads only those
    float* logits = logits_out ? logits_out : (float*)sp;
    e = early_topk_launch(p, d_model, vocab, norm, norm_eps, wdtype, norm_g, norm_b, head, h, k, logits,
                          (float*)(sp + NOALLOC_LOGITS_BYTES), (int32_t*)(sp + NOALLOC_LOGITS_BYTES + NOALLOC_PK_BYTES),
                          ids_out, vals_out, (hipStream_t)hip_stream);
  }
  if (e != hipSuccess) { set_global_hip_error((int)e); (void)hipGetLastError(); return PPD_EHIP; }
  return PPD_OK;
}

}  // extern "C"
