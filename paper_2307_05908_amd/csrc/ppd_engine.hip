// Host side of libppd: context, round state machine of Algorithm 2, launch
// sequences.  All arithmetic of the method runs in the kernels of
// ppd_kernels.h; this file only decides which layers run on which rows.
#define PPD_ENGINE_TU 1
#include "../../include/ppd.h"
#include "../../include/ppd_measure.h"
#include "ppd_kernels.h"
#include "ppd_launch.h"
#include "ppd_prefill.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <chrono>

#include <new>
#include <vector>

using namespace ppd;

namespace {

struct LayerW {
  const void *ln1_g, *ln1_b, *wq, *wk, *wv, *wo, *bq, *bk, *bv, *bo, *ln2_g, *ln2_b, *w_in, *w_up, *w_out, *b_in, *b_out;
};

}  // namespace

struct ppd_ctx {
  ppd_model_dims d;
  int k, dbar, nb;   // nb = d - dbar: layers each candidate runs, = pipelined steps per round
  hipStream_t user_stream;   // the caller's stream: ppd_prefill orders the context's work after what it holds
  hipStream_t stream;        // the context's own stream: every launch goes here (a graph cannot be captured on the null stream)
  hipStream_t cur;           // stream the launch helpers issue to
  hipEvent_t join_ev;
  int wbytes;                // bytes per weight element
  static constexpr int kvbytes = 4;   // keys and values are cached in fp32, like every other activation
  // weights (borrowed)
  const void *tok_emb, *pos_emb, *lnf_g, *lnf_b, *lm_head, *early_head;
  std::vector<LayerW> L;
  // bf16 models: weights repacked into MFMA blocks (owned copies); fp32 models stream the caller's tensors
  int mfma;
  int mg_passes_min;     // least number of staging passes of launches without a fused norm (1; tests force more)
  struct LayerP { void *qkv, *o, *fin, *fout; };
  std::vector<LayerP> LP;
  void *head_p, *early_p;
  std::vector<void*> owned;   // every repacked buffer, for ppd_destroy
  // device memory owned by the context
  char *Kc, *Vc;         // [L][H][16-position blocks][hd/16][64][4] fp32 (see k_index / v_index)
  char *tailK, *tailV;   // [nb][k][H][hd]
  // activation rows: max(1 + k, rows of a prompt chunk); row 0: main token, rows 1..k: candidates
  float *h;              // [rows][d_model]
  float *qkv;            // [rows][3*d_model]
  float *att;            // [rows][d_model]
  float *ffn;            // [rows][d_ff]
  float *part;           // [rows][H][nchunk_max][hd+2]
  float *logits, *early_logits;  // [1 + k][vocab] (row 0: the main token's), [vocab]
  float *early_spec;             // [2][vocab] early logits predicted at the end of the previous round (spec)
  float *pk_val; int32_t *pk_idx; // [1 + k][pk_slots][MAXM] block top-k candidates of the head GEMM, per row
  size_t pk_slots;
  // Speculative early prediction: with the exit layer at d/2 and no separate early head, the candidate
  // rows end a round exactly where the next round's early prediction reads the main row.  The final head
  // then runs on all 1 + k rows; after a match the matching row's top-k are the next candidates and the
  // next round (kind 3) starts with its parallel phase: one head pass per matching round instead of two.
  int spec;
  int last_kind;         // kind of the last round (which buffer holds its early logits)
  int prefill_chunk;     // prompt positions per chunk
  // compute-bound prompt pass (bf16 models, prompts of at least PREFILL_TILED_MIN rows): all rows at once through
  // tiled MFMA GEMMs and causal attention over two-term operand blocks; its buffers are made at the first such prompt
  int prefill_tiled;
  int pf_rows;           // rows the buffers below hold
  float *pf_h, *pf_qkv;  // [pf_rows][d_model | 3 d_model]
  uint16_t *pf_xp;       // packed two-term rows: the normalised hidden rows (input of the QKV and FFN-in GEMMs),
  uint16_t *pf_xa;       // the attention outputs (written by the attention kernel),
  uint16_t *pf_xf;       // the feed-forward activations (written by the FFN-in GEMM; zero beyond d_ff)
  uint16_t *pf_qp, *pf_kp, *pf_vp;   // one layer's queries, keys, values as two-term operand blocks of the prompt attention
  int dev_pos_pending;   // host mirror of the device state's pending position (-1: unknown)
  float* xn;             // [rows][d_model] normalised rows of a prompt chunk (norm_rows_kernel)
  // sampling-based final prediction (Appendix B): 0 arg max, 1 top-k sampling, 2 top-p sampling
  int samp_mode, samp_k; double samp_p; uint64_t samp_seed;
  double* samp_w; uint32_t* samp_keys; int samp_npad;   // scratch of the sampling kernel
  int head_grid;
  float2 *rope;          // [max_ctx][hd/2]
  DevState *ds;
  int32_t *prompt_dev;   // [max_ctx]
  int32_t *host_result;  // pinned: token, match index, the round's candidates, number of finished rounds
  int32_t rounds_seen;   // value of that counter after the last round the host waited for
  int32_t *host_result_dev; // the same memory as the GPU sees it
  // captured rounds: 0 ppd round from layer 1, 1 ppd round after a match, 2 plain step, 3 ppd round after a
  // match whose candidates were predicted by the round before
  int use_graphs;
  hipGraphExec_t graph[4];
  int graph_chunks[4];   // attention grid (64-position chunks) each graph was captured with
  int gmax1, gmax2;      // workgroup budget of an fp32 GEMM launch: one group / per group of a two-group launch
  int nchunk_max;
  // round state
  int n_ctx;      // absolute position of the pending token x_t (-1: no prefill yet)
  int matched;    // the pending token already went through layers 1..nb (its h is row 0)
  int finished;   // last token was EOS
  int have_early;
  ppd_stats st;
  int last_hip;
  // profiling
  int prof;
  std::vector<hipEvent_t> ev;   // pairs
  std::vector<int> ev_class;
  size_t ev_used;
  double kc_ms[2 * PPD_KC_COUNT];   // [groups-1][class]
  uint64_t kc_n[2 * PPD_KC_COUNT];
};

namespace {

int g_create_hip_error = 0;   // hipError_t of the last context-free call (ppd_create included) that failed with PPD_EHIP / PPD_ENOMEM

#define HIPCHK(ctx, call)                       \
  do {                                          \
    hipError_t e_ = (call);                     \
    if (e_ != hipSuccess) {                     \
      (ctx)->last_hip = (int)e_;                \
      return PPD_EHIP;                          \
    }                                           \
  } while (0)

inline size_t cache_head_floats(const ppd_ctx* c) { return kv_blocks(c->d.max_ctx) * KV_BLOCK * c->d.head_dim; }
inline size_t cache_layer_bytes(const ppd_ctx* c) { return (size_t)c->d.n_heads * cache_head_floats(c) * sizeof(float); }

struct ProfScope {
  ppd_ctx* c; int cls; size_t idx; bool on; hipStream_t st = nullptr;
  ProfScope(ppd_ctx* c_, int cls_, int groups = 1)
      : c(c_), cls(cls_ + (groups - 1) * PPD_KC_COUNT), idx(0), on(c_->prof >= 2 || (c_->prof == 1 && cls_ == PPD_KC_PHASE)) {
    if (!on) return;
    if (c->ev_used + 2 > c->ev.size()) {
      for (int i = 0; i < 2; ++i) { hipEvent_t e; if (hipEventCreate(&e) != hipSuccess) { on = false; return; } c->ev.push_back(e); }
      c->ev_class.push_back(cls);
    }
    idx = c->ev_used; c->ev_used += 2;
    c->ev_class[idx / 2] = cls;
    st = c->cur; (void)hipEventRecord(c->ev[idx], st);
  }
  ~ProfScope() { if (on) (void)hipEventRecord(c->ev[idx + 1], st); }
};

void prof_collect(ppd_ctx* c) {   // stream must be idle
  for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->ev[i], c->ev[i + 1]) == hipSuccess) {
      c->kc_ms[c->ev_class[i / 2]] += ms;
      c->kc_n[c->ev_class[i / 2]] += 1;
    }
  }
  c->ev_used = 0;
}

// ------------------------------------------------------------ launch helpers
// one skinny GEMM launch; group 0 is always one row, group 1 (optional) has MB rows
hipError_t launch_gemm(ppd_ctx* c, GemmArgs& a, int ngroups, bool paired) {
  const int vec = 16 / c->wbytes;
  const int gmax = ngroups == 2 ? c->gmax2 : c->gmax1;
  const int mmax = ngroups == 2 ? (a.g[1].M > a.g[0].M ? a.g[1].M : a.g[0].M) : a.g[0].M;
  const int x_budget = GEMM_X_FLOATS / mmax;   // k elements of x per row that fit the LDS tile
  // rows a wave streams together: 4, or 2 when 4 would leave waves of the grid without a set
  int wr = 4;
  const int wrows = a.ntot * (paired ? 2 : 1);
  if (a.topk == 0 && (wrows + 3) / 4 < gmax * GEMM_WAVES && x_budget >= (GEMM_BATCH / 2) * WAVE * vec && x_budget >= GEMM_THREADS * 4) wr = 2;
  int span2 = (GEMM_BATCH / wr) * WAVE * vec;
  if (span2 < GEMM_THREADS * 4) span2 = GEMM_THREADS * 4;   // tile rows are a whole number of float4 per thread too
  int kc_cap = x_budget / span2 * span2;
  if (kc_cap < span2) kc_cap = span2;
  const int kpad = (a.K + span2 - 1) / span2 * span2;
  a.KC = kpad < kc_cap ? kpad : kc_cap;
  const int lr = paired ? wr / 2 : wr;
  const int nsets = (a.ntot + lr - 1) / lr;
  int gx;
  if (a.topk > 0) gx = c->head_grid;
  else gx = pick_grid(nsets, gmax);
  dim3 grid(gx, ngroups);
  size_t lds = (GEMM_LDS_HDR + (size_t)mmax * a.KC + (a.topk > 0 ? HEAD_MAX_ROWS : 0)) * sizeof(float);
  int MB = ngroups == 2 ? a.g[1].M : 0;
  const int MA = a.g[0].M;
  if (c->wbytes == 4) {
    if (wr == 4) return paired ? launch_gemm_t<float, true, 4>(c->cur, a, MA, MB, grid, lds)
                               : launch_gemm_t<float, false, 4>(c->cur, a, MA, MB, grid, lds);
    return paired ? launch_gemm_t<float, true, 2>(c->cur, a, MA, MB, grid, lds)
                  : launch_gemm_t<float, false, 2>(c->cur, a, MA, MB, grid, lds);
  }
  return hipErrorInvalidValue;   // bf16 weights never come here: they take the MFMA kernel
}

// rows of a prompt chunk (ppd_prefill feeds the prompt through the decode kernels this many positions at a time:
// one pass over the weights per chunk instead of per token): the 16 columns of an MFMA tile for bf16 models,
// the 8 rows of the fp32 GEMM otherwise
constexpr int PREFILL_CHUNK = 16;
constexpr int PREFILL_CHUNK_FP32 = 8;

// ---- bf16 models: MFMA GEMM on repacked weights
constexpr size_t MG_LDS_MAX = 160 * 1024;

// One logical GEMM for one or two row groups.  Everything goes into one launch when the staged rows of
// the largest group fit LDS; otherwise every group is launched on its own, its rows in slices that fit
// (each slice streams the weights again).
hipError_t launch_mgemm(ppd_ctx* c, MGemmArgs& a, int ngroups, bool paired) {
  a.KT = (a.K + 31) / 32;
  if ((size_t)a.NT * a.KT * 1024 > 0x7fffffffu) return hipErrorInvalidValue;   // 32-bit offsets into one matrix
  a.wbytes = (unsigned)((size_t)a.NT * a.KT * 1024);
  int mmax = a.g[0].M;
  if (ngroups == 2 && a.g[1].M > mmax) mmax = a.g[1].M;
  auto lds_with = [&](int M, int tiles, int passes) {
    int b, p, x;
    return (size_t)mg_lds_layout(a.K, M, a.norm, tiles, mg_xrow_pass(a.KT, passes), b, p, x);
  };
  // Passes over the reduction length: 1 when the staged rows of the largest group fit LDS (next to the
  // partial sums of a one-workgroup-per-unit grid); launches without a fused norm otherwise stage the rows
  // in the fewest passes that fit (same arithmetic, weights still read once).  Launches with a fused
  // norm need whole rows: those fall back to row slices below.
  const int t1 = a.topk > 0 ? (a.NT + c->head_grid - 1) / c->head_grid : (a.NT + 255) / 256;
  const int tcap = (a.topk > 0 || ngroups == 1) ? t1 : t1 * 2;   // tiles per workgroup of this launch shape
  a.passes = c->mg_passes_min;
  if (a.norm >= 0) a.passes = 1;
  else while (a.passes < 8 && lds_with(mmax, tcap, a.passes) > MG_LDS_MAX) ++a.passes;
  {
    // a pass covers at least one batch of every wave's share: more passes than batches would be empty ones
    const int nb8 = (a.KT + MG_WAVES - 1) / MG_WAVES, useful = (nb8 + MG_BATCH - 1) / MG_BATCH;
    if (a.passes > useful) a.passes = useful;
  }
  a.xrow = mg_xrow_pass(a.KT, a.passes);
  // head launches keep HEAD_MAX_ROWS logits per row where the staged rows were
  if (a.topk > 0 && a.xrow < HEAD_MAX_ROWS * (int)sizeof(float)) a.xrow = HEAD_MAX_ROWS * (int)sizeof(float);
  auto lds_for = [&](int M, int tiles) { int b, p, x; return (size_t)mg_lds_layout(a.K, M, a.norm, tiles, a.xrow, b, p, x); };
  // Workgroups per group: the launch's share of the machine (one workgroup of 8 waves per compute unit),
  // then the smallest grid with the same number of tiles per workgroup, so that all of them finish together.
  auto go = [&](MGemmArgs x, int ng, int mm) -> hipError_t {
    int gx;
    if (x.topk > 0) gx = c->head_grid;
    else {
      const int gmax = 256 / ng;
      const int t = (x.NT + gmax - 1) / gmax;
      gx = (x.NT + t - 1) / t;
    }
    if (gx > x.NT) gx = x.NT;
    x.tiles_wg = (x.NT + gx - 1) / gx;
    const size_t lds = lds_for(mm, x.tiles_wg);
    if (lds > MG_LDS_MAX || (x.topk > 0 && x.tiles_wg * 16 > HEAD_MAX_ROWS)) return hipErrorInvalidValue;
    dim3 grid(gx, ng);
    if (x.passes > 1) {
      if (paired) hipLaunchKernelGGL((gemm_mfma_kernel<true, true>), grid, dim3(MG_THREADS), lds, c->cur, x);
      else hipLaunchKernelGGL((gemm_mfma_kernel<false, true>), grid, dim3(MG_THREADS), lds, c->cur, x);
    } else if (paired) hipLaunchKernelGGL((gemm_mfma_kernel<true, false>), grid, dim3(MG_THREADS), lds, c->cur, x);
    else hipLaunchKernelGGL((gemm_mfma_kernel<false, false>), grid, dim3(MG_THREADS), lds, c->cur, x);
    return hipGetLastError();
  };
  // rows whose staged form fits LDS
  int mcap = 0;
  while (mcap < 16 && lds_for(mcap + 1, tcap) <= MG_LDS_MAX) ++mcap;
  if (a.topk > 0 && mmax > mcap) return hipErrorInvalidValue;   // head launches are never cut into row slices
  if (mmax <= mcap) return go(a, ngroups, mmax);
  if (mcap < 1) return hipErrorInvalidValue;
  for (int g = 0; g < ngroups; ++g) {
    for (int r0 = 0; r0 < a.g[g].M; r0 += mcap) {
      MGemmArgs x = a;
      MGemmGroup G = a.g[g];
      const int mc = G.M - r0 < mcap ? G.M - r0 : mcap;
      G.X += (size_t)r0 * a.ldx; G.Y += (size_t)r0 * a.ldy; if (G.Rsd) G.Rsd += (size_t)r0 * a.ldy; G.M = mc;
      x.g[0] = G;
      hipError_t e = go(x, 1, mc);
      if (e != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

// pmax: largest position any row of the launch sits at (host-side bound for the grid; the kernel
// itself reads the position from the device state and idle chunks return at once)
hipError_t launch_attn(ppd_ctx* c, const AttnArgs& a, int ngroups, int pmax) {
  dim3 grid(pmax / ATT_CHUNK + 1, a.H, ngroups);
  int mmax = a.g[0].M;
  if (ngroups == 2 && a.g[1].M > mmax) mmax = a.g[1].M;
  const bool causal = a.g[0].causal != 0;
  if (causal && ngroups != 1) return hipErrorInvalidValue;
  if (c->d.head_dim == 64) return launch_attn_t<64>(c->cur, a, mmax, grid, causal);
  return launch_attn_t<128>(c->cur, a, mmax, grid, causal);
}

// the same launch described for the MFMA kernel: P[g] = group g's repacked weights
hipError_t mgemm_from(ppd_ctx* c, const GemmArgs& a, int ngroups, bool paired, void* const* P) {
  MGemmArgs m; memset(&m, 0, sizeof m);
  for (int g = 0; g < ngroups; ++g) {
    const GemmGroup& s = a.g[g];
    MGemmGroup& t = m.g[g];
    t.X = s.X; t.Rsd = s.Rsd; t.Y = s.Y; t.P = P[g];
    t.B[0] = s.B[0]; t.B[1] = s.B[1]; t.B[2] = s.B[2]; t.ng = s.ng; t.nb = s.nb; t.M = s.M;
  }
  m.K = a.K; m.N[0] = a.N[0]; m.N[1] = a.N[1]; m.N[2] = a.N[2]; m.ntot = a.ntot;
  m.NT = paired ? (a.ntot + 7) / 8 : (a.ntot + 15) / 16;
  m.ldx = a.ldx; m.ldy = a.ldy; m.norm = a.norm; m.eps = a.eps; m.act = a.act == 3 ? 0 : a.act;
  m.topk = a.topk; m.pk_val = a.pk_val; m.pk_idx = a.pk_idx; m.pk_stride = (int)c->pk_slots;
  return launch_mgemm(c, m, ngroups, paired);
}

// A row group of one layer step: which layer, how many rows, first row in the
// activation buffers, absolute position, and where the rows' own K/V go.
struct RowGroup {
  int layer;     // 0-based
  int M;
  int row0;      // 0: main row; 1: first candidate row
  int pos_off;   // the rows' token sits at position (device state pos) + pos_off
  bool tail;     // own K/V go to the candidate tails (slot = row index) instead of the cache
  bool chunk = false;   // prompt chunk: row m sits m positions further on and sees the rows before it
};

// Prompt chunk: the rows of group 0 are normalised by a kernel of their own (same arithmetic as the fused norm)
// and the GEMM runs without a fused norm on the result, so that it can stage its rows in passes.
int norm_chunk(ppd_ctx* c, GemmArgs& a, const void* gain, const void* bias) {
  NormRowsArgs n; memset(&n, 0, sizeof n);
  n.X = a.g[0].X; n.Y = c->xn; n.g = gain; n.b = bias; n.K = a.K; n.ld = a.ldx; n.norm = a.norm; n.eps = a.eps;
  hipLaunchKernelGGL(norm_rows_kernel, dim3(a.g[0].M), dim3(MG_THREADS), 0, c->cur, n);
  HIPCHK(c, hipGetLastError());
  a.g[0].X = c->xn; a.g[0].ng = nullptr; a.g[0].nb = nullptr; a.norm = -1;
  return PPD_OK;
}

// One transformer layer for one or two row groups (a pipelined step when two).
// pmax: host-side upper bound of the rows' positions (sizes the attention grid only).
int run_layer(ppd_ctx* c, int ngroups, const RowGroup* rg, int pmax, int stages = 15) {
  const ppd_model_dims& d = c->d;
  const int dm = d.d_model, F = d.d_ff;
  const bool bias = d.has_bias != 0;
  // stages: bit 0 = steps 1-2 (attention half), bit 1 = step 3, bit 2 = step 4, bit 3 = step 5
  // 1. norm1 + QKV
  if (stages & 1) {
    GemmArgs a; memset(&a, 0, sizeof a);
    for (int g = 0; g < ngroups; ++g) {
      const LayerW& w = c->L[rg[g].layer];
      GemmGroup& G = a.g[g];
      G.X = c->h + (size_t)rg[g].row0 * dm; G.Rsd = nullptr; G.Y = c->qkv + (size_t)rg[g].row0 * 3 * dm;
      G.W[0] = w.wq; G.W[1] = w.wk; G.W[2] = w.wv;
      G.B[0] = bias ? w.bq : nullptr; G.B[1] = bias ? w.bk : nullptr; G.B[2] = bias ? w.bv : nullptr;
      G.ng = w.ln1_g; G.nb = d.norm == 0 ? w.ln1_b : nullptr; G.M = rg[g].M;
    }
    a.K = dm; a.N[0] = a.N[1] = a.N[2] = dm; a.ntot = 3 * dm; a.ldx = dm; a.ldy = 3 * dm;
    a.norm = d.norm; a.eps = d.norm_eps; a.act = 0;
    if (rg[0].chunk && c->mfma) { int rc = norm_chunk(c, a, c->L[rg[0].layer].ln1_g, d.norm == 0 ? c->L[rg[0].layer].ln1_b : nullptr); if (rc) return rc; }
    ProfScope ps(c, PPD_KC_GEMM_QKV, ngroups);
    if (c->mfma) {
      void* P[2] = {c->LP[rg[0].layer].qkv, ngroups == 2 ? c->LP[rg[1].layer].qkv : nullptr};
      HIPCHK(c, mgemm_from(c, a, ngroups, false, P));
    } else
    HIPCHK(c, launch_gemm(c, a, ngroups, false));
  }
  // 2. RoPE + KV write + attention partials, then merge
  if (stages & 1) {
    AttnArgs a; memset(&a, 0, sizeof a);
    MergeArgs mg; memset(&mg, 0, sizeof mg);
    const size_t part_row = (size_t)d.n_heads * c->nchunk_max * (d.head_dim + 2);
    for (int g = 0; g < ngroups; ++g) {
      AttnGroup& G = a.g[g];
      const int l = rg[g].layer;
      G.qkv = c->qkv + (size_t)rg[g].row0 * 3 * dm;
      G.Kc = (float*)(c->Kc + (size_t)l * cache_layer_bytes(c));
      G.Vc = (float*)(c->Vc + (size_t)l * cache_layer_bytes(c));
      G.tailK = (float*)c->tailK + (size_t)l * c->k * dm;
      G.tailV = (float*)c->tailV + (size_t)l * c->k * dm;
      G.own_cache = rg[g].tail ? 0 : 1;
      G.part = c->part + (size_t)rg[g].row0 * part_row;
      G.pos_off = rg[g].pos_off; G.M = rg[g].M;
      G.causal = rg[g].chunk ? 1 : 0; mg.causal[g] = G.causal;
      if (rg[g].chunk) {
        // keys and values of all rows of the chunk go into the cache first
        if (ngroups != 1 || rg[g].tail || rg[g].pos_off != 0) return PPD_EINVAL;
        ChunkKvArgs kv; memset(&kv, 0, sizeof kv);
        kv.qkv = G.qkv; kv.Kc = G.Kc; kv.Vc = G.Vc; kv.rope = d.pos == 1 ? c->rope : nullptr; kv.ds = c->ds;
        kv.HD = d.head_dim; kv.d_model = dm; kv.max_ctx = d.max_ctx;
        hipLaunchKernelGGL(chunk_kv_kernel, dim3(G.M, d.n_heads), dim3(d.head_dim), 0, c->cur, kv);
        HIPCHK(c, hipGetLastError());
      }
      mg.part[g] = G.part; mg.out[g] = c->att + (size_t)rg[g].row0 * dm; mg.pos_off[g] = G.pos_off; mg.M[g] = G.M;
    }
    a.ds = c->ds; mg.ds = c->ds;
    a.rope = d.pos == 1 ? c->rope : nullptr;
    a.H = d.n_heads; a.d_model = dm; a.max_ctx = d.max_ctx; a.nchunk_max = c->nchunk_max;
    a.scale = 1.0f / sqrtf((float)d.head_dim);
    { ProfScope ps(c, PPD_KC_ATTN, ngroups); HIPCHK(c, launch_attn(c, a, ngroups, pmax)); }
    mg.H = d.n_heads; mg.HD = d.head_dim; mg.d_model = dm; mg.nchunk_max = c->nchunk_max;
    int mmax = rg[0].M; if (ngroups == 2 && rg[1].M > mmax) mmax = rg[1].M;
    ProfScope ps(c, PPD_KC_ATTN_MERGE, ngroups);
    hipLaunchKernelGGL(attn_merge_kernel, dim3(mmax, d.n_heads, ngroups), dim3(MERGE_THREADS), 0, c->cur, mg);
    HIPCHK(c, hipGetLastError());
  }
  // 3. output projection + residual
  if (stages & 2) {
    GemmArgs a; memset(&a, 0, sizeof a);
    for (int g = 0; g < ngroups; ++g) {
      const LayerW& w = c->L[rg[g].layer];
      GemmGroup& G = a.g[g];
      G.X = c->att + (size_t)rg[g].row0 * dm; G.Y = c->h + (size_t)rg[g].row0 * dm; G.Rsd = G.Y;
      G.W[0] = w.wo; G.B[0] = bias ? w.bo : nullptr; G.M = rg[g].M;
    }
    a.K = dm; a.N[0] = dm; a.ntot = dm; a.ldx = dm; a.ldy = dm; a.norm = -1; a.act = 0;
    ProfScope ps(c, PPD_KC_GEMM_O, ngroups);
    if (c->mfma) {
      void* P[2] = {c->LP[rg[0].layer].o, ngroups == 2 ? c->LP[rg[1].layer].o : nullptr};
      HIPCHK(c, mgemm_from(c, a, ngroups, false, P));
    } else
    HIPCHK(c, launch_gemm(c, a, ngroups, false));
  }
  // 4. norm2 + FFN in (+ gate/up pairing) + activation
  if (stages & 4) {
    GemmArgs a; memset(&a, 0, sizeof a);
    const bool swiglu = d.act == 2;
    for (int g = 0; g < ngroups; ++g) {
      const LayerW& w = c->L[rg[g].layer];
      GemmGroup& G = a.g[g];
      G.X = c->h + (size_t)rg[g].row0 * dm; G.Y = c->ffn + (size_t)rg[g].row0 * F; G.Rsd = nullptr;
      G.W[0] = w.w_in; G.W[1] = swiglu ? w.w_up : nullptr;
      G.B[0] = bias ? w.b_in : nullptr;
      G.ng = w.ln2_g; G.nb = d.norm == 0 ? w.ln2_b : nullptr; G.M = rg[g].M;
    }
    a.K = dm; a.N[0] = F; a.N[1] = swiglu ? F : 0; a.ntot = F; a.ldx = dm; a.ldy = F;
    a.norm = d.norm; a.eps = d.norm_eps; a.act = swiglu ? 3 : (d.act == 0 ? 1 : 2);
    if (rg[0].chunk && c->mfma) { int rc = norm_chunk(c, a, c->L[rg[0].layer].ln2_g, d.norm == 0 ? c->L[rg[0].layer].ln2_b : nullptr); if (rc) return rc; }
    ProfScope ps(c, PPD_KC_GEMM_FFN_IN, ngroups);
    if (c->mfma) {
      void* P[2] = {c->LP[rg[0].layer].fin, ngroups == 2 ? c->LP[rg[1].layer].fin : nullptr};
      HIPCHK(c, mgemm_from(c, a, ngroups, swiglu, P));
    } else
    HIPCHK(c, launch_gemm(c, a, ngroups, swiglu));
  }
  // 5. FFN out + residual
  if (stages & 8) {
    GemmArgs a; memset(&a, 0, sizeof a);
    for (int g = 0; g < ngroups; ++g) {
      const LayerW& w = c->L[rg[g].layer];
      GemmGroup& G = a.g[g];
      G.X = c->ffn + (size_t)rg[g].row0 * F; G.Y = c->h + (size_t)rg[g].row0 * dm; G.Rsd = G.Y;
      G.W[0] = w.w_out; G.B[0] = bias ? w.b_out : nullptr; G.M = rg[g].M;
    }
    a.K = F; a.N[0] = dm; a.ntot = dm; a.ldx = F; a.ldy = dm; a.norm = -1; a.act = 0;
    ProfScope ps(c, PPD_KC_GEMM_FFN_OUT, ngroups);
    if (c->mfma) {
      void* P[2] = {c->LP[rg[0].layer].fout, ngroups == 2 ? c->LP[rg[1].layer].fout : nullptr};
      HIPCHK(c, mgemm_from(c, a, ngroups, false, P));
    } else
    HIPCHK(c, launch_gemm(c, a, ngroups, false));
  }
  return PPD_OK;
}

EmbedArgs embed_args(ppd_ctx* c, const int32_t* ids_dev, int rows, int row0, int pos_off) {
  EmbedArgs a;
  a.tok_emb = c->tok_emb; a.pos_emb = c->d.pos == 0 ? c->pos_emb : nullptr; a.ids = ids_dev; a.ds = c->ds;
  a.h = c->h + (size_t)row0 * c->d.d_model; a.rows = rows; a.d_model = c->d.d_model; a.pos_off = pos_off; a.pos_step = 0;
  a.vocab = c->d.vocab;
  return a;
}

int run_embed(ppd_ctx* c, const int32_t* ids_dev, int rows, int row0, int pos_off) {
  EmbedArgs a = embed_args(c, ids_dev, rows, row0, pos_off);
  dim3 grid((c->d.d_model + 255) / 256, rows);
  ProfScope ps(c, PPD_KC_EMBED);
  if (c->wbytes == 4) hipLaunchKernelGGL(embed_kernel<float>, grid, dim3(256), 0, c->cur, a);
  else hipLaunchKernelGGL(embed_kernel<bf16_t>, grid, dim3(256), 0, c->cur, a);
  HIPCHK(c, hipGetLastError());
  return PPD_OK;
}

int set_state(ppd_ctx* c, int pos, int tok) {
  hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(64), 0, c->cur, c->ds, pos, tok);
  HIPCHK(c, hipGetLastError());
  c->dev_pos_pending = pos;
  return PPD_OK;
}

// Final norm + LM head on the main row with every workgroup's own top-k, then the selection
// kernel.  early: top-k -> candidates, which it also embeds as rows 1..k at the next position.
// final: arg max, verification; with adopt, the matching candidate's row and KV tails are adopted.
// With speculative early prediction the adopting head also runs on the candidate rows (see ppd_ctx::spec).
int run_head(ppd_ctx* c, bool early, bool adopt) {
  const ppd_model_dims& d = c->d;
  const bool spec = c->spec && adopt && !early;
  // top-k sampling with few kept tokens is drawn from the head's block lists inside the selection kernel;
  // other sampling goes through the sampling kernel
  const int ks_fast = (!early && c->samp_mode == 1 && c->samp_k <= MAXM) ? (c->samp_k < d.vocab ? c->samp_k : d.vocab) : 0;
  const bool samp_kernel = !early && c->samp_mode && !ks_fast;
  int topk = (early || spec) ? c->k : 1;
  if (ks_fast > topk) topk = ks_fast;
  {
    GemmArgs a; memset(&a, 0, sizeof a);
    GemmGroup& G = a.g[0];
    G.X = c->h; G.Y = early ? c->early_logits : c->logits; G.Rsd = nullptr;
    G.W[0] = (early && c->early_head) ? c->early_head : c->lm_head;
    G.ng = c->lnf_g; G.nb = d.norm == 0 ? c->lnf_b : nullptr; G.M = spec ? 1 + c->k : 1;
    a.K = d.d_model; a.N[0] = d.vocab; a.ntot = d.vocab; a.ldx = d.d_model; a.ldy = d.vocab;
    a.norm = d.norm; a.eps = d.norm_eps; a.act = 0;
    a.topk = topk; a.pk_val = c->pk_val; a.pk_idx = c->pk_idx;
    ProfScope ps(c, PPD_KC_HEAD);
    if (c->mfma) {
      void* P[2] = {(early && c->early_p) ? c->early_p : c->head_p, nullptr};
      HIPCHK(c, mgemm_from(c, a, 1, false, P));
    } else
    HIPCHK(c, launch_gemm(c, a, 1, false));
  }
  if (samp_kernel) {
    SampleArgs sa; memset(&sa, 0, sizeof sa);
    sa.z = c->logits; sa.n = d.vocab; sa.mode = c->samp_mode; sa.ks = c->samp_k; sa.p = c->samp_p; sa.seed = c->samp_seed;
    sa.ds = c->ds; sa.w = c->samp_w; sa.keys = c->samp_keys; sa.npad = c->samp_npad;
    ProfScope ps(c, PPD_KC_SELECT);
    if (d.vocab <= SAMP_VPT * SAMP_THREADS) hipLaunchKernelGGL(sample_kernel<true>, dim3(1), dim3(SAMP_THREADS), 0, c->cur, sa);
    else hipLaunchKernelGGL(sample_kernel<false>, dim3(1), dim3(SAMP_THREADS), 0, c->cur, sa);
    HIPCHK(c, hipGetLastError());
  }
  SelectArgs s; memset(&s, 0, sizeof s);
  s.sampled = samp_kernel ? 1 : 0; s.samp_topk = ks_fast; s.samp_seed = c->samp_seed;
  s.pk_val = c->pk_val; s.pk_idx = c->pk_idx; s.nblk = c->head_grid; s.kk = topk;
  s.pk_stride = (int)c->pk_slots;
  s.k = adopt || early ? c->k : 0; s.mode = early ? 0 : 1; s.ds = c->ds; s.host_result = c->host_result_dev;
  s.vocab = d.vocab;
  dim3 grid(1, 1);
  if (early) {
    s.emb = embed_args(c, nullptr, c->k, 1, 1);
    grid = dim3((d.d_model + SEL_THREADS - 1) / SEL_THREADS, c->k);
  } else if (adopt) {
    s.h = c->h; s.tailK = (const float*)c->tailK; s.tailV = (const float*)c->tailV; s.Kc = (float*)c->Kc; s.Vc = (float*)c->Vc;
    s.head_floats = cache_head_floats(c);
    s.nb = c->nb; s.H = d.n_heads; s.hd = d.head_dim; s.d_model = d.d_model; s.max_ctx = d.max_ctx;
    if (spec) {
      s.spec = 1; s.spec_logits = c->logits + d.vocab; s.early_spec = c->early_spec; s.vocab = d.vocab;
      s.emb = embed_args(c, nullptr, c->k, 1, 2);
    }
    // tail blocks, then (spec) blocks that copy the logits row / embed the next candidates, a column per thread
    const int extra = spec ? (d.d_model + SEL_THREADS - 1) / SEL_THREADS : 0;
    grid = dim3(c->nb + (extra > 16 ? 16 : extra), 2);
  }
  ProfScope ps(c, PPD_KC_SELECT);
  if (c->wbytes == 4) hipLaunchKernelGGL(select_kernel<float>, grid, dim3(SEL_THREADS), 0, c->cur, s);
  else hipLaunchKernelGGL(select_kernel<bf16_t>, grid, dim3(SEL_THREADS), 0, c->cur, s);
  HIPCHK(c, hipGetLastError());
  return PPD_OK;
}

// The launches of one round.  kind 0: PPD round from layer 1 (after a miss or a prefill);
// kind 1: PPD round after a match (layers 1..d-dbar were run by the matching candidate row);
// kind 2: plain greedy step; kind 3: PPD round after a match whose candidates the previous round's final head
// already predicted and embedded (speculative early prediction): parallel phase and final head only.  pmax bounds the positions touched (attention grid size only).
int issue_round(ppd_ctx* c, int kind, int pmax) {
  const int d = c->d.n_layers, dbar = c->dbar, nb = c->nb, k = c->k;
  int rc;
  hipLaunchKernelGGL(begin_round_kernel, dim3(1), dim3(64), 0, c->cur, c->ds, kind == 3 ? 1 : 0, c->host_result_dev + 2);
  HIPCHK(c, hipGetLastError());
  if (kind == 2) {
    if ((rc = run_embed(c, &c->ds->next_tok, 1, 0, 0))) return rc;
    for (int l = 0; l < d; ++l) {
      RowGroup g{l, 1, 0, 0, false};
      if ((rc = run_layer(c, 1, &g, pmax))) return rc;
    }
    return run_head(c, false, false);
  }
  // main token up to the exit layer
  int from = (kind == 1 || kind == 3) ? nb : 0;
  if (kind == 0 && (rc = run_embed(c, &c->ds->next_tok, 1, 0, 0))) return rc;
  if (from < dbar) {
    ProfScope phase(c, PPD_KC_PHASE, 1);
    for (int l = from; l < dbar; ++l) {
      RowGroup g{l, 1, 0, 0, false};
      if ((rc = run_layer(c, 1, &g, pmax))) return rc;
    }
  }
  // early prediction; the candidates become rows 1..k at the next position
  if (kind != 3 && (rc = run_head(c, true, false))) return rc;
  // parallel phase: step j runs the main row at layer dbar+j and the candidates at layer j
  {
    ProfScope phase(c, PPD_KC_PHASE, 2);
    for (int j = 0; j < nb; ++j) {
      RowGroup g[2] = {{dbar + j, 1, 0, 0, false}, {j, k, 1, 1, true}};
      if ((rc = run_layer(c, 2, g, pmax))) return rc;
    }
  }
  // final prediction, verification, adoption
  return run_head(c, false, true);
}

// Run one round: set the device state, replay (or capture, or issue eagerly) the launches,
// wait, read token and match index from pinned memory.
int run_round(ppd_ctx* c, int kind, int pos) {
  int rc;
  // (work the caller queued on its stream before ppd_prefill -- the weights -- was waited for there; a round
  // reads nothing else of the caller's)
  // the device already holds this position as pending when the previous call was a round at pos - 1
  if (c->dev_pos_pending != pos && (rc = set_state(c, pos, -1))) return rc;
  const int pmax = pos + (kind == 2 ? 0 : 1);
  if (c->use_graphs && !c->prof) {
    // Attention grid of the captured round: the chunks the round needs, rounded up to a power of two (at least 4,
    // at most the cache's), so that a sequence re-captures a handful of times instead of every 64 positions;
    // chunks past a row's position return at once.
    int nchunks = 4;
    while (nchunks < pmax / ATT_CHUNK + 1) nchunks *= 2;
    if (nchunks > c->nchunk_max) nchunks = c->nchunk_max;
    if (c->graph[kind] && c->graph_chunks[kind] < nchunks) {
      HIPCHK(c, hipGraphExecDestroy(c->graph[kind]));
      c->graph[kind] = nullptr;
    }
    if (!c->graph[kind]) {
      hipGraph_t g = nullptr;
      HIPCHK(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeRelaxed));
      rc = issue_round(c, kind, nchunks * ATT_CHUNK - 1);
      hipError_t e = hipStreamEndCapture(c->stream, &g);
      if (rc) { if (g) (void)hipGraphDestroy(g); return rc; }
      HIPCHK(c, e);
      e = hipGraphInstantiate(&c->graph[kind], g, nullptr, nullptr, 0);
      (void)hipGraphDestroy(g);
      HIPCHK(c, e);
      c->graph_chunks[kind] = nchunks;
    }
    HIPCHK(c, hipGraphLaunch(c->graph[kind], c->stream));
  } else {
    if ((rc = issue_round(c, kind, pmax))) return rc;
  }
  c->dev_pos_pending = -1;                       // (unknown until the round is known to have run)
  // The round's last kernel writes token and match index to pinned memory and then the count of finished rounds:
  // poll that word instead of sleeping in a stream synchronisation (the wake-up costs more than a round's tail).
  // Profiled rounds, and a round that does not report in time, take the synchronisation (which also surfaces errors).
  {
    volatile int32_t* seq = c->host_result + 2 + MAXM;
    const int32_t want = c->rounds_seen + 1;
    bool seen = false;
    if (!c->prof) {
      const auto t0 = std::chrono::steady_clock::now();
      for (unsigned spin = 0; !seen; ++spin) {
        seen = *seq == want;
        if (!seen && (spin & 1023u) == 1023u &&
            std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(200)) break;
      }
    }
    if (!seen) {
      HIPCHK(c, hipStreamSynchronize(c->stream));
      if (*seq != want) { c->last_hip = (int)hipErrorUnknown; return PPD_EHIP; }
    }
    std::atomic_thread_fence(std::memory_order_acquire);
    c->rounds_seen = want;
  }
  c->dev_pos_pending = pos + 1;                  // left by the round's final selection
  if (c->prof) prof_collect(c);
  return PPD_OK;
}

void account_round(ppd_ctx* c, int kind, int pos) {
  const ppd_model_dims& d = c->d;
  const uint64_t wl = ((uint64_t)4 * d.d_model * d.d_model + (uint64_t)(d.act == 2 ? 3 : 2) * d.d_model * d.d_ff) * c->wbytes;
  const uint64_t wh = (uint64_t)d.vocab * d.d_model * c->wbytes;
  const uint64_t kvp = (uint64_t)2 * d.d_model * c->kvbytes;    // K and V of one position of one layer
  if (kind == 2) {
    c->st.weight_bytes += d.n_layers * wl + wh;
    c->st.kv_bytes += (uint64_t)d.n_layers * pos * kvp;
    return;
  }
  const int solo = c->dbar - (kind == 0 ? 0 : c->nb);
  c->st.weight_bytes += (uint64_t)(solo + 2 * c->nb) * wl + (kind == 3 ? 1 : 2) * wh;
  c->st.kv_bytes += (uint64_t)(solo + c->nb) * pos * kvp + (uint64_t)c->nb * (pos + 1) * kvp;
}

void free_all(ppd_ctx* c) {
  for (int i = 0; i < 4; ++i) if (c->graph[i]) (void)hipGraphExecDestroy(c->graph[i]);
  void* dev[] = {c->Kc, c->Vc, c->tailK, c->tailV, c->h, c->qkv, c->att, c->ffn, c->part, c->logits,
                 c->early_logits, c->early_spec, c->samp_w, c->samp_keys, c->xn, c->pf_h, c->pf_qkv, c->pf_xp, c->pf_xa, c->pf_xf, c->pf_qp, c->pf_kp, c->pf_vp, c->rope, c->ds, c->prompt_dev, c->pk_val, c->pk_idx};
  for (void* p : dev) (void)hipFree(p);
  for (void* p : c->owned) (void)hipFree(p);
  if (c->host_result) (void)hipHostFree(c->host_result);
  for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
  if (c->join_ev) (void)hipEventDestroy(c->join_ev);
  if (c->stream) (void)hipStreamDestroy(c->stream);
}

constexpr int PREFILL_TILED_MIN = 32;

// The whole prompt (rows 0 .. rows-1 at positions 0 .. rows-1) through all layers: fills the cache.
int prefill_tiled(ppd_ctx* c, int rows) {
  const ppd_model_dims& d = c->d;
  const int dm = d.d_model, F = d.d_ff;
  const bool bias = d.has_bias != 0, swiglu = d.act == 2;
  if (rows > c->pf_rows) {
    void* old[] = {c->pf_h, c->pf_qkv, c->pf_xp, c->pf_xa, c->pf_xf, c->pf_qp, c->pf_kp, c->pf_vp};
    for (void* p : old) (void)hipFree(p);
    c->pf_h = c->pf_qkv = nullptr; c->pf_xp = c->pf_xa = c->pf_xf = nullptr; c->pf_qp = c->pf_kp = c->pf_vp = nullptr; c->pf_rows = 0;
    const size_t R = (size_t)((rows + 63) / 64) * 64;
    HIPCHK(c, hipMalloc((void**)&c->pf_h, R * dm * sizeof(float)));
    HIPCHK(c, hipMalloc((void**)&c->pf_qkv, R * 3 * dm * sizeof(float)));
    HIPCHK(c, hipMalloc((void**)&c->pf_xp, packed_bytes((int)R, dm)));
    HIPCHK(c, hipMalloc((void**)&c->pf_xa, packed_bytes((int)R, dm)));
    HIPCHK(c, hipMalloc((void**)&c->pf_xf, packed_bytes((int)R, F)));
    HIPCHK(c, hipMalloc((void**)&c->pf_qp, pattn_stage_bytes((int)R, d.n_heads, d.head_dim)));
    HIPCHK(c, hipMalloc((void**)&c->pf_kp, pattn_stage_bytes((int)R, d.n_heads, d.head_dim)));
    HIPCHK(c, hipMalloc((void**)&c->pf_vp, pattn_stage_bytes((int)R, d.n_heads, d.head_dim)));
    c->pf_rows = (int)R;
  }
  // (the packed layouts depend on the row count: the padding columns of the activations are cleared per prompt)
  HIPCHK(c, hipMemsetAsync(c->pf_xf, 0, packed_bytes(rows, F), c->cur));
  int rc = set_state(c, 0, -1);
  if (rc) return rc;
  {
    EmbedArgs ea = embed_args(c, c->prompt_dev, rows, 0, 0);
    ea.h = c->pf_h; ea.pos_step = 1;
    hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3((dm + 255) / 256, rows), dim3(256), 0, c->cur, ea);
    HIPCHK(c, hipGetLastError());
  }
  const int MT = (rows + 15) / 16;
  auto pack = [&](const float* X, int ld, int K, const void* g, const void* b, int norm) -> hipError_t {
    PackArgs p; memset(&p, 0, sizeof p);
    p.X = X; p.ld = ld; p.M = rows; p.K = K; p.KT = (K + 31) / 32; p.MT = MT; p.g = g; p.b = b; p.norm = norm; p.eps = d.norm_eps;
    p.out = c->pf_xp;
    return launch_pack_rows(c->cur, p);
  };
  auto gemm = [&](const uint16_t* Xp, const void* P, int K, int n0, int n1, int n2, bool paired, const void* b0, const void* b1, const void* b2,
                  const float* rsd, float* Y, int ldy, int act, uint16_t* Yp = nullptr) -> hipError_t {
    PGemmArgs g; memset(&g, 0, sizeof g);
    g.Xp = Xp; g.P = P; g.Yp = Yp; g.KTp = (n0 + 31) / 32; g.B[0] = b0; g.B[1] = b1; g.B[2] = b2; g.Rsd = rsd; g.Y = Y;
    g.M = rows; g.MT = MT; g.KT = (K + 31) / 32;
    g.N[0] = n0; g.N[1] = n1; g.N[2] = n2; g.ntot = paired ? n0 : n0 + n1 + n2;
    g.NT = paired ? (n0 + 7) / 8 : (g.ntot + 15) / 16;
    g.ldy = ldy; g.act = act;
    return launch_pgemm(c->cur, g, paired);
  };
  for (int l = 0; l < d.n_layers; ++l) {
    const LayerW& w = c->L[l];
    const ppd_ctx::LayerP& P = c->LP[l];
    HIPCHK(c, pack(c->pf_h, dm, dm, w.ln1_g, d.norm == 0 ? w.ln1_b : nullptr, d.norm));
    HIPCHK(c, gemm(c->pf_xp, P.qkv, dm, dm, dm, dm, false, bias ? w.bq : nullptr, bias ? w.bk : nullptr, bias ? w.bv : nullptr,
                   nullptr, c->pf_qkv, 3 * dm, 0));
    {
      PKvPackArgs pk; memset(&pk, 0, sizeof pk);
      pk.qkv = c->pf_qkv; pk.rope = d.pos == 1 ? c->rope : nullptr; pk.Qp = c->pf_qp; pk.Kp = c->pf_kp; pk.Vp = c->pf_vp;
      pk.Kc = (float*)(c->Kc + (size_t)l * cache_layer_bytes(c)); pk.Vc = (float*)(c->Vc + (size_t)l * cache_layer_bytes(c));
      pk.max_ctx = d.max_ctx; pk.M = rows; pk.H = d.n_heads; pk.d_model = dm; pk.JP = (rows + 31) / 32; pk.scale = 1.44269504088896340736f / sqrtf((float)d.head_dim);
      HIPCHK(c, launch_pkv_pack(c->cur, pk, d.head_dim));
      PAttnArgs pa; memset(&pa, 0, sizeof pa);
      pa.Qp = c->pf_qp; pa.Kp = c->pf_kp; pa.Vp = c->pf_vp; pa.outp = c->pf_xa;
      pa.M = rows; pa.H = d.n_heads; pa.d_model = dm; pa.JP = pk.JP;
      HIPCHK(c, launch_pattn(c->cur, pa, d.head_dim));
    }
    HIPCHK(c, gemm(c->pf_xa, P.o, dm, dm, 0, 0, false, bias ? w.bo : nullptr, nullptr, nullptr, c->pf_h, c->pf_h, dm, 0));
    HIPCHK(c, pack(c->pf_h, dm, dm, w.ln2_g, d.norm == 0 ? w.ln2_b : nullptr, d.norm));
    if (swiglu) HIPCHK(c, gemm(c->pf_xp, P.fin, dm, F, F, 0, true, bias ? w.b_in : nullptr, nullptr, nullptr, nullptr, nullptr, F, 0, c->pf_xf));
    else HIPCHK(c, gemm(c->pf_xp, P.fin, dm, F, 0, 0, false, bias ? w.b_in : nullptr, nullptr, nullptr, nullptr, nullptr, F, d.act == 0 ? 1 : 2, c->pf_xf));
    HIPCHK(c, gemm(c->pf_xf, P.fout, F, dm, 0, 0, false, bias ? w.b_out : nullptr, nullptr, nullptr, c->pf_h, c->pf_h, dm, 0));
  }
  return PPD_OK;
}

int env_int(const char* name, int dflt) {
  const char* v = getenv(name);
  if (!v || !*v) return dflt;
  int x = atoi(v);
  return x > 0 ? x : dflt;
}

}  // namespace

namespace ppd {
void set_global_hip_error(int e) { g_create_hip_error = e; }
}  // namespace ppd

extern "C" {

int ppd_create(const ppd_model_dims* dims, const ppd_weights* w, int k, int exit_layer, void* hip_stream,
               ppd_ctx** out) {
  if (!dims || !w || !out) return PPD_EINVAL;
  const ppd_model_dims& d = *dims;
  if (d.n_layers < 2 || d.d_model < 8 || d.d_model % 8 || d.d_ff < 8 || d.d_ff % 8 || d.vocab < 1 || d.max_ctx < 2)
    return PPD_EINVAL;
  if ((d.head_dim != 64 && d.head_dim != 128) || (int64_t)d.n_heads * d.head_dim != d.d_model) return PPD_EINVAL;
  if (d.norm < 0 || d.norm > 1 || d.act < 0 || d.act > 2 || d.pos < 0 || d.pos > 1 || d.wdtype < 0 || d.wdtype > 1)
    return PPD_EINVAL;
  if (k < 1 || k > PPD_MAX_K || k > d.vocab) return PPD_EINVAL;
  if (2 * exit_layer < d.n_layers || exit_layer > d.n_layers - 1) return PPD_EINVAL;   // Theorem 4.1: dbar >= d/2
  {
    // the kernels address one weight matrix (as launched: Q|K|V together, gate|up together) with 32-bit byte offsets
    const int64_t esz = d.wdtype == 0 ? 4 : 2;
    auto padded = [esz](int64_t rows, int64_t cols) { return ((rows + 15) / 16 * 16) * ((cols + 31) / 32 * 32) * esz; };
    const int64_t lim = (int64_t)1 << 32, dm = d.d_model, F = d.d_ff;
    if (padded(3 * dm, dm) >= lim || padded((d.act == 2 ? 2 : 1) * F, dm) >= lim || padded(dm, F) >= lim || padded(d.vocab, dm) >= lim)
      return PPD_ELIMIT;
  }
  if (!w->tok_emb || !w->lm_head || !w->lnf_g || (d.pos == 0 && !w->pos_emb) || (d.norm == 0 && !w->lnf_b))
    return PPD_EINVAL;
  if (!w->ln1_g || !w->wq || !w->wk || !w->wv || !w->wo || !w->ln2_g || !w->w_in || !w->w_out) return PPD_EINVAL;
  if (d.act == 2 && !w->w_up) return PPD_EINVAL;
  if (d.norm == 0 && (!w->ln1_b || !w->ln2_b)) return PPD_EINVAL;
  if (d.has_bias && (!w->bq || !w->bk || !w->bv || !w->bo || !w->b_in || !w->b_out)) return PPD_EINVAL;
  for (int l = 0; l < d.n_layers; ++l) {
    if (!w->ln1_g[l] || !w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->ln2_g[l] || !w->w_in[l] || !w->w_out[l])
      return PPD_EINVAL;
    if (d.act == 2 && !w->w_up[l]) return PPD_EINVAL;
    if (d.norm == 0 && (!w->ln1_b[l] || !w->ln2_b[l])) return PPD_EINVAL;
    if (d.has_bias && (!w->bq[l] || !w->bk[l] || !w->bv[l] || !w->bo[l] || !w->b_in[l] || !w->b_out[l])) return PPD_EINVAL;
  }
  ppd_ctx* c = new (std::nothrow) ppd_ctx();
  if (!c) return PPD_ENOMEM;
  c->d = d; c->k = k; c->dbar = exit_layer; c->nb = d.n_layers - exit_layer;
  c->user_stream = (hipStream_t)hip_stream;
  c->dev_pos_pending = -1;
  c->wbytes = d.wdtype == 0 ? 4 : 2;
  c->tok_emb = w->tok_emb; c->pos_emb = w->pos_emb; c->lnf_g = w->lnf_g; c->lnf_b = w->lnf_b;
  c->lm_head = w->lm_head; c->early_head = w->early_head;
  c->L.resize(d.n_layers);
  for (int l = 0; l < d.n_layers; ++l) {
    LayerW& x = c->L[l];
    x.ln1_g = w->ln1_g[l]; x.ln1_b = w->ln1_b ? w->ln1_b[l] : nullptr;
    x.wq = w->wq[l]; x.wk = w->wk[l]; x.wv = w->wv[l]; x.wo = w->wo[l];
    x.bq = w->bq ? w->bq[l] : nullptr; x.bk = w->bk ? w->bk[l] : nullptr;
    x.bv = w->bv ? w->bv[l] : nullptr; x.bo = w->bo ? w->bo[l] : nullptr;
    x.ln2_g = w->ln2_g[l]; x.ln2_b = w->ln2_b ? w->ln2_b[l] : nullptr;
    x.w_in = w->w_in[l]; x.w_up = w->w_up ? w->w_up[l] : nullptr; x.w_out = w->w_out[l];
    x.b_in = w->b_in ? w->b_in[l] : nullptr; x.b_out = w->b_out ? w->b_out[l] : nullptr;
  }
  c->nchunk_max = (d.max_ctx + ATT_CHUNK - 1) / ATT_CHUNK;
  c->n_ctx = -1;
  c->use_graphs = env_int("PPD_GRAPHS", 1) != 2;      // PPD_GRAPHS=2 switches graph replay off
  {
    const int cap = d.wdtype == 1 ? PREFILL_CHUNK : PREFILL_CHUNK_FP32;
    c->prefill_chunk = env_int("PPD_PREFILL_CHUNK", cap);
    if (c->prefill_chunk > cap) c->prefill_chunk = cap;
    // the compute-bound pass takes prompts of bf16 models unless the row-chunk path is asked for (PPD_PREFILL_CHUNK
    // set, or PPD_PREFILL_TILED=2)
    c->prefill_tiled = d.wdtype == 1 && !getenv("PPD_PREFILL_CHUNK") && env_int("PPD_PREFILL_TILED", 1) != 2;
  }
  c->gmax1 = 512;
  c->gmax2 = 256;
  // head GEMM: as many workgroups as a plain GEMM, more if a workgroup would otherwise
  // produce over HEAD_MAX_ROWS logits
  {
    c->head_grid = head_grid_valu(d.vocab, c->gmax1);
  }
  const size_t dm = d.d_model, R = 1 + k;
  const size_t RB = R > PREFILL_CHUNK ? R : PREFILL_CHUNK;   // activation rows: a round's 1 + k, or a prompt chunk
  hipError_t e = hipSuccess;
  auto alloc = [&](void** p, size_t bytes) { if (e == hipSuccess) e = hipMalloc(p, bytes); };
  alloc((void**)&c->Kc, (size_t)d.n_layers * cache_layer_bytes(c));
  alloc((void**)&c->Vc, (size_t)d.n_layers * cache_layer_bytes(c));
  alloc((void**)&c->tailK, (size_t)c->nb * k * dm * c->kvbytes);
  alloc((void**)&c->tailV, (size_t)c->nb * k * dm * c->kvbytes);
  alloc((void**)&c->h, RB * dm * sizeof(float));
  alloc((void**)&c->qkv, RB * 3 * dm * sizeof(float));
  alloc((void**)&c->att, RB * dm * sizeof(float));
  alloc((void**)&c->xn, RB * dm * sizeof(float));
  alloc((void**)&c->ffn, RB * (size_t)d.d_ff * sizeof(float));
  alloc((void**)&c->part, RB * d.n_heads * (size_t)c->nchunk_max * (d.head_dim + 2) * sizeof(float));
  alloc((void**)&c->logits, R * d.vocab * sizeof(float));
  alloc((void**)&c->early_spec, (size_t)2 * d.vocab * sizeof(float));
  c->samp_npad = (d.vocab + SAMP_THREADS * SAMP_MEMU - 1) / (SAMP_THREADS * SAMP_MEMU) * (SAMP_THREADS * SAMP_MEMU);
  alloc((void**)&c->samp_w, (size_t)c->samp_npad * sizeof(double));
  alloc((void**)&c->samp_keys, (size_t)c->samp_npad * sizeof(uint32_t));
  alloc((void**)&c->early_logits, (size_t)d.vocab * sizeof(float));
  const size_t pk_slots = (size_t)(c->head_grid > (d.vocab + 255) / 256 ? c->head_grid : (d.vocab + 255) / 256) + 1024;   // room for either head grid
  c->pk_slots = pk_slots;
  alloc((void**)&c->pk_val, R * pk_slots * MAXM * sizeof(float));
  alloc((void**)&c->pk_idx, R * pk_slots * MAXM * sizeof(int32_t));
  alloc((void**)&c->ds, sizeof(DevState));
  alloc((void**)&c->prompt_dev, (size_t)d.max_ctx * sizeof(int32_t));
  if (d.pos == 1) alloc((void**)&c->rope, (size_t)d.max_ctx * (d.head_dim / 2) * sizeof(float2));
  if (e == hipSuccess) e = hipHostMalloc((void**)&c->host_result, (2 + MAXM + 1) * sizeof(int32_t), hipHostMallocMapped);
  if (e == hipSuccess) memset(c->host_result, 0, (2 + MAXM + 1) * sizeof(int32_t));
  if (e == hipSuccess) e = hipHostGetDevicePointer((void**)&c->host_result_dev, c->host_result, 0);
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->stream, hipStreamNonBlocking);
  c->cur = c->stream;
  if (e == hipSuccess) e = hipEventCreateWithFlags(&c->join_ev, hipEventDisableTiming);
  if (e == hipSuccess && d.pos == 1) {
    // (cos, sin) of pos * theta^(-2i/hd), evaluated in double on the host
    const int half = d.head_dim / 2;
    std::vector<float2> tab((size_t)d.max_ctx * half);
    for (int p = 0; p < d.max_ctx; ++p)
      for (int i = 0; i < half; ++i) {
        double ang = (double)p * pow((double)d.rope_theta, -2.0 * i / d.head_dim);
        tab[(size_t)p * half + i] = make_float2((float)cos(ang), (float)sin(ang));
      }
    e = hipMemcpy(c->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice);
  }
  if (e == hipSuccess) e = hipMemset(c->ds, 0, sizeof(DevState));
  // the attention MFMAs read whole 16-position blocks: positions not yet written must hold finite numbers
  if (e == hipSuccess) e = hipMemset(c->Kc, 0, (size_t)d.n_layers * cache_layer_bytes(c));
  if (e == hipSuccess) e = hipMemset(c->Vc, 0, (size_t)d.n_layers * cache_layer_bytes(c));
  c->mfma = d.wdtype == 1;
  if (e == hipSuccess && c->mfma) {
    // repack every linear weight into MFMA blocks (owned copies), on the context's stream and after whatever
    // the caller has queued on its own stream so far (an asynchronous upload of the weights)
    e = hipEventRecord(c->join_ev, c->user_stream);
    if (e == hipSuccess) e = hipStreamWaitEvent(c->stream, c->join_ev, 0);
    auto repack = [&](const void* s0, const void* s1, const void* s2, int n0, int n1, int n2, int K, bool paired, void** out) {
      if (e != hipSuccess) return;
      RepackArgs r; memset(&r, 0, sizeof r);
      r.src[0] = (const uint16_t*)s0; r.src[1] = (const uint16_t*)s1; r.src[2] = (const uint16_t*)s2;
      r.nrows[0] = n0; r.nrows[1] = n1; r.nrows[2] = n2; r.K = K; r.KT = (K + 31) / 32; r.paired = paired ? 1 : 0;
      const int rows = paired ? n0 : n0 + n1 + n2;
      r.NT = paired ? (rows + 7) / 8 : (rows + 15) / 16;
      void* dst = nullptr;
      e = hipMalloc(&dst, (size_t)r.NT * r.KT * 1024);
      if (e != hipSuccess) return;
      c->owned.push_back(dst);
      r.dst = (uint16_t*)dst;
      hipLaunchKernelGGL(repack_kernel, dim3((unsigned)(r.NT * r.KT)), dim3(64), 0, c->stream, r);
      e = hipGetLastError();
      *out = dst;
    };
    c->LP.resize(d.n_layers);
    for (int l = 0; l < d.n_layers; ++l) {
      const LayerW& x = c->L[l];
      repack(x.wq, x.wk, x.wv, (int)dm, (int)dm, (int)dm, (int)dm, false, &c->LP[l].qkv);
      repack(x.wo, nullptr, nullptr, (int)dm, 0, 0, (int)dm, false, &c->LP[l].o);
      if (d.act == 2) repack(x.w_in, x.w_up, nullptr, d.d_ff, d.d_ff, 0, (int)dm, true, &c->LP[l].fin);
      else repack(x.w_in, nullptr, nullptr, d.d_ff, 0, 0, (int)dm, false, &c->LP[l].fin);
      repack(x.w_out, nullptr, nullptr, (int)dm, 0, 0, d.d_ff, false, &c->LP[l].fout);
    }
    repack(c->lm_head, nullptr, nullptr, d.vocab, 0, 0, (int)dm, false, &c->head_p);
    if (c->early_head) repack(c->early_head, nullptr, nullptr, d.vocab, 0, 0, (int)dm, false, &c->early_p);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_mfma_kernel<true, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)MG_LDS_MAX);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_mfma_kernel<false, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)MG_LDS_MAX);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_mfma_kernel<false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)MG_LDS_MAX);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_mfma_kernel<true, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)MG_LDS_MAX);
    // head launches: the same balanced grid as any other GEMM; a workgroup keeps at most
    // HEAD_MAX_ROWS logits = 16 tiles
    c->mg_passes_min = env_int("PPD_MGPASSES", 1);
    if (c->mg_passes_min < 1 || c->mg_passes_min > 8) c->mg_passes_min = 1;
    const int NTh = (d.vocab + 15) / 16;
    int th = (NTh + 255) / 256;
    c->head_grid = (NTh + th - 1) / th;
    while ((NTh + c->head_grid - 1) / c->head_grid > HEAD_MAX_ROWS / 16) ++c->head_grid;
    if ((size_t)c->head_grid > pk_slots) e = hipErrorInvalidValue;
    // speculative early prediction when the candidates end a round at the exit layer, the early head is the LM
    // head, and the 1 + k rows of the widened final head fit one launch (PPD_SPEC=2 switches it off)
    {
      const int KT = ((int)dm + 31) / 32;
      int xrow = mg_xrow(KT);
      if (xrow < HEAD_MAX_ROWS * (int)sizeof(float)) xrow = HEAD_MAX_ROWS * (int)sizeof(float);
      int ob, op, ox;
      const size_t need = (size_t)mg_lds_layout((int)dm, 1 + k, d.norm, (NTh + c->head_grid - 1) / c->head_grid, xrow, ob, op, ox);
      c->spec = 2 * c->dbar == d.n_layers && !c->early_head && need <= MG_LDS_MAX && env_int("PPD_SPEC", 1) != 2;
    }
  }
  // (the fills and copies above went to the null stream, which the context's own stream does not wait for)
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    g_create_hip_error = (int)e;
    (void)hipGetLastError();
    free_all(c);
    int rc = (e == hipErrorOutOfMemory) ? PPD_ENOMEM : PPD_EHIP;
    delete c;
    return rc;
  }
  *out = c;
  return PPD_OK;
}

int ppd_reset(ppd_ctx* c) {
  if (!c) return PPD_EINVAL;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  c->n_ctx = -1; c->matched = 0; c->finished = 0; c->have_early = 0; c->dev_pos_pending = -1;
  memset(&c->st, 0, sizeof c->st);
  return PPD_OK;
}

int ppd_prefill(ppd_ctx* c, const int32_t* prompt, int n_prompt) {
  if (!c || !prompt || n_prompt < 1) return PPD_EINVAL;
  if (n_prompt > c->d.max_ctx) return PPD_ECTX;
  for (int i = 0; i < n_prompt; ++i)
    if (prompt[i] < 0 || prompt[i] >= c->d.vocab) return PPD_EINVAL;
  int rc = ppd_reset(c);
  if (rc) return rc;
  HIPCHK(c, hipEventRecord(c->join_ev, c->user_stream));
  HIPCHK(c, hipStreamWaitEvent(c->stream, c->join_ev, 0));
  HIPCHK(c, hipMemcpyAsync(c->prompt_dev, prompt, (size_t)n_prompt * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));   // prompt is pageable host memory of the caller
  int prof = c->prof; c->prof = 0;
  // positions 0 .. n_prompt-2 in chunks of consecutive positions: every row's arithmetic is that of a
  // token-by-token pass (PPD_PREFILL_CHUNK=1 runs exactly that), the weights are streamed once per chunk
  const int chunk = c->prefill_chunk;
  const bool tiled = c->prefill_tiled && n_prompt - 1 >= PREFILL_TILED_MIN;
  if (tiled) rc = prefill_tiled(c, n_prompt - 1);
  for (int i = 0; !tiled && i + 1 < n_prompt && !rc; i += chunk) {
    const int m = n_prompt - 1 - i < chunk ? n_prompt - 1 - i : chunk;
    rc = set_state(c, i, -1);
    if (!rc) {
      EmbedArgs ea = embed_args(c, c->prompt_dev + i, m, 0, 0);
      ea.pos_step = 1;
      dim3 grid((c->d.d_model + 255) / 256, m);
      if (c->wbytes == 4) hipLaunchKernelGGL(embed_kernel<float>, grid, dim3(256), 0, c->cur, ea);
      else hipLaunchKernelGGL(embed_kernel<bf16_t>, grid, dim3(256), 0, c->cur, ea);
      if (hipGetLastError() != hipSuccess) rc = PPD_EHIP;
    }
    for (int l = 0; l < c->d.n_layers && !rc; ++l) {
      RowGroup g{l, m, 0, 0, false};
      g.chunk = m > 1;
      rc = run_layer(c, 1, &g, i + m - 1);
    }
  }
  c->prof = prof;
  if (rc) return rc;
  if ((rc = set_state(c, n_prompt - 1, prompt[n_prompt - 1]))) return rc;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  c->n_ctx = n_prompt - 1; c->matched = 0; c->finished = 0;
  return PPD_OK;
}

int ppd_step(ppd_ctx* c, int32_t* out_tokens, int max_out, ppd_step_info* info) {
  if (!c || !out_tokens || max_out < 1) return PPD_EINVAL;
  if (c->n_ctx < 0) return PPD_ESTATE;
  if (c->finished) return 0;
  const int pos = c->n_ctx;
  if (pos + 1 >= c->d.max_ctx) return PPD_ECTX;   // the candidates sit at position pos+1
  const int kind = c->matched ? (c->spec ? 3 : 1) : 0;
  int rc = run_round(c, kind, pos);
  if (rc) return rc;
  account_round(c, kind, pos);
  const int tok = c->host_result[0], midx = c->host_result[1];
  if (kind == 0) c->st.runs += 1;
  c->st.main_layer_rows += (uint64_t)(c->dbar - (kind == 0 ? 0 : c->nb)) + c->nb;
  c->st.branch_layer_rows += (uint64_t)c->k * c->nb;
  c->n_ctx = pos + 1;
  c->matched = midx >= 0;
  c->have_early = 1;
  c->last_kind = kind;
  c->st.rounds += 1;
  c->st.matches += c->matched;
  if (tok == c->d.eos_id) c->finished = 1;
  out_tokens[0] = tok;
  if (info) {
    info->token = tok; info->matched = c->matched; info->match_idx = midx;
    for (int i = 0; i < PPD_MAX_K; ++i) info->cand[i] = i < c->k ? c->host_result[2 + i] : -1;   // (pinned memory, written by the round)
  }
  return 1;
}

int plain_greedy_step(ppd_ctx* c, int32_t* out_token) {
  if (!c || !out_token) return PPD_EINVAL;
  if (c->n_ctx < 0) return PPD_ESTATE;
  if (c->finished) return 0;
  const int pos = c->n_ctx;
  if (pos >= c->d.max_ctx) return PPD_ECTX;
  int rc = run_round(c, 2, pos);
  if (rc) return rc;
  account_round(c, 2, pos);
  c->n_ctx = pos + 1;
  c->matched = 0;
  c->last_kind = 2;
  c->st.plain_steps += 1;
  if (c->host_result[0] == c->d.eos_id) c->finished = 1;
  *out_token = c->host_result[0];
  return 1;
}

int ppd_get_logits(ppd_ctx* c, float* host_logits) {
  if (!c || !host_logits) return PPD_EINVAL;
  if (c->n_ctx < 0) return PPD_ESTATE;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(host_logits, c->logits, (size_t)c->d.vocab * sizeof(float), hipMemcpyDeviceToHost));
  return PPD_OK;
}

int ppd_get_early_logits(ppd_ctx* c, float* host_logits) {
  if (!c || !host_logits) return PPD_EINVAL;
  if (c->n_ctx < 0 || !c->have_early) return PPD_ESTATE;
  // a round that started from a speculative prediction has its early logits in the half of early_spec that
  // its position's parity selects (the position of the last round's main token is n_ctx - 1)
  const float* src = c->last_kind == 3 ? c->early_spec + (size_t)((c->n_ctx - 1) & 1) * c->d.vocab : c->early_logits;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(host_logits, src, (size_t)c->d.vocab * sizeof(float), hipMemcpyDeviceToHost));
  return PPD_OK;
}

int ppd_get_stats(const ppd_ctx* c, ppd_stats* out) {
  if (!c || !out) return PPD_EINVAL;
  *out = c->st;
  return PPD_OK;
}

int ppd_set_profiling(ppd_ctx* c, int on) {
  if (!c) return PPD_EINVAL;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  c->prof = on < 0 ? 0 : (on > 2 ? 2 : on);
  c->ev_used = 0;
  if (on) { memset(c->kc_ms, 0, sizeof c->kc_ms); memset(c->kc_n, 0, sizeof c->kc_n); }
  return PPD_OK;
}

int ppd_set_sampling(ppd_ctx* c, int mode, int top_k, double top_p, uint64_t seed) {
  if (!c || mode < 0 || mode > 2) return PPD_EINVAL;
  if (mode == 1 && top_k < 1) return PPD_EINVAL;
  if (mode == 2 && !(top_p > 0.0 && top_p <= 1.0)) return PPD_EINVAL;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  c->samp_mode = mode; c->samp_k = top_k; c->samp_p = top_p; c->samp_seed = seed;
  // the captured rounds hold the old rule
  for (int i = 0; i < 4; ++i)
    if (c->graph[i]) { HIPCHK(c, hipGraphExecDestroy(c->graph[i])); c->graph[i] = nullptr; }
  return PPD_OK;
}

int ppd_set_graphs(ppd_ctx* c, int on) {
  if (!c) return PPD_EINVAL;
  c->use_graphs = on ? 1 : 0;
  return PPD_OK;
}

int ppd_get_kernel_time(ppd_ctx* c, int kernel_class, int groups, double* ms_total, uint64_t* launches) {
  if (!c || kernel_class < 0 || kernel_class >= PPD_KC_COUNT || groups < 1 || groups > 2 || !ms_total || !launches)
    return PPD_EINVAL;
  *ms_total = c->kc_ms[kernel_class + (groups - 1) * PPD_KC_COUNT];
  *launches = c->kc_n[kernel_class + (groups - 1) * PPD_KC_COUNT];
  return PPD_OK;
}

int ppd_time_ffn_in(ppd_ctx* c, int reps, int groups, double* ms_per_launch) {
  if (!c || reps < 1 || groups < 1 || groups > 2 || !ms_per_launch) return PPD_EINVAL;
  if (c->n_ctx < 0) return PPD_ESTATE;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  hipEvent_t e0 = nullptr, e1 = nullptr;
  HIPCHK(c, hipEventCreate(&e0));
  hipError_t e = hipEventCreate(&e1);
  int rc = PPD_OK;
  const int saved_prof = c->prof;
  c->prof = 0;
  c->cur = c->stream;
  if (e == hipSuccess) {
    // one untimed launch per distinct layer first would warm nothing that matters (the weights do not fit
    // any cache); one warm-up launch for the code, then the timed burst
    // groups == 2: the launch of a pipelined step (main row at one layer, the k candidate rows at another)
    const int L = c->d.n_layers;
    RowGroup g0[2] = {{0, 1, 0, 0, false}, {1 % L, c->k, 1, 1, true}};
    rc = run_layer(c, groups, g0, 0, 4);
    if (!rc) e = hipEventRecord(e0, c->stream);
    for (int i = 0; i < reps && !rc && e == hipSuccess; ++i) {
      RowGroup g[2] = {{(2 + 2 * i) % L, 1, 0, 0, false}, {(3 + 2 * i) % L, c->k, 1, 1, true}};
      rc = run_layer(c, groups, g, 0, 4);
    }
    if (!rc && e == hipSuccess) e = hipEventRecord(e1, c->stream);
    if (!rc && e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (!rc && e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (!rc && e == hipSuccess) *ms_per_launch = (double)ms / reps;
  }
  c->prof = saved_prof;
  c->n_ctx = -1;                 // the activation rows were overwritten
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (rc) return rc;
  HIPCHK(c, e);
  return PPD_OK;
}

}  // extern "C"

namespace {
// streaming-read probe, second pattern: every workgroup walks one contiguous part of the buffer, 32 KiB per step
// (grid-stride walks, where neighbouring workgroups interleave 4 KiB pieces, read about a tenth slower on this part)
__global__ __launch_bounds__(256) void stream_read_chunk_kernel(const u32x4* p, size_t n16, uint32_t* sink) {
  constexpr int U = 8;
  const size_t per = n16 / gridDim.x;                      // (the tail past per * gridDim.x is not read: at most 16 B x grid)
  const u32x4* q = p + (size_t)blockIdx.x * per;
  u32x4 acc = {0u, 0u, 0u, 0u};
  size_t i = threadIdx.x;
  for (; i + (U - 1) * 256 < per; i += U * 256) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = ld_stream(q + i + u * 256);
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= v[u];
  }
  for (; i < per; i += 256) acc ^= ld_stream(q + i);
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) *sink = acc.x;   // keeps the loads alive; practically never taken
}
}  // namespace

extern "C" {

int ppd_stream_read_probe(const void* dev_buf, uint64_t bytes, int iters, double* gbps) {
  if (!dev_buf || !gbps || bytes == 0 || (bytes & 15) || iters < 1) return PPD_EINVAL;
  hipStream_t st = nullptr; hipEvent_t e0 = nullptr, e1 = nullptr; uint32_t* sink = nullptr;
  hipError_t e = hipStreamCreateWithFlags(&st, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  if (e == hipSuccess) e = hipMalloc((void**)&sink, sizeof(uint32_t));
  // the best of a few launch shapes (workgroups x loads in flight per thread): what the GPU can stream
  double best = 0.0;
  if (e == hipSuccess) {
    const size_t n16 = bytes / 16;
    const int grids[] = {1024, 2048, 4096, 8192, 256, 512, 1024};   // the last three: contiguous parts per workgroup
    for (int gi = 0; gi < 7 && e == hipSuccess; ++gi)
      for (int u8 = 0; u8 < 2 && e == hipSuccess; ++u8) {
        if (gi >= 4 && u8) continue;
        const dim3 grid(grids[gi]), block(256);
        auto go = [&]() {
          if (gi >= 4) hipLaunchKernelGGL(stream_read_chunk_kernel, grid, block, 0, st, (const u32x4*)dev_buf, n16, sink);
          else if (u8) hipLaunchKernelGGL(stream_read_kernel<8>, grid, block, 0, st, (const u32x4*)dev_buf, n16, sink);
          else hipLaunchKernelGGL(stream_read_kernel<4>, grid, block, 0, st, (const u32x4*)dev_buf, n16, sink);
        };
        go();   // warm-up
        e = hipEventRecord(e0, st);
        for (int i = 0; i < iters && e == hipSuccess; ++i) { go(); e = hipGetLastError(); }
        if (e == hipSuccess) e = hipEventRecord(e1, st);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e == hipSuccess && ms > 0.f) {
          const double r = (double)bytes * iters / ((double)ms * 1e-3) / 1e9;
          if (r > best) best = r;
        }
      }
  }
  if (sink) (void)hipFree(sink);
  if (e1) (void)hipEventDestroy(e1);
  if (e0) (void)hipEventDestroy(e0);
  if (st) (void)hipStreamDestroy(st);
  if (e != hipSuccess) { g_create_hip_error = (int)e; (void)hipGetLastError(); return PPD_EHIP; }
  *gbps = best;
  return PPD_OK;
}

void ppd_destroy(ppd_ctx* c) {
  if (!c) return;
  if (c->stream) (void)hipStreamSynchronize(c->stream);
  free_all(c);
  delete c;
}

const char* ppd_strerror(int code) {
  switch (code) {
    case PPD_OK: return "ok";
    case PPD_EINVAL: return "invalid argument";
    case PPD_ENOMEM: return "out of memory";
    case PPD_ECTX: return "context window exhausted";
    case PPD_ESTATE: return "call out of order";
    case PPD_EHIP: return "HIP call failed";
    case PPD_ELIMIT: return "size beyond the fixed maximum of this entry point";
    default: return "unknown error";
  }
}

int ppd_last_hip_error(const ppd_ctx* c) { return c ? c->last_hip : g_create_hip_error; }

}  // extern "C"
