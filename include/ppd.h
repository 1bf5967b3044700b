/* libppd: Predictive Pipelined Decoding (PPD) on one MI355X (gfx950).
 *
 * The calls follow the paper's statement of the method (Sec. 3, Algorithm 1;
 * general exit layer: Appendix C, Algorithm 2).  Inputs of the method: number
 * of tokens l, number of decoder layers d, exit layer dbar >= d/2, number of
 * early candidates k, start token x_0.  Output: the token sequence of plain
 * greedy decoding, exactly.
 *
 * Where the paper runs k sub-processes on k extra compute units, this
 * library runs the k candidate tokens as k extra rows of the same kernel
 * launches on one GPU: during the parallel phase of a round, step j handles
 * the main token at layer dbar+j and the k candidates at layer j.
 *
 * Pointer kinds are stated per argument: HOST or DEVICE.  All functions
 * return 0 on success or a negative PPD_E* code.  A call that fails its
 * argument or state checks (PPD_EINVAL, PPD_ECTX, PPD_ESTATE) leaves the
 * context unchanged; after PPD_EHIP from ppd_prefill, ppd_step or
 * plain_greedy_step the sequence state is undefined and the next call must
 * be ppd_prefill (or ppd_destroy).  One context must be used by one thread
 * at a time.  No C++ exception crosses this boundary.
 */
#ifndef PPD_H
#define PPD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PPD_OK 0
#define PPD_EINVAL (-1) /* bad dims, k outside [1, PPD_MAX_K], exit layer outside [ceil(d/2), d-1], null pointer */
#define PPD_ENOMEM (-2) /* device or host allocation failed */
#define PPD_ECTX (-3)   /* context window exhausted */
#define PPD_ESTATE (-4) /* call out of order (e.g. step before prefill) */
#define PPD_EHIP (-5)   /* a HIP call failed; ppd_last_hip_error() tells which */
#define PPD_ELIMIT (-6) /* a size beyond the fixed maximum an entry point documents */

#define PPD_MAX_K 8

typedef struct ppd_ctx ppd_ctx; /* opaque */

/* Shape of the decoder-only transformer the rounds run on.  The paper treats
 * the transformer layer as a black box of equal cost per layer (Fig. 1,
 * Sec. 4.1); these fields select the block the benchmark configurations name. */
typedef struct {
  int32_t n_layers;  /* d */
  int32_t d_model;   /* multiple of 8 */
  int32_t n_heads;
  int32_t head_dim;  /* 64 or 128; n_heads * head_dim == d_model */
  int32_t d_ff;      /* multiple of 8 */
  int32_t vocab;
  int32_t max_ctx;   /* positions the KV cache (and the position table) holds */
  int32_t norm;      /* 0 LayerNorm with bias, 1 RMSNorm */
  int32_t act;       /* 0 GELU (erf form), 1 ReLU, 2 SwiGLU */
  int32_t pos;       /* 0 learned absolute position table, 1 RoPE (rotate-half pairs i, i+head_dim/2) */
  int32_t has_bias;  /* linear layers carry biases */
  int32_t wdtype;    /* 0 fp32, 1 bf16: type of every weight tensor (activations and the KV cache are fp32) */
  float norm_eps;
  float rope_theta;
  int32_t eos_id;    /* -1: never stop */
} ppd_model_dims;

/* DEVICE pointers to the weights, borrowed for the life of the context (the
 * caller keeps them alive and unchanged).  Linear weights are row-major
 * [out][in]; all tensors have type `wdtype` and 16-byte aligned rows.
 * The per-layer members are HOST arrays of n_layers DEVICE pointers.
 * Members a model does not have (biases, pos_emb, w_up, LayerNorm biases)
 * may be NULL. */
typedef struct {
  const void *tok_emb;  /* [vocab][d_model] */
  const void *pos_emb;  /* [max_ctx][d_model], pos == 0 only */
  const void *lnf_g, *lnf_b; /* final norm */
  const void *lm_head;  /* [vocab][d_model] */
  const void *early_head; /* [vocab][d_model] classifier for the early prediction, NULL: lm_head
                             (Sec. 4.3: classifier of the final layer reused, or one trained per layer) */
  const void *const *ln1_g, *const *ln1_b;
  const void *const *wq, *const *wk, *const *wv, *const *wo; /* [d_model][d_model] */
  const void *const *bq, *const *bk, *const *bv, *const *bo;
  const void *const *ln2_g, *const *ln2_b;
  const void *const *w_in;  /* [d_ff][d_model]; the gate matrix for SwiGLU */
  const void *const *w_up;  /* [d_ff][d_model], SwiGLU only */
  const void *const *w_out; /* [d_model][d_ff] */
  const void *const *b_in, *const *b_out;
} ppd_weights;

/* What one round did (Algorithm 2, one iteration of the while loop). */
typedef struct {
  int32_t token;     /* x_{t+1}: arg max of the final layer's logits, ties to the lowest id */
  int32_t matched;   /* 1 if one early candidate equals token: the next round resumes mid-stack */
  int32_t match_idx; /* index of that candidate in cand[], or -1 */
  int32_t cand[PPD_MAX_K]; /* early top-k ids, by (logit descending, id ascending); entries >= k are -1 */
} ppd_step_info;

/* Counters in the units of Sec. 4: one layer on one token = one unit. */
typedef struct {
  uint64_t rounds;            /* tokens emitted by ppd_step */
  uint64_t matches;           /* rounds with matched == 1 */
  uint64_t runs;              /* N of Sec. 4.1: rounds that started from layer 1 */
  uint64_t main_layer_rows;   /* layer executions of the main token: latency in time units */
  uint64_t branch_layer_rows; /* layer executions of candidate rows */
  uint64_t plain_steps;       /* tokens emitted by plain_greedy_step */
  uint64_t weight_bytes;      /* weight bytes the launched kernels had to stream */
  uint64_t kv_bytes;          /* KV-cache bytes the launched attention kernels had to read */
} ppd_stats;

/* Create a context.  Sec. 3 / Algorithm 2 inputs: d (dims->n_layers), dbar
 * (exit_layer, 1-based: the early prediction reads the output of that layer,
 * ceil(d/2) <= exit_layer <= d-1 as Theorem 4.1 requires dbar >= d/2), k.
 * dims, w: HOST structs, copied.  hip_stream: a hipStream_t (NULL = the
 * default stream), the caller's: the context runs on a stream of its own and
 * makes it wait, here and at every ppd_prefill, for what the caller has
 * queued on hip_stream until then.  The weights must be complete in device
 * memory once the work queued on hip_stream before this call has run: bf16
 * models are repacked here, once, into copies the context owns (same size;
 * linear weights changed afterwards are never seen), the remaining tensors
 * (embeddings, norm gains, biases; every tensor of an fp32 model) are read
 * again at every step and must not change.  Every call is synchronous: the
 * context's stream is idle on return.  The KV cache, the candidates' KV
 * tails and all scratch are allocated here (device memory, freed by
 * ppd_destroy).  *out receives the context (HOST).  PPD_ELIMIT for a model
 * one of whose matrices, as launched (Q|K|V together, gate|up together, the
 * LM head), reaches 4 GiB (rows padded to 16, columns to 32): the kernels
 * address a matrix with 32-bit byte offsets. */
int ppd_create(const ppd_model_dims *dims, const ppd_weights *w, int k, int exit_layer,
               void *hip_stream, ppd_ctx **out);

/* Forget the sequence: KV cache length 0, round state cleared, counters zeroed. */
int ppd_reset(ppd_ctx *ctx);

/* Feed a prompt (HOST int32 ids, n_prompt >= 1).  The algorithm starts from
 * one start token x_0; reading taken for prompts: positions 0..n_prompt-2 are
 * run through all d layers to fill the KV cache, the last prompt token
 * becomes x_0 with match = False.  Implies ppd_reset.  PPD_ECTX if
 * n_prompt > max_ctx; PPD_EINVAL for ids outside [0, vocab).
 * bf16 models with prompts of more than 32 tokens: all prompt rows go through
 * a layer at once (tiled MFMA GEMMs on rows split into two bf16 terms,
 * causal attention on the same operands): products exact in fp32 as in
 * decoding, other summation order, so the cache is close to, not
 * bit-identical with, a token-by-token pass (every decode step after it is
 * the same arithmetic either way).  Otherwise, or with PPD_PREFILL_TILED=2 /
 * PPD_PREFILL_CHUNK=n in the environment at ppd_create, the prompt goes
 * through the decode kernels in chunks of consecutive positions (16 for
 * bf16 weights, 8 for fp32; n lowers it): one pass over the weights per
 * chunk, every row's arithmetic that of a one-token pass, the cache equal to
 * a token-by-token prefill bit for bit (n = 1 runs exactly that).
 * Buffers of the first kind are allocated at the first such prompt and grow
 * with the longest prompt seen (PPD_ENOMEM / PPD_EHIP if that fails). */
int ppd_prefill(ppd_ctx *ctx, const int32_t *prompt, int n_prompt);

/* One round of Algorithm 2: main token to the exit layer (from layer 1, or
 * from layer d-dbar+1 after a match), early top-k, the parallel phase of
 * d-dbar pipelined steps, final arg max, verification, adoption or discard.
 * Writes the emitted token to out_tokens[0] (HOST, max_out >= 1) and returns
 * the number of tokens written: 1, or 0 once the previous token was EOS.
 * info (HOST, nullable) receives the round's record.  PPD_ECTX when position
 * t+1 would not fit in max_ctx.  Synchronous: the round's record (token, match, candidates) is complete on
 * return -- the call waits for the word the round's last kernel writes to pinned host memory after them; that
 * kernel may still be retiring, and every later call on the context is ordered after it.
 * When exit_layer = d/2 and w->early_head is NULL (bf16 weights), the candidate
 * rows finish a round at the exit layer, so the round's final LM-head pass also
 * covers them; after a match the matching row's top-k are the next round's
 * candidates and that round runs no early head of its own (same candidates,
 * logits and tokens; one LM-head pass less).  PPD_SPEC=2 in the environment
 * at ppd_create switches this off. */
int ppd_step(ppd_ctx *ctx, int32_t *out_tokens, int max_out, ppd_step_info *info);

/* Conventional decoding of one token (Sec. 4.2: d time units per token): all
 * d layers on the pending token, final arg max.  Same kernels, one row.
 * Writes the token to *out_token (HOST); returns 1, or 0 after EOS.  May be
 * mixed with ppd_step on one context: a pending match is dropped. */
int plain_greedy_step(ppd_ctx *ctx, int32_t *out_token);

/* Rule for the final prediction (Appendix B: sampling-based decoding uses PPD
 * unchanged except that the final prediction is drawn by top-k or top-p
 * sampling instead of the arg max).  mode 0: arg max (default); 1: top-k
 * sampling, the top_k most probable tokens kept; 2: top-p sampling, the
 * shortest prefix of the ranking by probability whose mass reaches top_p kept.
 * The token is drawn by inversion from the renormalised kept softmax of the
 * final fp32 logits, in fp64, tokens ranked by (logit descending, id
 * ascending); the uniform number of a step is the top 24 bits of the first
 * word of Philox-4x32-10 with key = seed and counter = sequence position of
 * the token being chosen, so ppd_step and plain_greedy_step draw the same
 * tokens.  Applies to both kinds of step from the next call on.  PPD_EINVAL
 * for an unknown mode, top_k < 1 (mode 1), top_p outside (0, 1] (mode 2). */
int ppd_set_sampling(ppd_ctx *ctx, int mode, int top_k, double top_p, uint64_t seed);

/* Copy the counters (HOST). */
int ppd_get_stats(const ppd_ctx *ctx, ppd_stats *out);

/* Rounds are replayed as captured HIP graphs (one per round shape) unless profiling is on;
 * on = 0 issues every launch eagerly instead.  Results are identical either way. */
int ppd_set_graphs(ppd_ctx *ctx, int on);

/* The early prediction of Sec. 3 on its own, outside any context: logits = head . Norm(h) for one
 * intermediate hidden row (the LM classifier applied to the exit layer's state; Sec. 4.3: the final layer's
 * classifier, or one trained for that layer), and their top-k by (logit descending, id ascending) -- the
 * k candidate tokens Algorithm 2 hands to the sub-processes.  For callers that run the layers themselves.
 * All tensors DEVICE, borrowed for the call: h float[d_model] (16-byte aligned); norm_g, norm_b (norm_b only for
 * norm == 0, LayerNorm) and head ([vocab][d_model] row-major, rows 16-byte aligned) of type wdtype (0 fp32,
 * 1 bf16); d_model a multiple of 8; 1 <= k <= min(PPD_MAX_K, vocab).  Outputs, DEVICE: ids_out int32[k];
 * vals_out float[k] (their logits) or NULL; logits_out float[vocab] or NULL.  Work is queued on hip_stream (a
 * hipStream_t, NULL = the default stream).  This call allocates its scratch (the logits when logits_out is NULL,
 * one top-k list per workgroup) with hipMalloc, waits for hip_stream and frees it: synchronous, outputs complete
 * on return.  PPD_EINVAL for bad arguments, PPD_ENOMEM / PPD_EHIP (ppd_last_hip_error(NULL)) otherwise. */
int ppd_early_topk(int d_model, int vocab, int norm, float norm_eps, int wdtype, const void *norm_g,
                   const void *norm_b, const void *head, const float *h, int k, int32_t *ids_out,
                   float *vals_out, float *logits_out, void *hip_stream);

/* ppd_early_topk for callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): same arguments, same kernels, same results, but the scratch is a fixed array inside the
 * library's code object (288 KiB per GPU, held until the process ends) and the call neither allocates nor frees
 * nor waits: it only queues its two launches on hip_stream, and the outputs are complete once that work has run.
 * Limits: vocab <= 65536 (PPD_ELIMIT beyond; d_model is not limited).  The first call on a GPU looks up that
 * GPU's copy of the array (make it outside any capture).  All calls on one GPU share the array and its contents
 * survive from call to call (nothing in it needs clearing: every entry read is written first); calls whose work
 * overlaps in time on one GPU -- different streams, or threads -- race on it: keep them on one stream or order
 * them yourself. */
int ppd_early_topk_noalloc(int d_model, int vocab, int norm, float norm_eps, int wdtype, const void *norm_g,
                           const void *norm_b, const void *head, const float *h, int k, int32_t *ids_out,
                           float *vals_out, float *logits_out, void *hip_stream);

void ppd_destroy(ppd_ctx *ctx);

const char *ppd_strerror(int code);
/* hipError_t value of the last failing HIP call on this context (0 if none); with ctx == NULL, of the
 * last ppd_create that failed. */
int ppd_last_hip_error(const ppd_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* PPD_H */
