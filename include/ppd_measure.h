/* Measurement aids and test hooks of libppd: timing of the kernels as they run, the streaming rate of the GPU,
 * and read-back of logits for tests.  Not part of the method (ppd.h holds that); the benchmark, the counter
 * probe and the tests call these. */
#ifndef PPD_MEASURE_H
#define PPD_MEASURE_H
#include "ppd.h"
#ifdef __cplusplus
extern "C" {
#endif

/* Kernel classes for ppd_get_kernel_time(). */
enum {
  PPD_KC_EMBED = 0,
  PPD_KC_GEMM_QKV,   /* norm + Q,K,V projections */
  PPD_KC_ATTN,       /* RoPE, KV write, attention over prefix + own position */
  PPD_KC_ATTN_MERGE, /* merge of the position-chunk partials */
  PPD_KC_GEMM_O,     /* output projection + residual */
  PPD_KC_GEMM_FFN_IN,  /* norm + first FFN matrix (both matrices for SwiGLU) + activation */
  PPD_KC_GEMM_FFN_OUT, /* second FFN matrix + residual */
  PPD_KC_HEAD,       /* final norm + LM head */
  PPD_KC_SELECT,     /* merge of the head's block top-k; early: candidates + their embedding rows;
                        final: arg max, verification, adoption of the matching candidate
                        (hidden row + KV tails -> cache) */
  PPD_KC_COMMIT,     /* unused (adoption runs inside PPD_KC_SELECT) */
  PPD_KC_PHASE,      /* not a kernel: one bracket around a whole phase of a round (groups = 1: the
                        main token alone up to the exit layer; groups = 2: the d-dbar pipelined steps) */
  PPD_KC_COUNT
};

/* Test hooks.  host_logits: HOST float[vocab].  Final-layer logits of the last
 * ppd_step / plain_greedy_step, and early-exit logits of the last ppd_step. */
int ppd_get_logits(ppd_ctx *ctx, float *host_logits);
int ppd_get_early_logits(ppd_ctx *ctx, float *host_logits);

/* Timing with HIP events on the context's streams.  level 2: every launch is bracketed by two
 * events; level 1: only the phases of a round are (class PPD_KC_PHASE), so the kernels run
 * back to back as in normal operation; level 0: off.  While on, rounds are issued eagerly
 * instead of replayed from graphs.  ppd_get_kernel_time returns, for one class and one launch
 * shape (groups = 1: one row group; groups = 2: a two-group launch, or for PPD_KC_PHASE the
 * whole parallel phase), the summed elapsed milliseconds and the number of brackets since
 * profiling was switched on (HOST outputs).  Prefill is never profiled. */
int ppd_set_profiling(ppd_ctx *ctx, int level);
int ppd_get_kernel_time(ppd_ctx *ctx, int kernel_class, int groups, double *ms_total, uint64_t *launches);

/* Measurement aid: launches the FFN-in GEMM (fused norm, first FFN matrix or the gate/up pair, activation)
 * reps times back to back between two HIP events on the context's stream, every launch on other layers' weights
 * than the one before, and reports the average milliseconds per launch (HOST output): the duration of the
 * kernel that bench.py prices against the HBM roofline, as it runs in a chain, without the event pair that
 * ppd_set_profiling(2) puts around every single launch.  groups = 2: the launch shape of a pipelined step (the
 * main row on one layer's matrices and the k candidate rows on another's: two weight streams per launch);
 * groups = 1: the main row alone (solo phase, plain steps).  Needs a prefilled context; overwrites the
 * activation rows, so the sequence state is gone afterwards (PPD_ESTATE until the next ppd_prefill). */
int ppd_time_ffn_in(ppd_ctx *ctx, int reps, int groups, double *ms_per_launch);

/* Measurement aid (not part of the method): read `bytes` of DEVICE memory at dev_buf `iters` times with a
 * kernel that does nothing but non-temporal 16-byte loads (a few launch shapes and two walks -- grid-stride, and one
 * contiguous part per workgroup --, the best counts), and report the rate in GB/s (HOST
 * output): the streaming rate this GPU reaches, next to which the decode kernels' rates are read.
 * bytes must be a positive multiple of 16; the buffer is only read.  Runs on its own stream, synchronous. */
int ppd_stream_read_probe(const void *dev_buf, uint64_t bytes, int iters, double *gbps);

#ifdef __cplusplus
}
#endif
#endif /* PPD_MEASURE_H */
