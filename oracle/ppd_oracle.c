/* CPU oracle for Predictive Pipelined Decoding (PPD).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * HIP library is checked against.  It shares no code with the HIP path and is
 * never on the product path: only the tests, the smoke check and the
 * benchmark's CPU-baseline leg may load it.
 *
 * What it computes
 *   - a decoder-only transformer forward in fp64 on the caller's weight bytes
 *     (fp32, or bf16 widened exactly).  The paper treats the transformer
 *     layer as a black box (Fig. 1, "TL"); its definition here is the
 *     benchmark configuration's: pre-norm blocks, causal softmax attention,
 *     GELU / ReLU / SwiGLU feed-forward, learned positions or rotate-half RoPE.
 *   - plain greedy decoding (Sec. 1: each token comes from the final layer's
 *     hidden state; Sec. 4.2: d time units per token), with a KV cache, and a
 *     second, cache-free version that re-runs the whole sequence in matrix
 *     form at every step.
 *   - the PPD loop of the general algorithm (Appendix C, Algorithm 2; the
 *     d/2 case is Algorithm 1), executed sequentially in the algorithm's own
 *     order: main process to the exit layer, top-k early prediction, main
 *     process to the final layer, each sub-process through layers
 *     1..d-dbar on its candidate, verification and adoption.
 *   - the per-sequence counters of Sec. 4.2 (main-process layer executions =
 *     latency in time units, sub-process layer executions, number of runs N).
 *   - the sampling-based variants of Appendix B: the final prediction is drawn
 *     by top-k sampling or top-p (nucleus) sampling instead of the arg max;
 *     everything else of the loop is unchanged.  The random number of a step
 *     is a counter-based one (Philox-4x32-10, Salmon et al., SC 2011) of
 *     (seed, position of the token being chosen), so that decoding with and
 *     without PPD draw the same numbers.
 *
 * Readings where the paper is silent are listed next to the code that takes
 * them.  Parity pins: tests/test_oracle_*.py.
 *
 * Pin status: forward numerics are pinned sub-op by sub-op and end to end
 * against library routines (torch CPU fp64) and closed forms; the control
 * loop by the paper's exactness invariant and counter identities; the
 * generator by the known-answer vectors of its reference distribution, the
 * samplers by closed forms (two-token cases, uniform logits, k = 1, p -> 0)
 * and by exact inversion against a library softmax.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim, d_ff, vocab, max_ctx;
  int32_t norm;     /* 0 LayerNorm with bias, 1 RMSNorm */
  int32_t act;      /* 0 GELU (erf), 1 ReLU, 2 SwiGLU */
  int32_t pos;      /* 0 learned absolute table, 1 RoPE (rotate-half) */
  int32_t has_bias; /* linear biases present */
  int32_t wdtype;   /* 0 fp32, 1 bf16 */
  double norm_eps, rope_theta;
} orc_dims;

typedef struct {
  const void *tok_emb, *pos_emb, *lnf_g, *lnf_b, *lm_head, *early_head;
  const void **ln1_g, **ln1_b, **wq, **wk, **wv, **wo, **bq, **bk, **bv, **bo;
  const void **ln2_g, **ln2_b, **w_in, **w_up, **w_out, **b_in, **b_out;
} orc_weights;

typedef struct {
  int64_t rounds;            /* rounds executed (= tokens emitted) */
  int64_t matches;           /* rounds whose early top-k held the final token */
  int64_t runs;              /* N of Sec. 4.1 */
  int64_t main_layer_rows;   /* layer executions of the main process */
  int64_t branch_layer_rows; /* layer executions of all sub-processes */
} orc_stats;

#define ORC_KMAX 64

typedef struct orc_model {
  orc_dims d;
  orc_weights w;
  int ctx_cap;
  double *K, *V;         /* [n_layers][ctx_cap][d_model] */
  double *tailK, *tailV; /* [n_layers][ORC_KMAX][d_model]: one slot per sub-process */
  /* rule for the final prediction (Appendix B): 0 arg max, 1 top-k sampling, 2 top-p sampling */
  int sel_mode, sel_k;
  double sel_p;
  uint64_t sel_seed;
} orc_model;

/* ------------------------------------------------------------------ helpers */

static inline double wload(const void *p, size_t i, int wdtype) {
  if (wdtype == 0) return (double)((const float *)p)[i];
  uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* y[o] = sum_i x[i] * W[o][i] (+ b[o]); W row-major [n_out][n_in] */
static void linear(const orc_model *m, const void *W, const void *b, int n_out, int n_in,
                   const double *x, double *y) {
  const int wd = m->d.wdtype;
#pragma omp parallel for schedule(static)
  for (int o = 0; o < n_out; ++o) {
    double acc = 0.0;
    if (wd == 0) {
      const float *row = (const float *)W + (size_t)o * n_in;
#pragma omp simd reduction(+ : acc)
      for (int i = 0; i < n_in; ++i) acc += x[i] * (double)row[i];
    } else {
      const uint16_t *row = (const uint16_t *)W + (size_t)o * n_in;
#pragma omp simd reduction(+ : acc)
      for (int i = 0; i < n_in; ++i) {
        union { uint32_t u; float f; } c;
        c.u = (uint32_t)row[i] << 16;
        acc += x[i] * (double)c.f;
      }
    }
    if (b) acc += wload(b, o, wd);
    y[o] = acc;
  }
}

/* LayerNorm: (x - mean) / sqrt(var + eps) * g + b, biased variance.
 * RMSNorm:   x / sqrt(mean(x^2) + eps) * g. */
static void norm_apply(const orc_model *m, const void *g, const void *b, const double *x, double *y) {
  const int n = m->d.d_model, wd = m->d.wdtype;
  if (m->d.norm == 0) {
    double mu = 0.0, var = 0.0;
    for (int i = 0; i < n; ++i) mu += x[i];
    mu /= n;
    for (int i = 0; i < n; ++i) var += (x[i] - mu) * (x[i] - mu);
    var /= n;
    double r = 1.0 / sqrt(var + m->d.norm_eps);
    for (int i = 0; i < n; ++i) y[i] = (x[i] - mu) * r * wload(g, i, wd) + (b ? wload(b, i, wd) : 0.0);
  } else {
    double ms = 0.0;
    for (int i = 0; i < n; ++i) ms += x[i] * x[i];
    ms /= n;
    double r = 1.0 / sqrt(ms + m->d.norm_eps);
    for (int i = 0; i < n; ++i) y[i] = x[i] * r * wload(g, i, wd);
  }
}

/* Rotary embedding, rotate-half pairing: inside every head the pair
 * (i, i + hd/2) is rotated by the angle pos * theta^(-2i/hd). */
static void rope_apply(const orc_model *m, double *v, int pos) {
  if (m->d.pos != 1) return;
  const int hd = m->d.head_dim, half = hd / 2;
  for (int h = 0; h < m->d.n_heads; ++h) {
    double *p = v + (size_t)h * hd;
    for (int i = 0; i < half; ++i) {
      double ang = (double)pos * pow(m->d.rope_theta, -2.0 * i / hd);
      double c = cos(ang), s = sin(ang);
      double a = p[i], b = p[i + half];
      p[i] = a * c - b * s;
      p[i + half] = b * c + a * s;
    }
  }
}

static void embed(const orc_model *m, int token, int pos, double *h) {
  const int n = m->d.d_model, wd = m->d.wdtype;
  for (int i = 0; i < n; ++i) {
    double v = wload(m->w.tok_emb, (size_t)token * n + i, wd);
    if (m->d.pos == 0) v += wload(m->w.pos_emb, (size_t)pos * n + i, wd);
    h[i] = v;
  }
}

static double act_fn(int act, double u) {
  if (act == 0) return 0.5 * u * (1.0 + erf(u * 0.70710678118654752440));
  if (act == 1) return u > 0.0 ? u : 0.0;
  return u / (1.0 + exp(-u)); /* silu, used on the gate */
}

/* feed-forward: GELU/ReLU: W_out act(W_in x + b_in) + b_out;
 * SwiGLU: W_out (silu(W_in x) * (W_up x)). */
static void ffn(const orc_model *m, int l, const double *x, double *y) {
  const int f = m->d.d_ff, dm = m->d.d_model;
  double *u = (double *)malloc(sizeof(double) * f);
  linear(m, m->w.w_in[l], m->d.has_bias ? m->w.b_in[l] : NULL, f, dm, x, u);
  if (m->d.act == 2) {
    double *g2 = (double *)malloc(sizeof(double) * f);
    linear(m, m->w.w_up[l], NULL, f, dm, x, g2);
    for (int i = 0; i < f; ++i) u[i] = act_fn(2, u[i]) * g2[i];
    free(g2);
  } else {
    for (int i = 0; i < f; ++i) u[i] = act_fn(m->d.act, u[i]);
  }
  linear(m, m->w.w_out[l], m->d.has_bias ? m->w.b_out[l] : NULL, dm, f, u, y);
  free(u);
}

static double *cacheK(const orc_model *m, int l, int pos) {
  return m->K + ((size_t)l * m->ctx_cap + pos) * m->d.d_model;
}
static double *cacheV(const orc_model *m, int l, int pos) {
  return m->V + ((size_t)l * m->ctx_cap + pos) * m->d.d_model;
}

/* One decoder block (0-based l) on one token at absolute position pos.
 * The token attends to the cached positions 0..pos-1 of this layer and to
 * itself; its own key and value are stored at kdst / vdst, which is either
 * the cache slot `pos` (main process) or a sub-process's private slot. */
static void block_forward(orc_model *m, int l, double *h, int pos, double *kdst, double *vdst) {
  const int dm = m->d.d_model, H = m->d.n_heads, hd = m->d.head_dim;
  const int hb = m->d.has_bias;
  double *a = (double *)malloc(sizeof(double) * dm * 3);
  double *q = a + dm, *o = a + 2 * dm;
  norm_apply(m, m->w.ln1_g[l], m->d.norm == 0 ? m->w.ln1_b[l] : NULL, h, a);
  linear(m, m->w.wq[l], hb ? m->w.bq[l] : NULL, dm, dm, a, q);
  linear(m, m->w.wk[l], hb ? m->w.bk[l] : NULL, dm, dm, a, kdst);
  linear(m, m->w.wv[l], hb ? m->w.bv[l] : NULL, dm, dm, a, vdst);
  rope_apply(m, q, pos);
  rope_apply(m, kdst, pos);
  const double scale = 1.0 / sqrt((double)hd);
#pragma omp parallel for schedule(static)
  for (int hh = 0; hh < H; ++hh) {
    double *s = (double *)malloc(sizeof(double) * (pos + 1));
    const double *qh = q + (size_t)hh * hd;
    double mx = -INFINITY;
    for (int j = 0; j <= pos; ++j) {
      const double *kj = (j < pos ? cacheK(m, l, j) : kdst) + (size_t)hh * hd;
      double acc = 0.0;
      for (int c = 0; c < hd; ++c) acc += qh[c] * kj[c];
      s[j] = acc * scale;
      if (s[j] > mx) mx = s[j];
    }
    double den = 0.0;
    for (int j = 0; j <= pos; ++j) { s[j] = exp(s[j] - mx); den += s[j]; }
    for (int c = 0; c < hd; ++c) {
      double acc = 0.0;
      for (int j = 0; j <= pos; ++j) {
        const double *vj = (j < pos ? cacheV(m, l, j) : vdst) + (size_t)hh * hd;
        acc += s[j] * vj[c];
      }
      o[(size_t)hh * hd + c] = acc / den;
    }
    free(s);
  }
  linear(m, m->w.wo[l], hb ? m->w.bo[l] : NULL, dm, dm, o, a);
  for (int i = 0; i < dm; ++i) h[i] += a[i];
  norm_apply(m, m->w.ln2_g[l], m->d.norm == 0 ? m->w.ln2_b[l] : NULL, h, a);
  ffn(m, l, a, q);
  for (int i = 0; i < dm; ++i) h[i] += q[i];
  free(a);
}

/* logits = W_head . Norm_f(h).  The paper's early prediction applies "a
 * language modeling classifier" to the intermediate state (Sec. 3); reading
 * taken here: the classifier is the final norm followed by the LM head, the
 * same module as the final prediction, unless a separate early head is given
 * (the per-layer trained classifier of Sec. 4.3), which replaces the matrix. */
static void head_logits(const orc_model *m, const double *h, int early, double *logits) {
  const int dm = m->d.d_model;
  double *a = (double *)malloc(sizeof(double) * dm);
  norm_apply(m, m->w.lnf_g, m->d.norm == 0 ? m->w.lnf_b : NULL, h, a);
  const void *W = (early && m->w.early_head) ? m->w.early_head : m->w.lm_head;
  linear(m, W, NULL, m->d.vocab, dm, a, logits);
  free(a);
}

/* Greedy choice; ties go to the lowest id (the paper is silent on ties). */
static int argmax_first(const double *z, int n) {
  int best = 0;
  for (int i = 1; i < n; ++i)
    if (z[i] > z[best]) best = i;
  return best;
}

/* Top-k by (logit descending, id ascending): k distinct ids.  The softmax of
 * Sec. 3 is monotone, so the order of the logits is the order of p(x|h). */
static void topk_ids(const double *z, int n, int k, int32_t *ids) {
  for (int r = 0; r < k; ++r) {
    int best = -1;
    for (int i = 0; i < n; ++i) {
      int taken = 0;
      for (int q = 0; q < r; ++q) taken |= (ids[q] == i);
      if (taken) continue;
      if (best < 0 || z[i] > z[best]) best = i;
    }
    ids[r] = best;
  }
}

/* ---- sampling-based final prediction (Appendix B)
 *
 * Philox-4x32-10: ten rounds of two 32x32->64 multiplications whose high and
 * low halves are crossed over and mixed with the counter words and the key;
 * the key moves on by the Weyl constants between rounds. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint64_t a = (uint64_t)0xD2511F53u * c0, b = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(b >> 32) ^ c1 ^ k0, n1 = (uint32_t)b;
    const uint32_t n2 = (uint32_t)(a >> 32) ^ c3 ^ k1, n3 = (uint32_t)a;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* u in [0, 1) for the token chosen at sequence position `index`: the top 24
 * bits of the first output word (exact in fp32 and fp64 alike). */
double orc_uniform(uint64_t seed, int64_t index) {
  const uint32_t ctr[4] = {(uint32_t)((uint64_t)index & 0xffffffffu), (uint32_t)((uint64_t)index >> 32), 0u, 0u};
  const uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
  uint32_t out[4];
  orc_philox4x32_10(ctr, key, out);
  return (double)(out[0] >> 8) / 16777216.0;
}

typedef struct { double z; int id; } orc_zi;
static int by_logit_desc(const void *a, const void *b) {
  const orc_zi *x = (const orc_zi *)a, *y = (const orc_zi *)b;
  if (x->z != y->z) return x->z > y->z ? -1 : 1;
  return x->id < y->id ? -1 : (x->id > y->id ? 1 : 0);
}

/* Draw from the truncated softmax by inversion.  Tokens are ranked by
 * (logit descending, id ascending); w_j = exp(z_j - z_max).
 *   mode 1, top-k sampling (Fan et al. 2018): the ks most probable tokens are kept;
 *   mode 2, top-p sampling (Holtzman et al. 2019): the shortest prefix of the
 *           ranking whose probability mass reaches p is kept.
 * With W the kept mass, the token is the first of the ranking whose cumulative
 * mass exceeds u W.  mode 0 is the arg max. */
int orc_sample(const double *z, int n, int mode, int ks, double p, double u) {
  if (mode == 0) return argmax_first(z, n);
  orc_zi *r = (orc_zi *)malloc(sizeof(orc_zi) * (size_t)n);
  for (int i = 0; i < n; ++i) { r[i].z = z[i]; r[i].id = i; }
  qsort(r, (size_t)n, sizeof(orc_zi), by_logit_desc);
  double *cum = (double *)malloc(sizeof(double) * (size_t)n);
  double acc = 0.0;
  for (int j = 0; j < n; ++j) { acc += exp(r[j].z - r[0].z); cum[j] = acc; }
  int keep;
  if (mode == 1) keep = ks < n ? (ks < 1 ? 1 : ks) : n;
  else {
    keep = n;
    for (int j = 0; j < n; ++j) if (cum[j] >= p * cum[n - 1]) { keep = j + 1; break; }
  }
  const double target = u * cum[keep - 1];
  int pick = keep - 1;
  for (int j = 0; j < keep; ++j) if (cum[j] > target) { pick = j; break; }
  const int id = r[pick].id;
  free(r); free(cum);
  return id;
}

/* The final prediction of the token that will sit at sequence position `index`. */
static int select_final(const orc_model *m, const double *z, int64_t index) {
  if (m->sel_mode == 0) return argmax_first(z, m->d.vocab);
  return orc_sample(z, m->d.vocab, m->sel_mode, m->sel_k, m->sel_p, orc_uniform(m->sel_seed, index));
}

/* ------------------------------------------------------------------ C API */

void orc_set_selection(orc_model *m, int mode, int ks, double p, uint64_t seed) {
  m->sel_mode = mode; m->sel_k = ks; m->sel_p = p; m->sel_seed = seed;
}

orc_model *orc_create(const orc_dims *d, const orc_weights *w, int ctx_cap) {
  orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
  m->d = *d;
  m->w = *w;
  m->ctx_cap = ctx_cap;
  size_t n = (size_t)d->n_layers * ctx_cap * d->d_model;
  m->K = (double *)malloc(sizeof(double) * n);
  m->V = (double *)malloc(sizeof(double) * n);
  size_t nt = (size_t)d->n_layers * ORC_KMAX * d->d_model;
  m->tailK = (double *)malloc(sizeof(double) * nt);
  m->tailV = (double *)malloc(sizeof(double) * nt);
  if (!m->K || !m->V || !m->tailK || !m->tailV) return NULL;
  return m;
}

void orc_destroy(orc_model *m) {
  if (!m) return;
  free(m->K); free(m->V); free(m->tailK); free(m->tailV); free(m);
}

/* Prompt handling (the algorithm takes a single start token x_0; experiments
 * use prompts): positions 0..P-2 of the prompt are run through all layers to
 * fill the cache, the last prompt token is the start token x_0. */
static void prefill(orc_model *m, const int32_t *prompt, int P) {
  double *h = (double *)malloc(sizeof(double) * m->d.d_model);
  for (int i = 0; i + 1 < P; ++i) {
    embed(m, prompt[i], i, h);
    for (int l = 0; l < m->d.n_layers; ++l) block_forward(m, l, h, i, cacheK(m, l, i), cacheV(m, l, i));
  }
  free(h);
}

/* Plain greedy decoding with a KV cache: ell tokens, each after all d layers.
 * logits_out (nullable): [ell][vocab] final-layer logits of every step. */
int orc_plain_greedy(orc_model *m, const int32_t *prompt, int P, int ell, int eos,
                     int32_t *tokens_out, double *logits_out) {
  const int dm = m->d.d_model, V = m->d.vocab, d = m->d.n_layers;
  if (P < 1 || P - 1 + ell > m->ctx_cap) return -1;
  prefill(m, prompt, P);
  double *h = (double *)malloc(sizeof(double) * dm);
  double *z = (double *)malloc(sizeof(double) * V);
  int x = prompt[P - 1], pos = P - 1, t = 0;
  while (t < ell && x != eos) {
    embed(m, x, pos, h);
    for (int l = 0; l < d; ++l) block_forward(m, l, h, pos, cacheK(m, l, pos), cacheV(m, l, pos));
    head_logits(m, h, 0, z);
    x = select_final(m, z, pos + 1);
    tokens_out[t] = x;
    if (logits_out) memcpy(logits_out + (size_t)t * V, z, sizeof(double) * V);
    ++pos; ++t;
  }
  free(h); free(z);
  return t;
}

/* Whole-sequence causal forward in matrix form, no cache: the textbook
 * definition.  logits_out: [n][vocab] (all positions) */
int orc_full_forward(orc_model *m, const int32_t *tokens, int n, double *logits_out) {
  const int dm = m->d.d_model, H = m->d.n_heads, hd = m->d.head_dim, d = m->d.n_layers;
  const int hb = m->d.has_bias;
  size_t sz = (size_t)n * dm;
  double *X = (double *)malloc(sizeof(double) * sz * 5);
  double *A = X + sz, *Q = X + 2 * sz, *Kx = X + 3 * sz, *Vx = X + 4 * sz;
  double *S = (double *)malloc(sizeof(double) * n);
  for (int i = 0; i < n; ++i) embed(m, tokens[i], i, X + (size_t)i * dm);
  const double scale = 1.0 / sqrt((double)hd);
  for (int l = 0; l < d; ++l) {
    for (int i = 0; i < n; ++i) {
      double *a = A + (size_t)i * dm;
      norm_apply(m, m->w.ln1_g[l], m->d.norm == 0 ? m->w.ln1_b[l] : NULL, X + (size_t)i * dm, a);
      linear(m, m->w.wq[l], hb ? m->w.bq[l] : NULL, dm, dm, a, Q + (size_t)i * dm);
      linear(m, m->w.wk[l], hb ? m->w.bk[l] : NULL, dm, dm, a, Kx + (size_t)i * dm);
      linear(m, m->w.wv[l], hb ? m->w.bv[l] : NULL, dm, dm, a, Vx + (size_t)i * dm);
      rope_apply(m, Q + (size_t)i * dm, i);
      rope_apply(m, Kx + (size_t)i * dm, i);
    }
    for (int i = 0; i < n; ++i) {
      double *a = A + (size_t)i * dm; /* reuse as attention output */
      for (int hh = 0; hh < H; ++hh) {
        const double *qh = Q + (size_t)i * dm + (size_t)hh * hd;
        double mx = -INFINITY, den = 0.0;
        for (int j = 0; j <= i; ++j) {
          const double *kj = Kx + (size_t)j * dm + (size_t)hh * hd;
          double acc = 0.0;
          for (int c = 0; c < hd; ++c) acc += qh[c] * kj[c];
          S[j] = acc * scale;
          if (S[j] > mx) mx = S[j];
        }
        for (int j = 0; j <= i; ++j) { S[j] = exp(S[j] - mx); den += S[j]; }
        for (int c = 0; c < hd; ++c) {
          double acc = 0.0;
          for (int j = 0; j <= i; ++j) acc += S[j] * Vx[(size_t)j * dm + (size_t)hh * hd + c];
          a[(size_t)hh * hd + c] = acc / den;
        }
      }
    }
    double *tmp = (double *)malloc(sizeof(double) * dm * 2);
    for (int i = 0; i < n; ++i) {
      double *x = X + (size_t)i * dm;
      linear(m, m->w.wo[l], hb ? m->w.bo[l] : NULL, dm, dm, A + (size_t)i * dm, tmp);
      for (int c = 0; c < dm; ++c) x[c] += tmp[c];
      norm_apply(m, m->w.ln2_g[l], m->d.norm == 0 ? m->w.ln2_b[l] : NULL, x, tmp);
      ffn(m, l, tmp, tmp + dm);
      for (int c = 0; c < dm; ++c) x[c] += tmp[dm + c];
    }
    free(tmp);
  }
  for (int i = 0; i < n; ++i) head_logits(m, X + (size_t)i * dm, 0, logits_out + (size_t)i * m->d.vocab);
  free(X); free(S);
  return 0;
}

/* Plain greedy decoding without a cache: every step re-runs the whole
 * sequence through orc_full_forward and takes the last position's argmax. */
int orc_plain_recompute(orc_model *m, const int32_t *prompt, int P, int ell, int32_t *tokens_out,
                        double *logits_out) {
  const int V = m->d.vocab;
  int32_t *seq = (int32_t *)malloc(sizeof(int32_t) * (P + ell));
  double *z = (double *)malloc(sizeof(double) * (size_t)(P + ell) * V);
  memcpy(seq, prompt, sizeof(int32_t) * P);
  for (int t = 0; t < ell; ++t) {
    int n = P + t;
    orc_full_forward(m, seq, n, z);
    const double *last = z + (size_t)(n - 1) * V;
    int x = select_final(m, last, n);
    seq[n] = x;
    tokens_out[t] = x;
    if (logits_out) memcpy(logits_out + (size_t)t * V, last, sizeof(double) * V);
  }
  free(seq); free(z);
  return ell;
}

/* Predictive Pipelined Decoding, Algorithm 2 (dbar >= d/2; dbar = d/2 is
 * Algorithm 1), run sequentially.  One loop iteration = one round = one token.
 *
 * Sub-process i keeps the key/value of its candidate token in a private slot
 * per layer ("tail"); on a match the matching sub-process's slots become the
 * cache entries of position t+1 for layers 1..d-dbar (the paper only says the
 * matching process's results are kept and the others disregarded, Sec. 3).
 * Every round launches its sub-processes, the last one included, as the
 * compute count k(d-dbar)l of Theorem 4.1 requires.
 *
 * Outputs (all nullable except tokens_out):
 *   cand_out      [ell][k]  early top-k ids of every round
 *   match_idx_out [ell]     index in 0..k-1 of the matching candidate, or -1
 *   early_logits_out / final_logits_out [ell][vocab]
 */
int orc_ppd(orc_model *m, const int32_t *prompt, int P, int ell, int k, int dbar, int eos,
            int32_t *tokens_out, int32_t *cand_out, int32_t *match_idx_out, orc_stats *stats,
            double *early_logits_out, double *final_logits_out) {
  const int dm = m->d.d_model, V = m->d.vocab, d = m->d.n_layers;
  if (P < 1 || P + ell > m->ctx_cap) return -1;       /* sub-processes touch position t+1 */
  if (k < 1 || k > ORC_KMAX || k > V) return -1;
  if (2 * dbar < d || dbar > d) return -1;             /* Theorem 4.1: dbar >= d/2 */
  prefill(m, prompt, P);
  double *h0 = (double *)malloc(sizeof(double) * dm);  /* main process state, h^(0) */
  double *hm = (double *)malloc(sizeof(double) * dm);
  double *hs = (double *)malloc(sizeof(double) * dm * k); /* h^(i), i = 1..k */
  double *ze = (double *)malloc(sizeof(double) * V);
  double *zf = (double *)malloc(sizeof(double) * V);
  int32_t *cand = (int32_t *)malloc(sizeof(int32_t) * k);
  orc_stats st;
  memset(&st, 0, sizeof st);
  const int nb = d - dbar; /* layers each sub-process runs */
  int x = prompt[P - 1], pos = P - 1, t = 0, match = 0;
  while (t < ell && x != eos) {
    /* main process up to the exit layer */
    if (!match) {
      st.runs += 1;
      embed(m, x, pos, h0);
      for (int l = 0; l < dbar; ++l) block_forward(m, l, h0, pos, cacheK(m, l, pos), cacheV(m, l, pos));
      st.main_layer_rows += dbar;
    } else {
      for (int l = nb; l < dbar; ++l) block_forward(m, l, h0, pos, cacheK(m, l, pos), cacheV(m, l, pos));
      st.main_layer_rows += dbar - nb;
    }
    /* early prediction and its distribution */
    head_logits(m, h0, 1, ze);
    topk_ids(ze, V, k, cand);
    /* parallel part: no data flows between the processes until verification */
    match = 0;
    memcpy(hm, h0, sizeof(double) * dm);
    for (int l = dbar; l < d; ++l) block_forward(m, l, hm, pos, cacheK(m, l, pos), cacheV(m, l, pos));
    st.main_layer_rows += d - dbar;
    head_logits(m, hm, 0, zf);
    int xn = select_final(m, zf, pos + 1);
    for (int i = 0; i < k; ++i) {
      double *hi = hs + (size_t)i * dm;
      embed(m, cand[i], pos + 1, hi);
      for (int l = 0; l < nb; ++l)
        block_forward(m, l, hi, pos + 1, m->tailK + ((size_t)l * ORC_KMAX + i) * dm,
                      m->tailV + ((size_t)l * ORC_KMAX + i) * dm);
      st.branch_layer_rows += nb;
    }
    /* verification and adoption */
    int midx = -1;
    for (int i = 0; i < k; ++i)
      if (cand[i] == xn) {
        match = 1;
        midx = i;
        memcpy(h0, hs + (size_t)i * dm, sizeof(double) * dm);
        for (int l = 0; l < nb; ++l) {
          memcpy(cacheK(m, l, pos + 1), m->tailK + ((size_t)l * ORC_KMAX + i) * dm, sizeof(double) * dm);
          memcpy(cacheV(m, l, pos + 1), m->tailV + ((size_t)l * ORC_KMAX + i) * dm, sizeof(double) * dm);
        }
        break;
      }
    st.rounds += 1;
    st.matches += match;
    tokens_out[t] = xn;
    if (cand_out) memcpy(cand_out + (size_t)t * k, cand, sizeof(int32_t) * k);
    if (match_idx_out) match_idx_out[t] = midx;
    if (early_logits_out) memcpy(early_logits_out + (size_t)t * V, ze, sizeof(double) * V);
    if (final_logits_out) memcpy(final_logits_out + (size_t)t * V, zf, sizeof(double) * V);
    x = xn; ++pos; ++t;
  }
  if (stats) *stats = st;
  free(h0); free(hm); free(hs); free(ze); free(zf); free(cand);
  return t;
}

/* Teacher-forced logits with the cache: feeds tokens[0..n) one by one and
 * writes, for every position i >= first, the final logits and (if requested,
 * dbar >= 1) the early logits taken after layer dbar.  Row i - first. */
int orc_teacher_forced(orc_model *m, const int32_t *tokens, int n, int first, int dbar,
                       double *final_logits_out, double *early_logits_out) {
  const int dm = m->d.d_model, V = m->d.vocab, d = m->d.n_layers;
  if (n > m->ctx_cap) return -1;
  double *h = (double *)malloc(sizeof(double) * dm);
  for (int i = 0; i < n; ++i) {
    embed(m, tokens[i], i, h);
    for (int l = 0; l < d; ++l) {
      block_forward(m, l, h, i, cacheK(m, l, i), cacheV(m, l, i));
      if (i >= first && early_logits_out && l + 1 == dbar)
        head_logits(m, h, 1, early_logits_out + (size_t)(i - first) * V);
    }
    if (i >= first && final_logits_out) head_logits(m, h, 0, final_logits_out + (size_t)(i - first) * V);
  }
  free(h);
  return 0;
}

/* ---- primitives exported for the pin tests ---- */
void orc_linear(orc_model *m, const void *W, const void *b, int n_out, int n_in, const double *x, double *y) {
  linear(m, W, b, n_out, n_in, x, y);
}
void orc_norm(orc_model *m, const void *g, const void *b, const double *x, double *y) { norm_apply(m, g, b, x, y); }
void orc_rope(orc_model *m, double *v, int pos) { rope_apply(m, v, pos); }
double orc_act(int act, double u) { return act_fn(act, u); }
void orc_topk(const double *z, int n, int k, int32_t *ids) { topk_ids(z, n, k, ids); }
int orc_argmax(const double *z, int n) { return argmax_first(z, n); }
