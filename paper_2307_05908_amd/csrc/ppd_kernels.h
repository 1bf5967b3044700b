// HIP kernels of the PPD decode path for gfx950 (64-wide wavefronts).
//
// Every kernel takes up to two row groups per launch.  In a pipelined step of
// the parallel phase (Algorithm 2, the "in parallel" block) group 0 is the
// main token at layer dbar+j (one row) and group 1 holds the k candidate
// tokens at layer j (k rows): two different layers' weights, each streamed
// from HBM once for all rows of its group.
//
// Bit-reproducibility rule: the arithmetic that produces one output row
// depends only on that row's inputs, never on how many rows share the launch,
// on the group, or on where the row's own key/value is stored.  Each reduction
// has one fixed order (lane -> k mapping, butterfly across lanes, waves in
// index order, position chunks in index order), and every multiply-add is an
// explicit fmaf.  This is what makes a candidate row's layers 1..d-dbar equal,
// bit for bit, to the layers plain decoding would run on the same token.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ppd {

struct bf16_t { uint16_t v; };

constexpr int WAVE = 64;
constexpr int GEMM_THREADS = 256;   // 4 waves
constexpr int GEMM_WAVES = GEMM_THREADS / WAVE;
constexpr int GEMM_WROWS = 4;       // weight rows per wave per tile
constexpr int ATT_THREADS = 256;
constexpr int ATT_WAVES = ATT_THREADS / WAVE;
constexpr int ATT_CHUNK = 128;      // positions per workgroup; chunk c covers [c*128, (c+1)*128)
constexpr int MAXM = 8;

__device__ __forceinline__ float bf16_to_f32(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename WT> struct WTr;
template <> struct WTr<float> {
  static constexpr int VEC = 4;
  __device__ static __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
  __device__ static __forceinline__ float load1(const void* p, size_t i) { return ((const float*)p)[i]; }
  __device__ static __forceinline__ float round(float x) { return x; }
  __device__ static __forceinline__ void store1(void* p, size_t i, float x) { ((float*)p)[i] = x; }
};
template <> struct WTr<bf16_t> {
  static constexpr int VEC = 8;
  __device__ static __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
  __device__ static __forceinline__ float load1(const void* p, size_t i) { return bf16_to_f32(((const uint16_t*)p)[i]); }
  __device__ static __forceinline__ float round(float x) { return bf16_to_f32(f32_to_bf16(x)); }
  __device__ static __forceinline__ void store1(void* p, size_t i, float x) { ((uint16_t*)p)[i] = f32_to_bf16(x); }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}
// Sum over a 256-thread workgroup: butterfly inside each wave, then the four wave
// sums in index order.  red: >= 4 floats of LDS.  Ends with every thread holding the sum.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float s = red[0];
#pragma unroll
  for (int w = 1; w < GEMM_WAVES; ++w) s += red[w];
  return s;
}

// ------------------------------------------------------------------ embedding
// Row set-up (start of the main process, start of every sub-process): h_0 = E[token] (+ P[pos]).
struct EmbedArgs {
  const void* tok_emb; const void* pos_emb;   // pos_emb null for RoPE models
  const int32_t* ids;   // DEVICE: token id of row r is ids[r]
  float* h;             // [rows][d_model]
  int rows, d_model, pos;
};
template <typename WT>
__global__ void embed_kernel(EmbedArgs a) {
  int r = blockIdx.y;
  int tok = a.ids[r];
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < a.d_model; i += gridDim.x * blockDim.x) {
    float v = WTr<WT>::load1(a.tok_emb, (size_t)tok * a.d_model + i);
    if (a.pos_emb) v += WTr<WT>::load1(a.pos_emb, (size_t)a.pos * a.d_model + i);
    a.h[(size_t)r * a.d_model + i] = v;
  }
}

// ------------------------------------------------------------------ skinny GEMM
// Y[m][n] = epilogue( sum_k norm(X)[m][k] * W[n][k] ), M <= 8 rows per group.
// The layer forward of the main process and of the sub-processes (Algorithm 2);
// the sub-processes' k rows share one pass over their layer's weights.
struct GemmGroup {
  const float* X;     // [M][ldx] input rows (before the fused norm)
  const float* Rsd;   // residual rows [M][ldy] added in the epilogue, or null
  float* Y;           // [M][ldy]
  const void* W[3];   // up to three row segments (Q,K,V); for SwiGLU W[0] = gate, W[1] = up, paired row by row
  const void* B[3];   // biases per segment or null
  const void* ng; const void* nb;  // gain / bias of the fused norm
  int M;
};
struct GemmArgs {
  GemmGroup g[2];
  int K;            // reduction length (multiple of VEC)
  int N[3];         // rows per segment
  int ntot;         // logical output rows (= N0+N1+N2, or N0 for SwiGLU)
  int ldx, ldy;
  int norm;         // -1 none, 0 LayerNorm, 1 RMSNorm
  float eps;
  int act;          // 0 none, 1 GELU, 2 ReLU, 3 SwiGLU (pairs W[0], W[1])
  int KC;           // K elements staged in LDS at a time (multiple of 64*VEC)
  int ntiles;       // tiles per group
};

__device__ __forceinline__ float gelu_erf(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752440f)); }
__device__ __forceinline__ float silu(float u) { return u / (1.0f + expf(-u)); }

template <typename WT, int MT, bool PAIRED>
__device__ __forceinline__ void gemm_body(const GemmArgs& a, const GemmGroup& G, float* lds) {
  constexpr int VEC = WTr<WT>::VEC;
  constexpr int LR = PAIRED ? GEMM_WROWS / 2 : GEMM_WROWS;  // logical rows per wave
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int M = G.M, K = a.K, KC = a.KC;
  float* red = lds;                 // 8 floats
  float* stat = lds + 8;            // mu[MAXM], rstd[MAXM]
  float4* xs4 = (float4*)(lds + 32);  // [M][KC/4] float4, swizzled per 8-group for VEC == 8

  // statistics of the fused norm: per row, fixed order
  if (a.norm >= 0) {
    for (int m = 0; m < M; ++m) {
      const float* x = G.X + (size_t)m * a.ldx;
      float mu = 0.f;
      if (a.norm == 0) {
        float s = 0.f;
        for (int i = tid; i < K; i += GEMM_THREADS) s += x[i];
        mu = block_sum(s, red) / (float)K;
      }
      float s2 = 0.f;
      for (int i = tid; i < K; i += GEMM_THREADS) { float d = x[i] - mu; s2 = fmaf(d, d, s2); }
      float var = block_sum(s2, red) / (float)K;
      if (tid == 0) { stat[m] = mu; stat[MAXM + m] = 1.0f / sqrtf(var + a.eps); }
    }
    __syncthreads();
  }

  // stage (normalised) x[m][k0 .. k0+kc) in LDS
  auto stage = [&](int k0, int kc) {
    for (int idx = tid * 4; idx < M * kc; idx += GEMM_THREADS * 4) {
      int m = idx / kc, kk = idx - m * kc;
      float4 v = *(const float4*)(G.X + (size_t)m * a.ldx + k0 + kk);
      if (a.norm >= 0) {
        float mu = stat[m], rs = stat[MAXM + m];
        float xv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float gq = WTr<WT>::load1(G.ng, k0 + kk + e);
          float t = (xv[e] - mu) * rs * gq;
          if (G.nb) t += WTr<WT>::load1(G.nb, k0 + kk + e);
          xv[e] = t;
        }
        v = make_float4(xv[0], xv[1], xv[2], xv[3]);
      }
      int slot = (VEC == 8) ? (((kk & 7) >> 2) * (KC >> 3) + (kk >> 3)) : (kk >> 2);
      xs4[m * (KC >> 2) + slot] = v;
    }
  };
  const bool single = KC >= K;   // the whole reduction length fits one LDS pass: stage once
  bool staged = false;

  for (int tile = blockIdx.x; tile < a.ntiles; tile += gridDim.x) {
    // the wave's weight rows
    const char* wp[GEMM_WROWS];
    int lrow[LR];
#pragma unroll
    for (int r = 0; r < LR; ++r) {
      int n = (tile * GEMM_WAVES + wave) * LR + r;
      lrow[r] = n;
      int nc = n < a.ntot ? n : a.ntot - 1;
      if (PAIRED) {
        wp[2 * r] = (const char*)G.W[0] + (size_t)nc * K * sizeof(WT);
        wp[2 * r + 1] = (const char*)G.W[1] + (size_t)nc * K * sizeof(WT);
      } else {
        int seg = 0, loc = nc;
        if (loc >= a.N[0]) { loc -= a.N[0]; seg = 1; if (loc >= a.N[1]) { loc -= a.N[1]; seg = 2; } }
        wp[r] = (const char*)G.W[seg] + (size_t)loc * K * sizeof(WT);
      }
    }
    float acc[GEMM_WROWS][MT];
#pragma unroll
    for (int r = 0; r < GEMM_WROWS; ++r)
#pragma unroll
      for (int m = 0; m < MT; ++m) acc[r][m] = 0.f;

    for (int k0 = 0; k0 < K; k0 += KC) {
      const int kc = (K - k0) < KC ? (K - k0) : KC;
      if (!single || !staged) {
        __syncthreads();
        stage(k0, kc);
        __syncthreads();
        staged = true;
      }
      // stream the weight rows of this chunk
#pragma unroll 2
      for (int kb = lane * VEC; kb < kc; kb += WAVE * VEC) {
        uint4 wv[GEMM_WROWS];
#pragma unroll
        for (int r = 0; r < GEMM_WROWS; ++r) wv[r] = *(const uint4*)(wp[r] + (size_t)(k0 + kb) * sizeof(WT));
        float xf[MT][VEC];
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          if (m < M) {
            float4 lo = xs4[m * (KC >> 2) + (VEC == 8 ? (kb >> 3) : (kb >> 2))];
            xf[m][0] = lo.x; xf[m][1] = lo.y; xf[m][2] = lo.z; xf[m][3] = lo.w;
            if constexpr (VEC == 8) {
              float4 hi = xs4[m * (KC >> 2) + (KC >> 3) + (kb >> 3)];
              xf[m][4] = hi.x; xf[m][5] = hi.y; xf[m][6] = hi.z; xf[m][7] = hi.w;
            }
          } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) xf[m][e] = 0.f;
          }
        }
#pragma unroll
        for (int r = 0; r < GEMM_WROWS; ++r) {
          float wf[VEC];
          WTr<WT>::unpack(wv[r], wf);
#pragma unroll
          for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[r][m] = fmaf(xf[m][e], wf[e], acc[r][m]);
        }
      }
    }
    // cross-lane reduction and epilogue
#pragma unroll
    for (int r = 0; r < GEMM_WROWS; ++r)
#pragma unroll
      for (int m = 0; m < MT; ++m) acc[r][m] = wave_sum(acc[r][m]);
    if (lane == 0) {
#pragma unroll
      for (int r = 0; r < LR; ++r) {
        int n = lrow[r];
        if (n >= a.ntot) continue;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          if (m >= M) continue;
          float y;
          if (PAIRED) {
            float gt = acc[2 * r][m], up = acc[2 * r + 1][m];
            if (G.B[0]) gt += WTr<WT>::load1(G.B[0], n);
            if (G.B[1]) up += WTr<WT>::load1(G.B[1], n);
            y = silu(gt) * up;
          } else {
            y = acc[r][m];
            int seg = 0, loc = n;
            if (loc >= a.N[0]) { loc -= a.N[0]; seg = 1; if (loc >= a.N[1]) { loc -= a.N[1]; seg = 2; } }
            if (G.B[seg]) y += WTr<WT>::load1(G.B[seg], loc);
            if (a.act == 1) y = gelu_erf(y);
            else if (a.act == 2) y = fmaxf(y, 0.f);
          }
          if (G.Rsd) y += G.Rsd[(size_t)m * a.ldy + n];
          G.Y[(size_t)m * a.ldy + n] = y;
        }
      }
    }
  }
}

// MA rows in group 0, MB rows in group 1 (MB == 0: single-group launch)
template <typename WT, int MA, int MB, bool PAIRED>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_kernel(GemmArgs a) {
  extern __shared__ float4 lds4[];
  float* lds = (float*)lds4;
  if (MB == 0 || blockIdx.y == 0) gemm_body<WT, MA, PAIRED>(a, a.g[0], lds);
  else gemm_body<WT, (MB < 1 ? 1 : MB), PAIRED>(a, a.g[1], lds);
}

// ------------------------------------------------------------------ attention
// Decode attention of one token per row over the layer's cached positions
// [0, p) plus the row's own position p.  The rows of a group share p and the
// cached prefix (the sub-processes all extend x_<=t by one candidate); each
// row has its own key/value for position p, which this kernel also rotates
// (RoPE), rounds to the cache type and stores: at cache slot p for the main
// token, in the row's tail slot for a candidate.
struct AttnGroup {
  const float* qkv;     // [M][3*d_model]: q | k | v as produced by the QKV projection
  const void* Kc; const void* Vc;   // this layer's cache, [H][max_ctx][hd]
  void* ownK; void* ownV;           // destination of the rows' own key/value
  long own_row_stride, own_head_stride;   // in elements: dst = own + m*row + h*head + i
  float* part;          // [M][H][nchunk_max][hd+2] partial (unnormalised o, max, sum)
  int p;                // number of cached positions attended to = position of the rows
  int M;
};
struct AttnArgs {
  AttnGroup g[2];
  const float2* rope;   // [max_ctx][hd/2] (cos, sin) or null
  int H, d_model, max_ctx, nchunk_max;
  float scale;
};

template <typename WT, int HD, int MT>
__device__ __forceinline__ void attn_body(const AttnArgs& a, const AttnGroup& G, float* lds) {
  constexpr int VEC = WTr<WT>::VEC;
  constexpr int LPR = HD / VEC;        // lanes per cached row
  constexpr int RPW = WAVE / LPR;      // cached rows per wave per load
  constexpr int RPP = RPW * ATT_WAVES; // rows per pass of the workgroup
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int h = blockIdx.y, c = blockIdx.x;
  const int p = G.p, M = G.M;
  const int j0 = c * ATT_CHUNK;
  if (j0 > p) return;
  const int j1 = (j0 + ATT_CHUNK < p + 1) ? j0 + ATT_CHUNK : p + 1;   // exclusive; position p is the row's own
  const bool owns_p = (p < j0 + ATT_CHUNK);
  float* qs = lds;                    // [MT][HD]
  float* ko = qs + MT * HD;           // [MT][HD] own key, rounded to cache type
  float* vo = ko + MT * HD;           // [MT][HD]
  float* sc = vo + MT * HD;           // [MT][ATT_CHUNK]
  float* st = sc + MT * ATT_CHUNK;    // [MT][2] max, sum
  float* ored = st + MT * 2;          // [ATT_WAVES][MT][HD]

  // own q, k, v of every row: rotate, scale / round, store
  for (int idx = tid; idx < M * HD; idx += ATT_THREADS) {
    int m = idx / HD, i = idx - m * HD;
    const float* row = G.qkv + (size_t)m * 3 * a.d_model + (size_t)h * HD;
    float q = row[i], k = row[a.d_model + i], v = row[2 * a.d_model + i];
    if (a.rope) {
      constexpr int half = HD / 2;
      int ii = i < half ? i : i - half;
      float2 cs = a.rope[(size_t)p * half + ii];
      float qo = i < half ? row[i + half] : row[i - half];
      float kk = i < half ? row[a.d_model + i + half] : row[a.d_model + i - half];
      if (i < half) { q = fmaf(q, cs.x, -(qo * cs.y)); k = fmaf(k, cs.x, -(kk * cs.y)); }
      else          { q = fmaf(q, cs.x, qo * cs.y);    k = fmaf(k, cs.x, kk * cs.y); }
    }
    qs[m * HD + i] = q * a.scale;
    ko[m * HD + i] = WTr<WT>::round(k);
    vo[m * HD + i] = WTr<WT>::round(v);
    if (owns_p) {
      size_t d = (size_t)m * G.own_row_stride + (size_t)h * G.own_head_stride + i;
      WTr<WT>::store1(G.ownK, d, k);
      WTr<WT>::store1(G.ownV, d, v);
    }
  }
  __syncthreads();

  const int cs = lane % LPR, rs = lane / LPR;
  float qr[MT][VEC];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int e = 0; e < VEC; ++e) qr[m][e] = (m < M) ? qs[m * HD + cs * VEC + e] : 0.f;

  const char* Kh = (const char*)G.Kc + (size_t)h * a.max_ctx * HD * sizeof(WT);
  const char* Vh = (const char*)G.Vc + (size_t)h * a.max_ctx * HD * sizeof(WT);

  // scores
  for (int base = j0; base < j1; base += RPP) {
    int j = base + wave * RPW + rs;
    bool valid = j < j1;
    float kf[VEC];
    if (valid && j < p) {
      uint4 r = *(const uint4*)(Kh + ((size_t)j * HD + cs * VEC) * sizeof(WT));
      WTr<WT>::unpack(r, kf);
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) kf[e] = 0.f;
    }
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      float s = 0.f;
      if (valid && j == p) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) s = fmaf(qr[m][e], ko[m * HD + cs * VEC + e], s);
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) s = fmaf(qr[m][e], kf[e], s);
      }
#pragma unroll
      for (int o = LPR / 2; o >= 1; o >>= 1) s += __shfl_xor(s, o, WAVE);
      if (cs == 0 && valid && m < M) sc[m * ATT_CHUNK + (j - j0)] = s;
    }
  }
  __syncthreads();
  // chunk-local softmax numerators: one wave per row
  const int nj = j1 - j0;
  for (int m = wave; m < M; m += ATT_WAVES) {
    float mx = -INFINITY;
    for (int j = lane; j < nj; j += WAVE) mx = fmaxf(mx, sc[m * ATT_CHUNK + j]);
    mx = wave_max(mx);
    float sum = 0.f;
    for (int j = lane; j < nj; j += WAVE) {
      float e = expf(sc[m * ATT_CHUNK + j] - mx);
      sc[m * ATT_CHUNK + j] = e;
      sum += e;
    }
    sum = wave_sum(sum);
    if (lane == 0) { st[m * 2] = mx; st[m * 2 + 1] = sum; }
  }
  __syncthreads();
  // weighted values
  float acc[MT][VEC];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[m][e] = 0.f;
  for (int base = j0; base < j1; base += RPP) {
    int j = base + wave * RPW + rs;
    bool valid = j < j1;
    float vf[VEC];
    if (valid && j < p) {
      uint4 r = *(const uint4*)(Vh + ((size_t)j * HD + cs * VEC) * sizeof(WT));
      WTr<WT>::unpack(r, vf);
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) vf[e] = 0.f;
    }
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      if (m >= M) continue;
      float pj = valid ? sc[m * ATT_CHUNK + (j - j0)] : 0.f;
      if (valid && j == p) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[m][e] = fmaf(pj, vo[m * HD + cs * VEC + e], acc[m][e]);
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[m][e] = fmaf(pj, vf[e], acc[m][e]);
      }
    }
  }
  // rows of the wave (lanes with equal cs), then the waves in index order
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      float v = acc[m][e];
#pragma unroll
      for (int o = 32; o >= LPR; o >>= 1) v += __shfl_xor(v, o, WAVE);
      acc[m][e] = v;
    }
  if (rs == 0) {
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        if (m < M) ored[(wave * MT + m) * HD + cs * VEC + e] = acc[m][e];
  }
  __syncthreads();
  for (int idx = tid; idx < M * HD; idx += ATT_THREADS) {
    int m = idx / HD, i = idx - m * HD;
    float o = ored[(0 * MT + m) * HD + i];
#pragma unroll
    for (int w = 1; w < ATT_WAVES; ++w) o += ored[(w * MT + m) * HD + i];
    float* dst = G.part + (((size_t)m * a.H + h) * a.nchunk_max + c) * (HD + 2);
    dst[i] = o;
    if (i == 0) { dst[HD] = st[m * 2]; dst[HD + 1] = st[m * 2 + 1]; }
  }
}

template <typename WT, int HD, int MA, int MB>
__global__ __launch_bounds__(ATT_THREADS) void attn_kernel(AttnArgs a) {
  extern __shared__ float4 lds4[];
  float* lds = (float*)lds4;
  if (MB == 0 || blockIdx.z == 0) attn_body<WT, HD, MA>(a, a.g[0], lds);
  else attn_body<WT, HD, (MB < 1 ? 1 : MB)>(a, a.g[1], lds);
}
template <int HD, int MT> constexpr size_t attn_lds_bytes() {
  return sizeof(float) * (3 * MT * HD + MT * ATT_CHUNK + MT * 2 + ATT_WAVES * MT * HD);
}

// merge of the chunk partials, chunks in index order
struct MergeArgs {
  const float* part[2]; float* out[2];   // out: [M][d_model]
  int p[2]; int M[2];
  int H, HD, d_model, nchunk_max;
};
__global__ void attn_merge_kernel(MergeArgs a) {
  int g = blockIdx.z, h = blockIdx.y, m = blockIdx.x;
  if (m >= a.M[g]) return;
  int nc = a.p[g] / ATT_CHUNK + 1;
  int i = threadIdx.x;
  if (i >= a.HD) return;
  const float* base = a.part[g] + (((size_t)m * a.H + h) * a.nchunk_max) * (a.HD + 2);
  float mx = -INFINITY;
  for (int c = 0; c < nc; ++c) mx = fmaxf(mx, base[(size_t)c * (a.HD + 2) + a.HD]);
  float o = 0.f, l = 0.f;
  for (int c = 0; c < nc; ++c) {
    const float* pc = base + (size_t)c * (a.HD + 2);
    float w = expf(pc[a.HD] - mx);
    o = fmaf(w, pc[i], o);
    l = fmaf(w, pc[a.HD + 1], l);
  }
  a.out[g][(size_t)m * a.d_model + (size_t)h * a.HD + i] = o / l;
}

// ------------------------------------------------------------------ selection
// Early prediction: top-k of the early logits by (logit descending, id ascending).
// Final prediction: arg max of the final logits (ties to the lowest id), then
// verification against the early candidates (Algorithm 2: "if x-hat^(PID) = x_{t+1}").
// One workgroup of 1024 threads; every thread keeps its own sorted top-k of a
// strided slice, then k rounds of a workgroup-wide best-of selection.
struct SelectArgs {
  const float* logits; int vocab; int k;
  int mode;            // 0: early top-k -> cand[0..k); 1: final arg max + verify
  int32_t* cand;       // DEVICE [MAXM]
  int32_t* result;     // DEVICE: [0] token, [1] match_idx  (mode 1)
  int32_t* next_tok;   // DEVICE: token id the next main row embeds (mode 1)
};
constexpr int SEL_THREADS = 1024;

__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

__global__ __launch_bounds__(SEL_THREADS) void select_kernel(SelectArgs a) {
  __shared__ float wv[SEL_THREADS / WAVE];
  __shared__ int wi[SEL_THREADS / WAVE];
  __shared__ int win_id;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int k = a.mode == 0 ? a.k : 1;
  float lv[MAXM]; int li[MAXM];
#pragma unroll
  for (int q = 0; q < MAXM; ++q) { lv[q] = -INFINITY; li[q] = 0x7fffffff; }
  for (int i = tid; i < a.vocab; i += SEL_THREADS) {
    float v = a.logits[i];
    if (better(v, i, lv[MAXM - 1], li[MAXM - 1])) {
      lv[MAXM - 1] = v; li[MAXM - 1] = i;
#pragma unroll
      for (int q = MAXM - 1; q > 0; --q)
        if (better(lv[q], li[q], lv[q - 1], li[q - 1])) {
          float tv = lv[q]; lv[q] = lv[q - 1]; lv[q - 1] = tv;
          int ti = li[q]; li[q] = li[q - 1]; li[q - 1] = ti;
        }
    }
  }
  int head = 0;   // index of this thread's best remaining candidate
  for (int r = 0; r < k; ++r) {
    float v = -INFINITY; int i = 0x7fffffff;
#pragma unroll
    for (int q = 0; q < MAXM; ++q) if (q == head) { v = lv[q]; i = li[q]; }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      float ov = __shfl_xor(v, o, WAVE); int oi = __shfl_xor(i, o, WAVE);
      if (better(ov, oi, v, i)) { v = ov; i = oi; }
    }
    __syncthreads();
    if (lane == 0) { wv[wave] = v; wi[wave] = i; }
    __syncthreads();
    if (tid == 0) {
      int bw = 0;
      for (int w = 1; w < SEL_THREADS / WAVE; ++w) if (better(wv[w], wi[w], wv[bw], wi[bw])) bw = w;
      int id = wi[bw];
      win_id = id;
      if (a.mode == 0) a.cand[r] = id;
      else {
        int midx = -1;
        for (int q = 0; q < a.k; ++q) if (a.cand[q] == id) { midx = q; break; }
        a.result[0] = id; a.result[1] = midx; *a.next_tok = id;
      }
    }
    __syncthreads();
    // ids are unique across threads: only the owner of the winner moves on
    int wid = win_id;
    int cur = 0x7fffffff;
#pragma unroll
    for (int q = 0; q < MAXM; ++q) if (q == head) cur = li[q];
    if (cur == wid) ++head;
  }
}

// ------------------------------------------------------------------ adoption
// On a match the matching sub-process's state becomes the main process's
// (Algorithm 2: h^(0)_{d-dbar} <- h^(PID)_{d-dbar}); its key/value tails of layers
// 1..d-dbar become cache position t+1.  Without a match nothing is copied: the
// tails are simply overwritten by the next round.
struct CommitArgs {
  const int32_t* result;    // DEVICE: [1] = match_idx
  float* h;                 // [1+k][d_model]: row 0 main, rows 1.. candidates
  const void* tailK; const void* tailV;   // [nb][k][H][hd]
  void* Kc; void* Vc;       // [L][H][max_ctx][hd]
  int k, H, hd, d_model, max_ctx, pos_next, wbytes;
};
__global__ void commit_kernel(CommitArgs a) {
  int midx = a.result[1];
  if (midx < 0) return;
  int l = blockIdx.x;
  if (l == 0 && blockIdx.y == 0)
    for (int i = threadIdx.x; i < a.d_model; i += blockDim.x) a.h[i] = a.h[(size_t)(1 + midx) * a.d_model + i];
  const char* src = (const char*)(blockIdx.y == 0 ? a.tailK : a.tailV) + ((size_t)l * a.k + midx) * a.d_model * a.wbytes;
  char* dst = (char*)(blockIdx.y == 0 ? a.Kc : a.Vc) + (size_t)l * a.H * a.max_ctx * a.hd * a.wbytes;
  int row_bytes = a.hd * a.wbytes;   // multiple of 16
  for (int idx = threadIdx.x; idx < a.H * (row_bytes / 16); idx += blockDim.x) {
    int hh = idx / (row_bytes / 16), q = idx - hh * (row_bytes / 16);
    uint4 v = *(const uint4*)(src + (size_t)hh * row_bytes + q * 16);
    *(uint4*)(dst + ((size_t)hh * a.max_ctx + a.pos_next) * row_bytes + q * 16) = v;
  }
}

}  // namespace ppd
