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
// on the group, on the grid, or on where the row's own key/value is stored.
// Each reduction has one fixed order (lane -> k mapping, butterfly across
// lanes, waves in index order, position chunks in index order), and every
// multiply-add is an explicit fmaf.  This is what makes a candidate row's
// layers 1..d-dbar equal, bit for bit, to the layers plain decoding would run
// on the same token.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ppd {

struct bf16_t { uint16_t v; };
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int WAVE = 64;
constexpr int GEMM_THREADS = 256;   // 4 waves
constexpr int GEMM_WAVES = GEMM_THREADS / WAVE;
constexpr int GEMM_X_FLOATS = 15360; // floats of the LDS x tile (60 KB): 15 float4 per thread
constexpr int GEMM_BATCH = 8;       // 16-byte loads per lane in one register batch: WR weight rows x 8/WR k-blocks
constexpr int GEMM_AHEAD = 3;       // batches requested ahead of the arithmetic (ring of four register buffers)
constexpr int GEMM_LDS_HDR = 80;    // floats in front of the x tile: norm statistics and their reduction scratch
constexpr int HEAD_MAX_ROWS = 256;  // logits one workgroup of the head GEMM may produce (block top-k buffer)
constexpr int ATT_THREADS = 256;
constexpr int ATT_WAVES = ATT_THREADS / WAVE;
constexpr int ATT_CHUNK = 64;       // positions per workgroup; chunk c covers [c*64, (c+1)*64)
constexpr int MAXM = 8;

// Round state in device memory, written by the tiny state kernel before a round and by the
// selection kernels during it; read by every kernel that needs a position or a token id.
struct DevState {
  int32_t pos;        // absolute position of the main token x_t
  int32_t next_tok;   // id of x_t
  int32_t result[2];  // token x_{t+1}, match_idx of the last final selection
  int32_t cand[MAXM]; // early top-k ids
  int32_t cand_next[MAXM]; // candidates of the next round, predicted at the end of a matching round
  int32_t sampled;    // final prediction drawn by the sampling kernel (sampling-based variants)
  int32_t pos_pending; // position of the next round: set explicitly, or left by a round's final selection (pos + 1)
  int32_t seq;         // rounds finished since the context was created (the host waits for the next value)
};

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
  __device__ static __forceinline__ void unpack(const u32x4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
  __device__ static __forceinline__ float load1(const void* p, size_t i) { return ((const float*)p)[i]; }
  __device__ static __forceinline__ float round(float x) { return x; }
  __device__ static __forceinline__ void store1(void* p, size_t i, float x) { ((float*)p)[i] = x; }
};
template <> struct WTr<bf16_t> {
  static constexpr int VEC = 8;
  __device__ static __forceinline__ void unpack(const u32x4& r, float* f) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
  __device__ static __forceinline__ float load1(const void* p, size_t i) { return bf16_to_f32(((const uint16_t*)p)[i]); }
  __device__ static __forceinline__ float round(float x) { return bf16_to_f32(f32_to_bf16(x)); }
  __device__ static __forceinline__ void store1(void* p, size_t i, float x) { ((uint16_t*)p)[i] = f32_to_bf16(x); }
};

// weights and cached keys/values are read once per launch: stream them past the caches
__device__ __forceinline__ u32x4 ld_stream(const void* p) { return __builtin_nontemporal_load((const u32x4*)p); }

// 64 lanes x 16 bytes from per-lane global addresses to LDS at lds_dst + 16 * lane (lds_dst is the same
// for the whole wave and goes through M0).  Written as assembly so that the wait for it stays ours:
// the request counts in vmcnt like any load, and loads return in order.
__device__ __forceinline__ void dma16(const void* src, void* lds_dst) {
  const unsigned la = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds_dst;
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(la) : "memory", "m0");
}

// Wave reductions on the data-parallel-primitive path: inside each row of 16 lanes with four
// lane-permuting adds (partner lanes compute a + b and b + a, so all 16 agree), then the four row
// results in row order.  Every lane returns the same value.
template <int CTRL> __device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float lane_f32(float v, int l) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l)); }
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f32<0xB1>(v);     // quad_perm [1,0,3,2]
  v += dpp_f32<0x4E>(v);     // quad_perm [2,3,0,1]
  v += dpp_f32<0x141>(v);    // row_half_mirror
  v += dpp_f32<0x140>(v);    // row_mirror
  return ((lane_f32(v, 0) + lane_f32(v, 16)) + lane_f32(v, 32)) + lane_f32(v, 48);
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f32<0xB1>(v));
  v = fmaxf(v, dpp_f32<0x4E>(v));
  v = fmaxf(v, dpp_f32<0x141>(v));
  v = fmaxf(v, dpp_f32<0x140>(v));
  return fmaxf(fmaxf(lane_f32(v, 0), lane_f32(v, 16)), fmaxf(lane_f32(v, 32), lane_f32(v, 48)));
}
__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }
// arg max by (value descending, id ascending) over a wave; every lane ends with the winner
__device__ __forceinline__ void wave_best(float& v, int& i) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    float ov = __shfl_xor(v, o, WAVE); int oi = __shfl_xor(i, o, WAVE);
    if (better(ov, oi, v, i)) { v = ov; i = oi; }
  }
}

// ------------------------------------------------------------------ round state
// (plain, non-template kernels are compiled into the engine's translation unit only)
#ifdef PPD_ENGINE_TU
// streaming-read probe: every thread walks the buffer with U 16-byte non-temporal loads in flight
template <int U>
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* p, size_t n16, uint32_t* sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (; i + (U - 1) * stride < n16; i += U * stride) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = ld_stream(p + i + u * stride);
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= v[u];
  }
  for (; i < n16; i += stride) acc ^= ld_stream(p + i);
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) *sink = acc.x;   // keeps the loads alive; practically never taken
}
// take_next: the round about to start uses the candidates the previous round predicted for it
__global__ void set_state_kernel(DevState* ds, int pos, int tok) {
  if (threadIdx.x == 0) { ds->pos = pos; ds->pos_pending = pos; if (tok >= 0) ds->next_tok = tok; }
}
// First launch of every round: the position the previous round (or set_state_kernel) left pending becomes the
// current one; take_next: the round uses the candidates the previous round predicted for it
// (host_cand: the candidates' copy in pinned host memory, for the round's record)
__global__ void begin_round_kernel(DevState* ds, int take_next, int32_t* host_cand) {
  if (threadIdx.x == 0) ds->pos = ds->pos_pending;
  if (take_next && threadIdx.x < MAXM) {
    const int32_t c = ds->cand_next[threadIdx.x];
    ds->cand[threadIdx.x] = c;
    host_cand[threadIdx.x] = c;
  }
}
#endif

// ------------------------------------------------------------------ embedding
// Row set-up (start of the main process, start of every sub-process): h_0 = E[token] (+ P[pos]).
struct EmbedArgs {
  const void* tok_emb; const void* pos_emb;   // pos_emb null for RoPE models
  const int32_t* ids;   // DEVICE: token id of row r is ids[r]
  const DevState* ds;
  float* h;             // [rows][d_model]
  int rows, d_model, pos_off;   // the rows sit at position ds->pos + pos_off (+ r * pos_step for row r)
  int pos_step;
  int vocab;            // rows of tok_emb
};
// An id outside the vocabulary can only come out of a selection over logits that are not numbers (every comparison
// with a NaN fails, and the "nothing found" id stays): it must never become an address.
__device__ __forceinline__ int id_in_vocab(int id, int vocab) { return (unsigned)id < (unsigned)vocab ? id : 0; }
template <typename WT>
__device__ __forceinline__ void embed_rows(const EmbedArgs& a, int r, int i0, int stride) {
  const int tok = id_in_vocab(a.ids[r], a.vocab);
  int pos = a.ds->pos + a.pos_off + r * a.pos_step;
  for (int i = i0; i < a.d_model; i += stride) {
    float v = WTr<WT>::load1(a.tok_emb, (size_t)tok * a.d_model + i);
    if (a.pos_emb) v += WTr<WT>::load1(a.pos_emb, (size_t)pos * a.d_model + i);
    a.h[(size_t)r * a.d_model + i] = v;
  }
}
template <typename WT>
__global__ void embed_kernel(EmbedArgs a) {
  embed_rows<WT>(a, blockIdx.y, blockIdx.x * blockDim.x + threadIdx.x, gridDim.x * blockDim.x);
}

// ------------------------------------------------------------------ skinny GEMM
// Y[m][n] = epilogue( sum_k norm(X)[m][k] * W[n][k] ), M <= 8 rows per group.
// The layer forward of the main process and of the sub-processes (Algorithm 2);
// the sub-processes' k rows share one pass over their layer's weights.
//
// A workgroup requests its group's input rows, then the first three register
// batches of its weight rows, and only then normalises the rows and puts them
// in LDS: a wave's loads return in order, so the rows arrive first and the
// weights stream in behind them.  Its four waves each take sets of weight rows,
// read with 16-byte non-temporal loads three batches ahead of the arithmetic.
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
  int KC;           // K elements staged in LDS at a time (multiple of the batch span (8/WR)*64*VEC)
  int topk;         // > 0: LM-head launch; every workgroup also writes its own top-k (value, id)
  float* pk_val; int32_t* pk_idx;   // [gridDim.x][MAXM] block candidates (topk > 0)
};

__device__ __forceinline__ float gelu_erf(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752440f)); }
__device__ __forceinline__ float silu(float u) { return u / (1.0f + expf(-u)); }

// WR: weight rows a wave streams together (4, or 2 when the matrix has few rows per wave);
// a register batch is always 8 loads per lane: WR rows x (8 / WR) k-blocks.
template <typename WT, int MT, bool PAIRED, int WR>
__device__ __forceinline__ void gemm_body(const GemmArgs& a, const GemmGroup& G, float* lds) {
  constexpr int VEC = WTr<WT>::VEC;
  constexpr int BK = WAVE * VEC;                 // k elements per block
  constexpr int NBK = GEMM_BATCH / WR;           // k-blocks per batch
  constexpr int SPAN = NBK * BK;                 // k elements per batch
  constexpr int LR = PAIRED ? WR / 2 : WR;       // logical rows per set
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int M = G.M, K = a.K, KC = a.KC;
  float4* xs4 = (float4*)(lds + GEMM_LDS_HDR);  // [MT][KC/4] float4; for VEC == 8 the two halves of every 8-group are split

  const int nsets = (a.ntot + LR - 1) / LR;
  const int nwaves = gridDim.x * GEMM_WAVES;
  const int gw = blockIdx.x * GEMM_WAVES + wave;
  const int nbps = (K + SPAN - 1) / SPAN;                  // batches per set
  const int bpc = KC / SPAN;                               // batches per staged chunk
  const bool single = KC >= K;
  // Sets gw, gw + nwaves, ... belong to this wave.  When the reduction length is staged in
  // chunks the waves of a workgroup meet at barriers, so they all run the same number of sets
  // (a wave without a set left repeats its last one and drops the result).
  const int nmine = gw < nsets ? (nsets - gw + nwaves - 1) / nwaves : 0;
  const int nit = single ? nmine : (nsets + nwaves - 1) / nwaves;
  const int Q = nit * nbps;

  // ---- load side: runs GEMM_AHEAD batches ahead of the arithmetic.  Every request is issued
  // unconditionally (lanes past the end of a row re-read its last 16 bytes and zero them), so
  // the loads of one wave return in a known order and the arithmetic waits for its own batch only.
  const char* wp[WR];
  int l_it = 0, l_b = 0;
  auto set_rows = [&](int it) {
    int s = gw + it * nwaves;
    if (s >= nsets) s = nsets - 1;
#pragma unroll
    for (int r = 0; r < LR; ++r) {
      int n = s * LR + r;
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
  };
  // request batch (l_it, l_b) into buf and move on.  Once the wave has requested all its batches
  // the loads go to the start of the (cache-resident) input row instead: still issued, never used.
  const char* idle = (const char*)(G.X + (lane * 4) % K);
  bool l_done = false;
  auto issue_next = [&](u32x4 (&buf)[NBK][WR]) {
#pragma unroll
    for (int j = 0; j < NBK; ++j) {
      const int k = l_b * SPAN + j * BK + lane * VEC;
      const int kcl = k < K ? k : K - VEC;
#pragma unroll
      for (int r = 0; r < WR; ++r) buf[j][r] = ld_stream(l_done ? idle : wp[r] + (size_t)kcl * sizeof(WT));
    }
    if (l_b + 1 < nbps) ++l_b;
    else if (l_it + 1 < nit) { l_b = 0; ++l_it; set_rows(l_it); }
    else l_done = true;
  };
  // zero what lies past the end of the row
  auto mask_tail = [&](int c_b, u32x4 (&buf)[NBK][WR]) {
#pragma unroll
    for (int j = 0; j < NBK; ++j) {
      const bool ok = c_b * SPAN + j * BK + lane * VEC < K;
#pragma unroll
      for (int r = 0; r < WR; ++r)
        if (!ok) buf[j][r] = (u32x4){0u, 0u, 0u, 0u};
    }
  };

  float* stat = lds;                  // mu[MAXM], rstd[MAXM]
  float* redA = lds + 16;             // [MAXM][GEMM_WAVES] partial sums
  float* redB = lds + 48;             // [MAXM][GEMM_WAVES] partial sums of squared deviations
  u32x4 b0[NBK][WR], b1[NBK][WR], b2[NBK][WR], b3[NBK][WR];
  set_rows(0);

  // Norm statistics use one fixed order per row whatever the tile shape: thread t owns the
  // elements k = 4t + 1024 j (+0..3), sums them for j = 0, 1, ... in turn, then a butterfly
  // inside each wave, then the four wave sums in index order.  LayerNorm: mean first, then
  // the squared deviations.
  auto combine4 = [&](const float* r) { return ((r[0] + r[1]) + r[2]) + r[3]; };
  constexpr int XR = GEMM_X_FLOATS / (GEMM_THREADS * 4);   // float4 registers per thread that hold the whole tile
  if (single) {
    // The whole reduction length fits the tile.  Memory returns a wave's loads in order, so the
    // input rows (and gains) are requested first, the weight batches right behind them, and
    // everything up to the staged tile then only waits for the rows.
    const int spr = KC >> 10;              // float4 slots per row per thread
    float4 xr[XR];
#pragma unroll
    for (int i = 0; i < XR; ++i) {
      xr[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      const int m = i / spr, kk = (i - m * spr) * 1024 + tid * 4;
      if (m < M && kk < K) xr[i] = *(const float4*)(G.X + (size_t)m * a.ldx + kk);
    }
    issue_next(b0);
    issue_next(b1);
    issue_next(b2);
    if (a.norm >= 0) {
      if (a.norm == 0) {
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          float sm = 0.f;
#pragma unroll
          for (int i = 0; i < XR; ++i)
            if (i / spr == m) { sm += xr[i].x; sm += xr[i].y; sm += xr[i].z; sm += xr[i].w; }
          sm = wave_sum(sm);
          if (lane == 0) redA[m * GEMM_WAVES + wave] = sm;
        }
        __syncthreads();
      }
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        const float mu = a.norm == 0 ? combine4(redA + m * GEMM_WAVES) / (float)K : 0.f;
        float s2 = 0.f;
#pragma unroll
        for (int i = 0; i < XR; ++i)
          if (i / spr == m && (i - m * spr) * 1024 + tid * 4 < K) {
            float d0 = xr[i].x - mu, d1 = xr[i].y - mu, d2 = xr[i].z - mu, d3 = xr[i].w - mu;
            s2 = fmaf(d0, d0, s2); s2 = fmaf(d1, d1, s2); s2 = fmaf(d2, d2, s2); s2 = fmaf(d3, d3, s2);
          }
        s2 = wave_sum(s2);
        if (lane == 0) redB[m * GEMM_WAVES + wave] = s2;
        if (tid == 0) stat[m] = mu;
      }
      __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < XR; ++i) {
      const int m = i / spr, kk = (i - m * spr) * 1024 + tid * 4;
      if (m >= M) continue;
      float4 v = xr[i];
      if (a.norm >= 0 && kk < K) {
        const float mu = stat[m];
        const float rs = 1.0f / sqrtf(combine4(redB + m * GEMM_WAVES) / (float)K + a.eps);
        float xv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float t = (xv[e] - mu) * rs * WTr<WT>::load1(G.ng, kk + e);
          if (G.nb) t += WTr<WT>::load1(G.nb, kk + e);
          xv[e] = t;
        }
        v = make_float4(xv[0], xv[1], xv[2], xv[3]);
      }
      int slot = (VEC == 8) ? (((kk & 7) >> 2) * (KC >> 3) + (kk >> 3)) : (kk >> 2);
      xs4[m * (KC >> 2) + slot] = v;       // beyond K: zeros (the weights there are zero too)
    }
    __syncthreads();
  } else {
    // The reduction length is staged chunk by chunk.  Statistics first (same order as above).
    if (a.norm >= 0) {
      if (a.norm == 0) {
        for (int m = 0; m < M; ++m) {
          const float* x = G.X + (size_t)m * a.ldx;
          float sm = 0.f;
          for (int i = tid * 4; i < K; i += 1024) {
            float4 v = *(const float4*)(x + i);
            sm += v.x; sm += v.y; sm += v.z; sm += v.w;
          }
          sm = wave_sum(sm);
          if (lane == 0) redA[m * GEMM_WAVES + wave] = sm;
        }
        __syncthreads();
      }
      for (int m = 0; m < M; ++m) {
        const float* x = G.X + (size_t)m * a.ldx;
        const float mu = a.norm == 0 ? combine4(redA + m * GEMM_WAVES) / (float)K : 0.f;
        float s2 = 0.f;
        for (int i = tid * 4; i < K; i += 1024) {
          float4 v = *(const float4*)(x + i);
          float d0 = v.x - mu, d1 = v.y - mu, d2 = v.z - mu, d3 = v.w - mu;
          s2 = fmaf(d0, d0, s2); s2 = fmaf(d1, d1, s2); s2 = fmaf(d2, d2, s2); s2 = fmaf(d3, d3, s2);
        }
        s2 = wave_sum(s2);
        if (lane == 0) redB[m * GEMM_WAVES + wave] = s2;
        if (tid == 0) stat[m] = mu;
      }
      __syncthreads();
      if (tid < M) stat[MAXM + tid] = 1.0f / sqrtf(combine4(redB + tid * GEMM_WAVES) / (float)K + a.eps);
      // (the barrier in front of the first chunk's staging publishes stat[])
    }
    issue_next(b0);
    issue_next(b1);
    issue_next(b2);
  }
  // chunked mode: x rows [k0, k0 + KC) -> LDS, normalised when the launch fuses a norm
  auto stage = [&](int k0) {
    const int kc = (K - k0) < KC ? (K - k0) : KC;          // valid elements, multiple of VEC (>= 4)
    for (int idx = tid * 4; idx < M * KC; idx += GEMM_THREADS * 4) {
      int m = idx / KC, kk = idx - m * KC;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);          // zero tail: weights beyond K are zero too
      if (kk < kc) {
        v = *(const float4*)(G.X + (size_t)m * a.ldx + k0 + kk);
        if (a.norm >= 0) {
          float mu = stat[m], rs = stat[MAXM + m];
          float xv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float t = (xv[e] - mu) * rs * WTr<WT>::load1(G.ng, k0 + kk + e);
            if (G.nb) t += WTr<WT>::load1(G.nb, k0 + kk + e);
            xv[e] = t;
          }
          v = make_float4(xv[0], xv[1], xv[2], xv[3]);
        }
      }
      int slot = (VEC == 8) ? (((kk & 7) >> 2) * (KC >> 3) + (kk >> 3)) : (kk >> 2);
      xs4[m * (KC >> 2) + slot] = v;
    }
  };

  float acc[WR][MT];
#pragma unroll
  for (int r = 0; r < WR; ++r)
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[r][m] = 0.f;
  float* hlog = lds + GEMM_LDS_HDR + (size_t)MT * KC;   // [HEAD_MAX_ROWS] logits of this workgroup (topk launches)
  float pb[WR], prs[LR][MT];                            // bias and residual of the current set

  // arithmetic of batch q (held in cur)
  auto step = [&](int q, u32x4 (&cur)[NBK][WR]) {
    const int c_it = q / nbps, c_b = q - c_it * nbps;
    if (!single && (c_b % bpc) == 0) {
      __syncthreads();
      stage(c_b * SPAN);
      __syncthreads();
    }
    if (c_b == nbps - 1) mask_tail(c_b, cur);
    if (c_b == 0) {
      // bias and residual of this set's outputs: requested now, needed after the set's last batch
      const int s0 = gw + c_it * nwaves;
#pragma unroll
      for (int r = 0; r < LR; ++r) {
        int n = s0 * LR + r;
        if (n >= a.ntot) n = a.ntot - 1;
        if (PAIRED) {
          pb[2 * r] = G.B[0] ? WTr<WT>::load1(G.B[0], n) : 0.f;
          pb[2 * r + 1] = G.B[1] ? WTr<WT>::load1(G.B[1], n) : 0.f;
        } else {
          int seg = 0, loc = n;
          if (loc >= a.N[0]) { loc -= a.N[0]; seg = 1; if (loc >= a.N[1]) { loc -= a.N[1]; seg = 2; } }
          pb[r] = G.B[seg] ? WTr<WT>::load1(G.B[seg], loc) : 0.f;
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) prs[r][m] = (G.Rsd && m < M) ? G.Rsd[(size_t)m * a.ldy + n] : 0.f;
      }
    }
    const int k0 = single ? 0 : (c_b / bpc) * KC;
#pragma unroll
    for (int j = 0; j < NBK; ++j) {
      const int kl = c_b * SPAN + j * BK + lane * VEC - k0;    // < KC
      float xf[MT][VEC];
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        if (m < M) {
          float4 lo = xs4[m * (KC >> 2) + (VEC == 8 ? (kl >> 3) : (kl >> 2))];
          xf[m][0] = lo.x; xf[m][1] = lo.y; xf[m][2] = lo.z; xf[m][3] = lo.w;
          if constexpr (VEC == 8) {
            float4 hi = xs4[m * (KC >> 2) + (KC >> 3) + (kl >> 3)];
            xf[m][4] = hi.x; xf[m][5] = hi.y; xf[m][6] = hi.z; xf[m][7] = hi.w;
          }
        } else {
#pragma unroll
          for (int e = 0; e < VEC; ++e) xf[m][e] = 0.f;
        }
      }
#pragma unroll
      for (int r = 0; r < WR; ++r) {
        float wf[VEC];
        WTr<WT>::unpack(cur[j][r], wf);
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
          for (int e = 0; e < VEC; ++e) acc[r][m] = fmaf(xf[m][e], wf[e], acc[r][m]);
      }
    }
    if (c_b == nbps - 1) {
      // the set is complete: cross-lane reduction and epilogue
#pragma unroll
      for (int r = 0; r < WR; ++r)
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[r][m] = wave_sum(acc[r][m]);
      const int s = gw + c_it * nwaves;
      if (lane == 0 && c_it < nmine) {
#pragma unroll
        for (int r = 0; r < LR; ++r) {
          int n = s * LR + r;
          if (n >= a.ntot) continue;
#pragma unroll
          for (int m = 0; m < MT; ++m) {
            if (m >= M) continue;
            float y;
            if (PAIRED) {
              y = silu(acc[2 * r][m] + pb[2 * r]) * (acc[2 * r + 1][m] + pb[2 * r + 1]);
            } else {
              y = acc[r][m] + pb[r];
              if (a.act == 1) y = gelu_erf(y);
              else if (a.act == 2) y = fmaxf(y, 0.f);
            }
            y += prs[r][m];
            G.Y[(size_t)m * a.ldy + n] = y;
            if (a.topk > 0 && m == 0) hlog[(c_it * GEMM_WAVES + wave) * LR + r] = y;
          }
        }
      }
#pragma unroll
      for (int r = 0; r < WR; ++r)
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[r][m] = 0.f;
    }
  };
  // one request and one batch of arithmetic per step, buffers rotating
  int q = 0;
  for (; q + 4 <= Q; q += 4) {
    issue_next(b3); step(q, b0);
    issue_next(b0); step(q + 1, b1);
    issue_next(b1); step(q + 2, b2);
    issue_next(b2); step(q + 3, b3);
  }
  if (q < Q) { issue_next(b3); step(q, b0); }
  if (q + 1 < Q) { issue_next(b0); step(q + 1, b1); }
  if (q + 2 < Q) { issue_next(b1); step(q + 2, b2); }

  // ---- LM head: this workgroup's top-k by (logit descending, id ascending)
  if (a.topk > 0) {
    __syncthreads();
    if (wave == 0) {
      // entry e = (it*4 + w)*LR + r  <->  vocabulary id ((blockIdx.x*4 + w) + it*nwaves)*LR + r
      constexpr int EPL = HEAD_MAX_ROWS / WAVE;
      float ev[EPL]; int ei[EPL];
      const int nent = nit * GEMM_WAVES * LR;
#pragma unroll
      for (int u = 0; u < EPL; ++u) {
        int e = lane + u * WAVE;
        ev[u] = -INFINITY; ei[u] = 0x7fffffff;
        if (e < nent) {
          int r = e % LR, t = e / LR, w = t % GEMM_WAVES, it = t / GEMM_WAVES;
          int id = ((blockIdx.x * GEMM_WAVES + w) + it * nwaves) * LR + r;
          if (id < a.ntot) { ev[u] = hlog[e]; ei[u] = id; }
        }
      }
      for (int r = 0; r < a.topk; ++r) {
        float v = -INFINITY; int i = 0x7fffffff;
#pragma unroll
        for (int u = 0; u < EPL; ++u) if (better(ev[u], ei[u], v, i)) { v = ev[u]; i = ei[u]; }
        wave_best(v, i);
#pragma unroll
        for (int u = 0; u < EPL; ++u) if (ei[u] == i) { ev[u] = -INFINITY; ei[u] = 0x7fffffff; }
        if (lane == 0) { a.pk_val[blockIdx.x * MAXM + r] = v; a.pk_idx[blockIdx.x * MAXM + r] = i; }
      }
    }
  }
}

// MA rows in group 0, MB rows in group 1 (MB == 0: single-group launch)
template <typename WT, int MA, int MB, bool PAIRED, int WR>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_kernel(GemmArgs a) {
  extern __shared__ float4 lds4[];
  float* lds = (float*)lds4;
  if (MB == 0 || blockIdx.y == 0) gemm_body<WT, MA, PAIRED, WR>(a, a.g[0], lds);
  else gemm_body<WT, (MB < 1 ? 1 : MB), PAIRED, WR>(a, a.g[1], lds);
}

// ------------------------------------------------------------------ attention
// Decode attention of one token per row over the layer's cached positions
// [0, p) plus the row's own position p.  The rows of a group share p and the
// cached prefix (the sub-processes all extend x_<=t by one candidate); each
// row has its own key/value for position p, which this kernel also rotates
// (RoPE) and stores: at cache position p for the main token, in the row's
// tail slot for a candidate.
//
// Keys and values are cached in fp32, in blocks that are operands of
// v_mfma_f32_16x16x4_f32 as they lie in memory.  A block holds 16 positions of
// one head; inside it, for each group s of 16 components, 64 lanes x 4 floats:
//   keys:   lane i + 16 c, float u = K[position i]        [component 16 s + 4 c + u]
//   values: lane i + 16 c, float u = V[position 4 c + u]  [component 16 s + i]
// so a wave reads one kilobyte per load, and one such register quadruple feeds
// four MFMAs: scores = K q (rows: positions, columns: the group's token rows,
// reduction over components) and outputs = V^T p (rows: components, reduction
// over positions).  No shuffles, and up to 16 rows cost what one costs.
//
// A workgroup takes one head and one chunk of 64 positions, one block per
// wave.  Request order (a wave's loads return in order): the rows' own q, k, v
// (direct to LDS) and the rotation table first, then the block's keys, then
// its values.
constexpr int KV_BLOCK = 16;
__host__ __device__ inline size_t kv_blocks(int max_ctx) { return (size_t)((max_ctx + ATT_CHUNK - 1) / ATT_CHUNK) * (ATT_CHUNK / KV_BLOCK); }
// float index inside one head's cache
__host__ __device__ inline size_t k_index(int pos, int comp, int HD) {
  return (((size_t)(pos >> 4) * (HD / 16) + (comp >> 4)) * 64 + (pos & 15) + 16 * ((comp >> 2) & 3)) * 4 + (comp & 3);
}
__host__ __device__ inline size_t v_index(int pos, int comp, int HD) {
  return (((size_t)(pos >> 4) * (HD / 16) + (comp >> 4)) * 64 + (comp & 15) + 16 * ((pos >> 2) & 3)) * 4 + (pos & 3);
}

struct AttnGroup {
  const float* qkv;     // [M][3*d_model]: q | k | v as produced by the QKV projection
  float* Kc; float* Vc; // this layer's cache: [H][blocks][HD/16][64][4]
  float* tailK; float* tailV;   // own_cache == 0: destination of the rows' own key/value, [M][H][HD]
  float* part;          // [M][H][nchunk_max][hd+2] partial (unnormalised o, max, sum)
  int pos_off;          // the rows sit at position p = ds->pos + pos_off and attend to cached positions [0, p)
  int own_cache;        // the row's own key/value go to cache position p (one row only)
  int M;                // rows, 1..16
  int causal;           // prompt chunk: row m sits at position p + m and attends to [0, p + m); the keys and
                        // values of all rows are in the cache already (chunk_kv_kernel), nothing is stored here
};
struct AttnArgs {
  AttnGroup g[2];
  const DevState* ds;
  const float2* rope;   // [max_ctx][hd/2] (cos, sin) or null
  int H, d_model, max_ctx, nchunk_max;
  float scale;
};

template <int HD> __host__ __device__ constexpr int attn_lds_floats(int M) {
  // raw q|k|v and, later, the wave partials in the same place (the raw rows are done with after the rotation),
  // then q (scaled), own k, own v, scores, statistics (max, sum, own weight, -)
  return M * (ATT_WAVES * HD + 3 * HD + ATT_CHUNK + 4);
}

template <int HD, bool CAUSAL = false>
__global__ __launch_bounds__(ATT_THREADS) void attn_kernel(AttnArgs a) {
  extern __shared__ float4 lds4[];
  float* lds = (float*)lds4;
  const AttnGroup& G = a.g[blockIdx.z];
  constexpr int NS = HD / 16, half = HD / 2;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int h = blockIdx.y, c = blockIdx.x;
  const int p = a.ds->pos + G.pos_off, M = G.M;
  const int j0 = c * ATT_CHUNK;
  if (j0 > p + (CAUSAL ? M - 1 : 0)) return;
  // position of row m; whether this chunk holds it; whether the chunk lies before or at it at all
  auto pos_of = [&](int m) { return CAUSAL ? p + m : p; };
  auto owns = [&](int m) { const int pm = pos_of(m); return pm >= j0 && pm < j0 + ATT_CHUNK; };
  auto live = [&](int m) { return !CAUSAL || j0 <= pos_of(m); };
  static_assert(ATT_WAVES >= 3, "the wave partials reuse the raw rows' place");
  float* raw = lds;                   // [M][3][HD]
  float* ored = lds;                  // [ATT_WAVES][M][HD], written only after the barriers that follow the rotation
  float* qs = lds + M * ATT_WAVES * HD;   // [M][HD]
  float* ko = qs + M * HD;            // [M][HD]
  float* vo = ko + M * HD;            // [M][HD]
  float* sc = vo + M * HD;            // [M][ATT_CHUNK]
  float* st = sc + M * ATT_CHUNK;     // [M][4]

  // own q, k, v of every row, as they are: kilobyte pieces of the [M][3][HD] image
  {
    const int nfl = M * 3 * HD;
    for (int f0 = wave * 256; f0 < nfl; f0 += ATT_WAVES * 256) {
      const int f = f0 + lane * 4;
      if (f < nfl) {
        const int m = f / (3 * HD), r = f - m * (3 * HD), sec = r / HD, i = r - sec * HD;
        dma16(G.qkv + (size_t)m * 3 * a.d_model + (size_t)sec * a.d_model + (size_t)h * HD + i, raw + f0);
      }
    }
  }
  // rotation pair of this thread's component (the same for every row)
  const int ci = tid % HD;
  float2 cz = make_float2(1.f, 0.f);
  if (a.rope) cz = a.rope[(size_t)p * half + (ci < half ? ci : ci - half)];
  // this wave's block: keys, then values
  const size_t hb = (size_t)h * kv_blocks(a.max_ctx) + (size_t)(c * (ATT_CHUNK / KV_BLOCK) + wave);
  const char* kb = (const char*)G.Kc + hb * (NS * 1024) + lane * 16;
  const char* vb = (const char*)G.Vc + hb * (NS * 1024) + lane * 16;
  f32x4_t kreg[NS], vreg[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) kreg[s] = __builtin_nontemporal_load((const f32x4_t*)(kb + s * 1024));
#pragma unroll
  for (int s = 0; s < NS; ++s) vreg[s] = __builtin_nontemporal_load((const f32x4_t*)(vb + s * 1024));

  // the rows' own loads have arrived once only the 2 NS block loads are outstanding
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * NS) : "memory");
  // rotate, scale, store the rows' own key and value
  for (int idx = tid; idx < M * HD; idx += ATT_THREADS) {
    const int m = idx / HD, i = idx - m * HD;     // i == ci: ATT_THREADS is a multiple of HD
    const float* r = raw + m * 3 * HD;
    float q = r[i], k = r[HD + i];
    const float v = r[2 * HD + i];
    if (CAUSAL && a.rope) cz = a.rope[(size_t)pos_of(m) * half + (i < half ? i : i - half)];
    if (a.rope) {
      const int ip = i < half ? i + half : i - half;
      const float qo = r[ip], kk = r[HD + ip];
      if (i < half) { q = fmaf(q, cz.x, -(qo * cz.y)); k = fmaf(k, cz.x, -(kk * cz.y)); }
      else          { q = fmaf(q, cz.x, qo * cz.y);    k = fmaf(k, cz.x, kk * cz.y); }
    }
    qs[m * HD + i] = q * a.scale;
    ko[m * HD + i] = k;
    vo[m * HD + i] = v;
  }
  __syncthreads();

  // scores of the block's 16 positions: lane l = n + 16 c feeds column n (row n of the group; lanes
  // past M repeat row 0, their columns are never read) and components 16 s + 4 c + u
  const int bn = lane & 15, bc = lane >> 4;
  const int bm = bn < M ? bn : 0;
  {
    f32x4_t sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const f32x4_t q4 = *(const f32x4_t*)(qs + bm * HD + 16 * s + 4 * bc);
#pragma unroll
      for (int u = 0; u < 4; ++u) sacc = __builtin_amdgcn_mfma_f32_16x16x4f32(kreg[s][u], q4[u], sacc, 0, 0, 0);
    }
    // sacc[jj]: position 16 wave + 4 bc + jj of the chunk, row bn.  Cached positions keep their score,
    // later ones get -inf, the rows' own position is filled in below.
    if (bn < M) {
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int jl = 16 * wave + 4 * bc + jj, j = j0 + jl, pm = pos_of(bn);
        if (j != pm) sc[bn * ATT_CHUNK + jl] = j < pm ? sacc[jj] : -INFINITY;
      }
    }
  }
  {
    for (int m = wave; m < M; m += ATT_WAVES) {
      if (!owns(m)) continue;
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < HD / WAVE; ++e) s = fmaf(qs[m * HD + lane + e * WAVE], ko[m * HD + lane + e * WAVE], s);
      s = wave_sum(s);
      if (lane == 0) sc[m * ATT_CHUNK + (pos_of(m) - j0)] = s;
    }
  }
  __syncthreads();
  // chunk-local softmax numerators: one wave per row, one position per lane
  for (int m = wave; m < M; m += ATT_WAVES) {
    if (!live(m)) continue;      // (the chunk lies past this row: its scores are not used and nothing is written for it)
    const float v = sc[m * ATT_CHUNK + lane];
    const float mx = wave_max(v);
    const float e = expf(v - mx);
    const float sum = wave_sum(e);
    const bool own = owns(m) && lane == pos_of(m) - j0;
    sc[m * ATT_CHUNK + lane] = own ? 0.f : e;       // the own position is added outside the MFMAs
    if (own) st[m * 4 + 2] = e;
    if (lane == 0) { st[m * 4] = mx; st[m * 4 + 1] = sum; }
  }
  __syncthreads();
  // weighted values of the block: rows = components 16 s + i, reduction over its 16 positions 4 c + u
  {
    const f32x4_t p4 = *(const f32x4_t*)(sc + bm * ATT_CHUNK + 16 * wave + 4 * bc);
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      f32x4_t oacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int u = 0; u < 4; ++u) oacc = __builtin_amdgcn_mfma_f32_16x16x4f32(vreg[s][u], p4[u], oacc, 0, 0, 0);
      // oacc[jj]: component 16 s + 4 bc + jj, row bn
      if (bn < M) *(f32x4_t*)(ored + (wave * M + bn) * HD + 16 * s + 4 * bc) = oacc;
    }
  }
  __syncthreads();
  // the four blocks in wave order, then the rows' own position
  for (int idx = tid; idx < M * HD; idx += ATT_THREADS) {
    const int m = idx / HD, i = idx - m * HD;
    if (!live(m)) continue;
    const bool owns_p = owns(m);
    float o = ored[(0 * M + m) * HD + i];
#pragma unroll
    for (int w = 1; w < ATT_WAVES; ++w) o += ored[(w * M + m) * HD + i];
    if (owns_p) o = fmaf(st[m * 4 + 2], vo[m * HD + i], o);
    float* dst = G.part + (((size_t)m * a.H + h) * a.nchunk_max + c) * (HD + 2);
    dst[i] = o;
    if (i == 0) { dst[HD] = st[m * 4]; dst[HD + 1] = st[m * 4 + 1]; }
    // the row's own key and value (stored last: no store waits in the request queue behind the block loads)
    if (owns_p && !CAUSAL) {
      if (G.own_cache) {
        const size_t base = (size_t)h * kv_blocks(a.max_ctx) * (KV_BLOCK * HD);
        G.Kc[base + k_index(p, i, HD)] = ko[m * HD + i];
        G.Vc[base + v_index(p, i, HD)] = vo[m * HD + i];
      } else {
        const size_t d = ((size_t)m * a.H + h) * HD + i;
        G.tailK[d] = ko[m * HD + i];
        G.tailV[d] = vo[m * HD + i];
      }
    }
  }
}

// Prompt chunk: rows m = 0..M-1 sit at consecutive positions p + m.  Their keys (rotated exactly as the
// attention kernel rotates a row's own key) and values go into the cache before the chunk's attention runs,
// so that every row finds the rows before it there.  One workgroup per (row, head), one thread per component.
struct ChunkKvArgs {
  const float* qkv;     // [M][3*d_model]
  float* Kc; float* Vc; // this layer's cache
  const float2* rope;
  const DevState* ds;
  int HD, d_model, max_ctx;
};
#ifdef PPD_ENGINE_TU
__global__ void chunk_kv_kernel(ChunkKvArgs a) {
  const int m = blockIdx.x, h = blockIdx.y, i = threadIdx.x, HD = a.HD, half = HD / 2;
  const int pos = a.ds->pos + m;
  const float* r = a.qkv + (size_t)m * 3 * a.d_model + (size_t)h * HD;
  float k = r[a.d_model + i];
  const float v = r[2 * a.d_model + i];
  if (a.rope) {
    const float2 cz = a.rope[(size_t)pos * half + (i < half ? i : i - half)];
    const float kk = r[a.d_model + (i < half ? i + half : i - half)];
    if (i < half) k = fmaf(k, cz.x, -(kk * cz.y));
    else          k = fmaf(k, cz.x, kk * cz.y);
  }
  const size_t base = (size_t)h * kv_blocks(a.max_ctx) * (KV_BLOCK * HD);
  a.Kc[base + k_index(pos, i, HD)] = k;
  a.Vc[base + v_index(pos, i, HD)] = v;
}
#endif

// merge of the chunk partials, chunks in index order
struct MergeArgs {
  const float* part[2]; float* out[2];   // out: [M][d_model]
  int pos_off[2]; int M[2];
  int causal[2];       // row m sits m positions further on (prompt chunk)
  const DevState* ds;
  int H, HD, d_model, nchunk_max;
};
#ifdef PPD_ENGINE_TU
constexpr int MERGE_THREADS = 512;
// One workgroup per (row, head, group): thread t = component t % HD, slice t / HD.  Slice s merges the
// chunks s, s + S, s + 2S, ... (S = MERGE_THREADS / HD slices) in that order with a running maximum,
// 16 chunks' loads in flight together; then the slices are merged in slice order.
__global__ __launch_bounds__(MERGE_THREADS) void attn_merge_kernel(MergeArgs a) {
  __shared__ float sm_o[MERGE_THREADS], sl_m[8], sl_l[8];
  const int g = blockIdx.z, h = blockIdx.y, m = blockIdx.x;
  if (m >= a.M[g]) return;
  const int nc = (a.ds->pos + a.pos_off[g] + (a.causal[g] ? m : 0)) / ATT_CHUNK + 1;
  const int S = MERGE_THREADS / a.HD;          // 4 (head_dim 128) or 8 (64)
  const int i = threadIdx.x % a.HD, sl = threadIdx.x / a.HD;
  const float* base = a.part[g] + (((size_t)m * a.H + h) * a.nchunk_max) * (a.HD + 2);
  const size_t cs = a.HD + 2;
  constexpr int UB = 16;    // chunks whose loads are in flight together
  float mx = -INFINITY, o = 0.f, l = 0.f;
  for (int c0 = sl; c0 < nc; c0 += UB * S) {
    float tm[UB], ts[UB], to[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      const int c = c0 + u * S;
      const float* pc = base + (size_t)(c < nc ? c : c0) * cs;
      tm[u] = pc[a.HD]; ts[u] = pc[a.HD + 1]; to[u] = pc[i];
    }
    float bm = mx;
#pragma unroll
    for (int u = 0; u < UB; ++u) if (c0 + u * S < nc) bm = fmaxf(bm, tm[u]);
    const float rescale = expf(mx - bm);     // 0 for the first batch (mx = -inf), 1 when the maximum stays
    o *= rescale; l *= rescale; mx = bm;
#pragma unroll
    for (int u = 0; u < UB; ++u)
      if (c0 + u * S < nc) {
        const float w = expf(tm[u] - mx);
        o = fmaf(w, to[u], o);
        l = fmaf(w, ts[u], l);
      }
  }
  // slices in order; a slice without chunks has mx = -inf and weight 0
  sm_o[threadIdx.x] = o;
  if (i == 0) { sl_m[sl] = mx; sl_l[sl] = l; }
  __syncthreads();
  if (sl == 0) {
    float gm = -INFINITY;
    for (int q = 0; q < S; ++q) gm = fmaxf(gm, sl_m[q]);
    float oo = 0.f, ll = 0.f;
    for (int q = 0; q < S; ++q) {
      const float w = expf(sl_m[q] - gm);     // exp(-inf) = 0 for an empty slice
      oo = fmaf(w, sm_o[q * a.HD + i], oo);
      ll = fmaf(w, sl_l[q], ll);
    }
    a.out[g][(size_t)m * a.d_model + (size_t)h * a.HD + i] = oo / ll;
  }
}
#endif

// ------------------------------------------------------------------ selection
// Early prediction: top-k of the early logits by (logit descending, id ascending); the head GEMM
// leaves every workgroup's own top-k, this kernel merges them and sets up the k candidate rows
// (Algorithm 2: the early top-k and its hand-out to the sub-processes -- here: their embedding rows).
// Final prediction: arg max of the final logits (ties to the lowest id), verification against the
// early candidates (Algorithm 2's comparison of each candidate with the final token), then adoption:
// on a match the matching candidate's hidden row becomes the main row and its key/value tails of layers
// 1..d-dbar become cache position t+1; without a match nothing is copied and the tails are overwritten
// by the next round.
// Appendix B's sampling-based variants replace only the arg max: the token verified here is then the one
// drawn by top-k sampling (inside this kernel, from the merged lists) or by the sampling kernel (top-p).
struct SelectArgs {
  const float* pk_val; const int32_t* pk_idx;   // [nblk][MAXM] block candidates, first kk of each valid
  int nblk; int kk;     // kk = k (early) or 1 (final)
  int k;
  int mode;             // 0: early top-k -> cand[0..k) + embed; 1: final arg max + verify + adopt
  DevState* ds;
  int32_t* host_result; // device-visible pinned host memory: [0] token, [1] match_idx (mode 1), [2..2+k) candidates (mode 0),
                        // [2 + MAXM] number of finished rounds, written after the rest (mode 1): the host polls it
  EmbedArgs emb;        // candidate rows (mode 0)
  // adoption (mode 1)
  float* h;                 // [1+k][d_model]: row 0 main, rows 1.. candidates
  const float* tailK; const float* tailV;   // [nb][k][H][hd]
  float* Kc; float* Vc;     // [L][H][blocks][hd/16][64][4]
  size_t head_floats;       // floats of one head's cache
  int nb, H, hd, d_model, max_ctx;
  // speculative early prediction (mode 1, exit layer d/2, early head = LM head): the head pass that made the
  // final logits of row 0 also made, for every candidate row, the early logits of the next round (the
  // candidate's state after d/2 layers is that round's exit-layer state).  On a match the matching row's
  // top-k become the next candidates here and now, and the next round starts with its parallel phase.
  int spec;
  int pk_stride;            // block lists of row m start at (m * pk_stride) * MAXM
  const float* spec_logits; // [k][vocab] logits of the candidate rows
  float* early_spec;        // [2][vocab]: the matching row's logits are kept as the early logits of the round at
                            // the next position, in the half that position's parity selects
  int vocab;
  int sampled;              // mode 1: the final prediction is ds->sampled (drawn by sample_kernel), not the arg max
  // mode 1, top-k sampling with samp_topk <= kk kept tokens: they are the head of the merged block lists, so the
  // draw happens here (fp64 inversion over the samp_topk best in ranking order, same uniform as sample_kernel)
  int samp_topk;
  uint64_t samp_seed;
};
// ------------------------------------------------------------------ sampling-based final prediction
// Appendix B: the final prediction is drawn by top-k or top-p sampling instead of the arg max; the rest of a
// round is unchanged.  One workgroup draws the token by inversion from the fp32 logits, in fp64: tokens are
// ranked by (logit descending, id ascending), w_i = exp(z_i - z_max); top-k sampling keeps the ks first of the
// ranking, top-p the shortest prefix whose mass reaches p times the total; with W the kept mass, the token is
// the first of the ranking whose cumulative mass exceeds u W.  u comes from Philox-4x32-10 (Salmon et al.,
// SC 2011) keyed by the seed, counter = sequence position of the token being chosen: decoding with and
// without PPD draws the same numbers.
// No sort: each of the two questions ("where does the kept prefix end", "where does the cumulative mass pass
// u W") asks for the largest key kappa whose mass-at-or-above G(kappa) meets a bound; G is evaluated in full, in
// one fixed order of additions, for one trial key per pass (so it is monotone in the key whatever the rounding),
// and kappa is fixed bit by bit from the top of an order-preserving 32-bit image of the logit.
// ten rounds: two 32x32->64 products, halves crossed over and mixed with counter and key; key steps by the Weyl constants
__device__ inline uint32_t philox4x32_10_word0(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
  for (int r = 0; r < 10; ++r) {
    if (r) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
    const uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = h1 ^ c1 ^ k0, n2 = h0 ^ c3 ^ k1;
    c0 = n0; c1 = l1; c2 = n2; c3 = l0;
  }
  return c0;
}

#ifdef PPD_ENGINE_TU
constexpr int SAMP_THREADS = 1024;
constexpr int SAMP_MEMU = 8;     // loads in flight per thread when the logits are re-read from memory
constexpr int SAMP_VPT = 32;     // logits per thread kept on chip (weights in registers, keys in LDS): vocabularies up to 32768;
                                 // larger ones re-read memory every pass
struct SampleArgs {
  const float* z; int n;     // logits [n]
  int mode, ks;              // 1 top-k sampling (ks kept), 2 top-p sampling
  double p;
  uint64_t seed;
  DevState* ds;              // reads pos, writes sampled
  double* w; uint32_t* keys; // scratch [npad] each (only used when the logits do not fit the chip): weights and keys,
  int npad;                  // zero beyond n; npad = n rounded up to a multiple of SAMP_THREADS * SAMP_MEMU
};

// larger logit <-> larger key; -0 and +0 are one value; no finite or infinite logit has key 0
__device__ inline uint32_t samp_key(float z) {
  const uint32_t b = __float_as_uint(z == 0.f ? 0.f : z);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ inline float samp_unkey(uint32_t k) { return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k); }

template <int CTRL> __device__ __forceinline__ double dpp_f64(double v) {
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)b, CTRL, 0xf, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xf, 0xf, false);
  return __longlong_as_double((long long)(((unsigned long long)(unsigned)hi << 32) | (unsigned)lo));
}
__device__ __forceinline__ double lane_f64(double v, int l) {
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_readlane((int)b, l), hi = __builtin_amdgcn_readlane((int)(b >> 32), l);
  return __longlong_as_double((long long)(((unsigned long long)(unsigned)hi << 32) | (unsigned)lo));
}
__device__ __forceinline__ double wave_sum_f64(double v) {     // same scheme as wave_sum
  v += dpp_f64<0xB1>(v);
  v += dpp_f64<0x4E>(v);
  v += dpp_f64<0x141>(v);
  v += dpp_f64<0x140>(v);
  return ((lane_f64(v, 0) + lane_f64(v, 16)) + lane_f64(v, 32)) + lane_f64(v, 48);
}

template <bool REG>
__global__ __launch_bounds__(SAMP_THREADS) void sample_kernel(SampleArgs a) {
  constexpr int NW = SAMP_THREADS / WAVE;
  constexpr int VPT = REG ? SAMP_VPT : 1;
  __shared__ double s_m[2][NW];
  __shared__ int s_c[2][NW];
  __shared__ float s_redf[NW];
  __shared__ int s_bc[NW][16];
  __shared__ int s_cnt[16];
  __shared__ uint32_t s_prefix; __shared__ int s_need, s_min;
  __shared__ uint32_t s_key[REG ? SAMP_VPT * SAMP_THREADS : 1];     // key of token tid + e * SAMP_THREADS at [e][tid]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = a.n;
  uint32_t* const key = s_key + tid;
  constexpr int KS = SAMP_THREADS;     // stride between a thread's keys

  // ---- keys, largest logit, weights
  double wr[VPT];
  float mx = -INFINITY;
  if (REG) {
#pragma unroll
    for (int e = 0; e < VPT; ++e) {
      const int i = tid + e * SAMP_THREADS;
      uint32_t k = 0u;
      if (i < n) { const float z = a.z[i]; k = samp_key(z); mx = fmaxf(mx, z); }
      key[e * KS] = k;
    }
  } else {
    for (int i = tid; i < n; i += SAMP_THREADS) mx = fmaxf(mx, a.z[i]);
  }
  mx = wave_max(mx);
  if (lane == 0) s_redf[wave] = mx;
  __syncthreads();
  mx = s_redf[0];
  for (int w = 1; w < NW; ++w) mx = fmaxf(mx, s_redf[w]);
  const double zmax = (double)mx;
  if (REG) {
#pragma unroll
    for (int e = 0; e < VPT; ++e) { const uint32_t k = key[e * KS]; wr[e] = k ? exp((double)samp_unkey(k) - zmax) : 0.0; }
  } else {
    for (int i = tid; i < a.npad; i += SAMP_THREADS) {
      const bool in = i < n;
      const float z = in ? a.z[i] : 0.f;
      a.keys[i] = in ? samp_key(z) : 0u;
      a.w[i] = in ? exp((double)z - zmax) : 0.0;
    }
    __syncthreads();
  }

  // ---- G(kth): mass and number of the tokens whose key is at least kth (kth >= 1); every thread gets both
  int par = 0;
  auto G = [&](uint32_t kth, double& mass, int& count) {
    double m = 0.0; int c = 0;
    if (REG) {
#pragma unroll
      for (int e = 0; e < VPT; ++e) {
        const bool ge = key[e * KS] >= kth;
        m += ge ? wr[e] : 0.0;
        c += __popcll(__ballot(ge));
      }
    } else {
      for (int i0 = tid; i0 < a.npad; i0 += SAMP_THREADS * SAMP_MEMU) {
        uint32_t k[SAMP_MEMU]; double w[SAMP_MEMU];
#pragma unroll
        for (int q = 0; q < SAMP_MEMU; ++q) { k[q] = a.keys[i0 + q * SAMP_THREADS]; w[q] = a.w[i0 + q * SAMP_THREADS]; }
#pragma unroll
        for (int q = 0; q < SAMP_MEMU; ++q) {
          const bool ge = k[q] >= kth;
          m += ge ? w[q] : 0.0;
          c += __popcll(__ballot(ge));
        }
      }
    }
    m = wave_sum_f64(m);
    if (lane == 0) { s_m[par][wave] = m; s_c[par][wave] = c; }
    __syncthreads();
    mass = 0.0; count = 0;
    for (int w = 0; w < NW; ++w) { mass += s_m[par][w]; count += s_c[par][w]; }
    par ^= 1;        // the next evaluation writes the other half: no second barrier needed
  };
  // ---- the largest key kappa with G(kappa) >= T (kind 0), G(kappa) > T (kind 1) or count(kappa) >= K (kind 2);
  // the bound holds at the smallest key present, so kappa >= 1.  Also the mass and count strictly above kappa
  // and the number of tokens at kappa.
  double S; int n_all;
  G(1u, S, n_all);
  // The keys still in question after bit b are those that agree with the prefix above b; once a single token
  // is left (count at the prefix minus count above the bucket), its key is kappa and the remaining bits need
  // no passes: the mass and count above the bucket are the ones already found.
  auto search = [&](int kind, double T, int K, uint32_t& kappa, double& above, int& nabove, int& ties) {
    uint32_t pre = 0u;
    int c_at = n_all, c_hi = 0, bit = 31;
    double g_hi = 0.0;
    bool single = c_at - c_hi == 1;
    for (; bit >= 0 && !single; --bit) {
      const uint32_t t = pre | (1u << bit);
      double g; int c;
      G(t, g, c);
      const bool ok = kind == 0 ? g >= T : (kind == 1 ? g > T : c >= K);
      if (ok) { pre = t; c_at = c; }
      else { c_hi = c; g_hi = g; }
      single = c_at - c_hi == 1;
    }
    if (single) {
      // bits above `bit` are fixed (the loop has already stepped past the last one it tried)
      const int sh = bit + 1;
      __syncthreads();
      if (REG) {
#pragma unroll
        for (int e = 0; e < VPT; ++e) {
          const uint32_t k = key[e * KS];
          if (k && (sh >= 32 || (k >> sh) == (pre >> sh))) s_prefix = k;
        }
      } else {
        for (int i = tid; i < a.npad; i += SAMP_THREADS) {
          const uint32_t k = a.keys[i];
          if (k && (sh >= 32 || (k >> sh) == (pre >> sh))) s_prefix = k;
        }
      }
      __syncthreads();
      kappa = s_prefix; above = g_hi; nabove = c_hi; ties = 1;
      __syncthreads();
      return;
    }
    kappa = pre;
    above = 0.0; nabove = 0;
    if (kappa != 0xffffffffu) G(kappa + 1u, above, nabove);
    ties = c_at - nabove;
  };
  const int pos_new = a.ds->pos + 1;
  const uint32_t word = philox4x32_10_word0((uint32_t)pos_new, 0u, 0u, 0u, (uint32_t)(a.seed & 0xffffffffu), (uint32_t)(a.seed >> 32));
  const double u = (double)(word >> 8) * (1.0 / 16777216.0);
  uint32_t kappa; double above; int nabove, ties;
  // ---- kept mass W (every thread computes the same numbers)
  double W = S;
  if (a.mode == 1) {
    const int ks = a.ks < 1 ? 1 : a.ks;
    if (ks < n) {
      search(2, 0.0, ks, kappa, above, nabove, ties);
      const double wk = exp((double)samp_unkey(kappa) - zmax);
      W = above;
      for (int r = nabove; r < ks; ++r) W += wk;
    }
  } else {
    const double T = a.p * S;
    search(0, T, 0, kappa, above, nabove, ties);
    const double wk = exp((double)samp_unkey(kappa) - zmax);
    W = above;
    int r = 0;
    do { W += wk; ++r; } while (W < T && r < ties);
  }
  // ---- the first token of the ranking whose cumulative mass exceeds u W: the r-th smallest id among those at kappa
  const double t = u * W;
  search(1, t, 0, kappa, above, nabove, ties);
  int r = 0;
  {
    const double wk = exp((double)samp_unkey(kappa) - zmax);
    double c = above;
    do { c += wk; ++r; } while (!(c > t) && r < ties);
  }
  if (tid == 0) { s_min = 0x7fffffff; s_prefix = 0u; s_need = r; }
  __syncthreads();
  if (r == 1) {
    if (REG) {
#pragma unroll
      for (int e = 0; e < VPT; ++e) if (key[e * KS] == kappa) atomicMin(&s_min, tid + e * SAMP_THREADS);
    } else {
      for (int i = tid; i < n; i += SAMP_THREADS) if (samp_key(a.z[i]) == kappa) atomicMin(&s_min, i);
    }
    __syncthreads();
    if (tid == 0) a.ds->sampled = s_min;
    return;
  }
  // several tokens share the logit and the draw falls past the first of them: the id is fixed four bits at a
  // time from the top (counts of the tied ids per digit, ascending)
  for (int shift = 28; shift >= 0; shift -= 4) {
    __syncthreads();
    const uint32_t prefix = s_prefix;
    int cn[16];
#pragma unroll
    for (int b = 0; b < 16; ++b) cn[b] = 0;
    for (int i = tid; i < n; i += SAMP_THREADS) {
      const bool in = samp_key(a.z[i]) == kappa && (shift == 28 || ((uint32_t)i >> (shift + 4)) == prefix);
      if (in) {
        const int nib = ((uint32_t)i >> shift) & 15;
#pragma unroll
        for (int b = 0; b < 16; ++b) cn[b] += nib == b ? 1 : 0;
      }
    }
#pragma unroll
    for (int b = 0; b < 16; ++b) {
      int c = cn[b];
      for (int o = 32; o >= 1; o >>= 1) c += __shfl_xor(c, o);
      if (lane == 0) s_bc[wave][b] = c;
    }
    __syncthreads();
    if (tid < 16) { int c = 0; for (int w = 0; w < NW; ++w) c += s_bc[w][tid]; s_cnt[tid] = c; }
    __syncthreads();
    if (tid == 0) {
      int need = s_need, pick = 15;
      for (int b = 0; b < 16; ++b) { if (s_cnt[b] >= need) { pick = b; break; } need -= s_cnt[b]; }
      s_need = need; s_prefix = (prefix << 4) | (uint32_t)pick;
    }
  }
  __syncthreads();
  if (tid == 0) a.ds->sampled = (int32_t)s_prefix;
}
#endif

constexpr int SEL_THREADS = 256;

// Merge of the head GEMM's block lists (nblk lists, the first kk entries of each valid, MAXM apart): the best nk
// by (value descending, id ascending) land in win[] / winv[] (shared memory, MAXM entries each; wv / wi: shared
// scratch of one entry per wave).  Called by all SEL_THREADS threads of a workgroup; ends with a barrier.
__device__ __forceinline__ void merge_block_lists(const float* pkv, const int32_t* pki, int nblk, int kk, int nk,
                                                  float* wv, int* wi, int* win, float* winv) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int total = nblk * kk;
  // each thread scans its strided share and keeps its own sorted best MAXM
  float lv[MAXM]; int li[MAXM];
#pragma unroll
  for (int q = 0; q < MAXM; ++q) { lv[q] = -INFINITY; li[q] = 0x7fffffff; }
  for (int e = tid; e < total; e += SEL_THREADS) {
    int b = e / kk, r = e - b * kk;
    float v = pkv[b * MAXM + r]; int i = pki[b * MAXM + r];
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
  int head = 0;
  for (int r = 0; r < nk; ++r) {
    float v = -INFINITY; int i = 0x7fffffff;
#pragma unroll
    for (int q = 0; q < MAXM; ++q) if (q == head) { v = lv[q]; i = li[q]; }
    wave_best(v, i);
    __syncthreads();
    if (lane == 0) { wv[wave] = v; wi[wave] = i; }
    __syncthreads();
    int bw = 0;
#pragma unroll
    for (int w = 1; w < SEL_THREADS / WAVE; ++w) if (better(wv[w], wi[w], wv[bw], wi[bw])) bw = w;
    const int wid = wi[bw];
    if (tid == 0) { win[r] = wid; winv[r] = wv[bw]; }
    int cur = 0x7fffffff;
#pragma unroll
    for (int q = 0; q < MAXM; ++q) if (q == head) cur = li[q];
    if (cur == wid) ++head;     // ids are unique: only the owner of the winner moves on
  }
  __syncthreads();
}

// Stand-alone early prediction: the merged top-k of one row's block lists written out (ids, and values when asked for).
struct TopkMergeArgs {
  const float* pk_val; const int32_t* pk_idx;   // [nblk][MAXM]
  int nblk, kk, k;
  int32_t* ids; float* vals;                    // [k]; vals may be null
};

// every workgroup merges the block candidates redundantly (they are few); winners land in win[]
template <typename WT>
__global__ __launch_bounds__(SEL_THREADS) void select_kernel(SelectArgs a) {
  __shared__ float wv[SEL_THREADS / WAVE];
  __shared__ int wi[SEL_THREADS / WAVE];
  __shared__ int win[MAXM];
  __shared__ float winv[MAXM];
  __shared__ int s_midx, s_tok;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // merge of one row's block lists: the best nk by (value descending, id ascending) land in win[]
  auto merge_row = [&](int prow, int nk) {
    merge_block_lists(a.pk_val + (size_t)prow * a.pk_stride * MAXM, a.pk_idx + (size_t)prow * a.pk_stride * MAXM,
                      a.nblk, a.kk, nk, wv, wi, win, winv);
  };
  merge_row(0, a.mode == 0 ? a.k : (a.samp_topk > 0 ? a.samp_topk : 1));
  if (a.mode == 0) {
    // candidates and their rows; block x handles row blockIdx.y
    if (blockIdx.x == 0 && blockIdx.y == 0 && tid < a.k) { a.ds->cand[tid] = win[tid]; a.host_result[2 + tid] = win[tid]; }
    const int r = blockIdx.y;
    EmbedArgs e = a.emb;
    const int tok = id_in_vocab(win[r], a.vocab);
    int pos = a.ds->pos + e.pos_off;
    for (int i = blockIdx.x * SEL_THREADS + tid; i < e.d_model; i += gridDim.x * SEL_THREADS) {
      float v = WTr<WT>::load1(e.tok_emb, (size_t)tok * e.d_model + i);
      if (e.pos_emb) v += WTr<WT>::load1(e.pos_emb, (size_t)pos * e.d_model + i);
      e.h[(size_t)r * e.d_model + i] = v;
    }
    return;
  }
  // final: verification
  if (a.samp_topk > 0) {
    if (tid == 0) {
      const uint32_t word = philox4x32_10_word0((uint32_t)(a.ds->pos + 1), 0u, 0u, 0u, (uint32_t)(a.samp_seed & 0xffffffffu), (uint32_t)(a.samp_seed >> 32));
      const double u = (double)(word >> 8) * (1.0 / 16777216.0);
      double cum[MAXM], acc = 0.0;
      for (int r = 0; r < a.samp_topk; ++r) { acc += exp((double)winv[r] - (double)winv[0]); cum[r] = acc; }
      const double target = u * acc;
      int pick = a.samp_topk - 1;
      for (int r = a.samp_topk - 1; r >= 0; --r) if (cum[r] > target) pick = r;
      s_tok = win[pick];
    }
    __syncthreads();
  }
  const int token = id_in_vocab(a.samp_topk > 0 ? s_tok : (a.sampled ? a.ds->sampled : win[0]), a.vocab);
  if (tid == 0) {
    int midx = -1;
    for (int q = 0; q < a.k; ++q) if (a.ds->cand[q] == token) { midx = q; break; }
    s_midx = midx;
  }
  __syncthreads();
  const int midx = s_midx;
  if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) {
    a.ds->result[0] = token; a.ds->result[1] = midx; a.ds->next_tok = token;
    a.ds->pos_pending = a.ds->pos + 1;      // the next round's position (its first launch takes it over)
    a.host_result[0] = token; a.host_result[1] = midx;
    // the round's record is complete: let the host see it, then the new count
    const int32_t seq = a.ds->seq + 1;
    a.ds->seq = seq;
    __threadfence_system();
    *(volatile int32_t*)(a.host_result + 2 + MAXM) = seq;
  }
  if (midx < 0 || a.nb == 0) return;
  // adoption: block (l, which), l < nb, copies one layer's K or V tail; block (0,0) also the hidden row.
  // With speculative early prediction the grid has further blocks (l >= nb) that prepare the next round.
  const int l = blockIdx.x;
  const int pos_next = a.ds->pos + 1;
  if (l >= a.nb) {
    if (!a.spec) return;
    const int b = l - a.nb, nblocks = gridDim.x - a.nb;
    if (blockIdx.y == 0) {
      // the matching row's logits are the next round's early logits
      const float* src = a.spec_logits + (size_t)midx * a.vocab;
      float* dst = a.early_spec + (size_t)(pos_next & 1) * a.vocab;
      for (int i = b * SEL_THREADS + tid; i < a.vocab; i += nblocks * SEL_THREADS) dst[i] = src[i];
      return;
    }
    // the next round's candidates: top-k of the matching row's logits; then, column by column (each thread
    // its own columns, so no thread waits for another): the matching row becomes row 0, and the candidates'
    // embeddings become rows 1..k, one position on
    merge_row(1 + midx, a.k);
    if (b == 0 && tid < a.k) a.ds->cand_next[tid] = win[tid];
    const EmbedArgs e = a.emb;
    const int pos2 = pos_next + 1;
    for (int i = b * SEL_THREADS + tid; i < a.d_model; i += nblocks * SEL_THREADS) {
      a.h[i] = a.h[(size_t)(1 + midx) * a.d_model + i];
      if (pos2 < a.max_ctx)
        for (int r = 0; r < a.k; ++r) {
          float v = WTr<WT>::load1(e.tok_emb, (size_t)id_in_vocab(win[r], a.vocab) * e.d_model + i);
          if (e.pos_emb) v += WTr<WT>::load1(e.pos_emb, (size_t)pos2 * e.d_model + i);
          e.h[(size_t)r * e.d_model + i] = v;
        }
    }
    return;
  }
  if (!a.spec && l == 0 && blockIdx.y == 0)
    for (int i = tid; i < a.d_model; i += SEL_THREADS) a.h[i] = a.h[(size_t)(1 + midx) * a.d_model + i];
  // tails are [nb][k][H][hd] rows; the cache is blocked (k_index / v_index)
  const float* src = (blockIdx.y == 0 ? a.tailK : a.tailV) + ((size_t)l * a.k + midx) * a.d_model;
  float* dst = (blockIdx.y == 0 ? a.Kc : a.Vc) + (size_t)l * a.H * a.head_floats;
  for (int idx = tid; idx < a.H * a.hd; idx += SEL_THREADS) {
    const int hh = idx / a.hd, i = idx - hh * a.hd;
    const size_t o = (size_t)hh * a.head_floats + (blockIdx.y == 0 ? k_index(pos_next, i, a.hd) : v_index(pos_next, i, a.hd));
    dst[o] = src[idx];
  }
}

}  // namespace ppd

// ==================================================================== bf16 weights: MFMA path
// For bf16 models every linear weight is repacked once (at context creation) into blocks that are
// both one contiguous kilobyte in HBM and one A operand of v_mfma_f32_16x16x32_bf16: block (nt, kt)
// holds rows 16*nt .. 16*nt+15, columns 32*kt .. 32*kt+31; inside it lane l = i + 16*c owns the eight
// consecutive bf16 of row i, columns 8*c .. 8*c+7.  A wave-load is then a flat 1 KiB read, needs no
// unpacking, and a skinny GEMM with up to 16 rows costs the same as with one: the candidates' rows
// ride along in the B operand's other columns.
//
// The B operand carries the input rows split into two bf16 terms, x = hi + lo with hi = bf16(x) and
// lo = bf16(x - hi) (|x - hi - lo| <= 2^-17 |x|), so the products are exact in fp32 and the fp32
// activations keep 16 mantissa bits.
//
// The kernel is built around instruction count: at 8 TB/s a compute unit has about 80 cycles per
// kilobyte block, i.e. some twenty vector instructions per block and wave.  Everything that is the
// same for a whole wave lives in scalar registers (the wave index goes through readfirstlane), the
// weight stream uses buffer loads (scalar base + scalar offset + one lane offset), the input rows come
// into LDS with direct-to-LDS loads, and the main loop has no barrier: every wave streams its eighth
// of the reduction length of all the workgroup's tiles and leaves its partial sums in LDS; one
// barrier, then the epilogue adds the eight partials of every output in wave order.
namespace ppd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int MG_THREADS = 512;     // 8 waves: each takes one eighth of the reduction length of a 16-row tile
constexpr int MG_WAVES = MG_THREADS / WAVE;
constexpr int MG_BATCH = 4;         // 1 KiB blocks requested per register batch
constexpr int MG_RING = 4;          // register batches in flight per wave
constexpr int MG_EP = 2;            // outputs per thread whose bias and residual are requested in the prologue
constexpr int MG_LDS_HLOG = 2048;   // byte offsets: [0, 2048) norm statistics, then 1 KiB of head logits,
constexpr int MG_LDS_G = 3072;      // then the norm's gain (and bias), the partial sums, the staged rows

struct RepackArgs {
  const uint16_t* src[3]; int nrows[3];   // up to three row segments, concatenated (Q | K | V); paired: src[0] gate, src[1] up
  int K, KT, NT, paired;
  uint16_t* dst;
};
#ifdef PPD_ENGINE_TU
__global__ void repack_kernel(RepackArgs a) {
  // one workgroup of 64 lanes per block
  const int blk = blockIdx.x, lane = threadIdx.x;
  const int nt = blk / a.KT, kt = blk - nt * a.KT;
  const int i = lane & 15, c = lane >> 4;
  const uint16_t* row = nullptr;
  if (a.paired) {
    int n = nt * 8 + (i & 7);
    if (n < a.nrows[0]) row = a.src[i < 8 ? 0 : 1] + (size_t)n * a.K;
  } else {
    int n = nt * 16 + i, seg = 0;
    while (seg < 3 && n >= a.nrows[seg]) { n -= a.nrows[seg]; ++seg; }
    if (seg < 3) row = a.src[seg] + (size_t)n * a.K;
  }
  uint16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    int k = kt * 32 + c * 8 + e;
    v[e] = (row && k < a.K) ? row[k] : (uint16_t)0;
  }
  uint4 o;
  o.x = v[0] | ((uint32_t)v[1] << 16); o.y = v[2] | ((uint32_t)v[3] << 16);
  o.z = v[4] | ((uint32_t)v[5] << 16); o.w = v[6] | ((uint32_t)v[7] << 16);
  *(uint4*)(a.dst + ((size_t)blk * 64 + lane) * 8) = o;
}
#endif

struct MGemmGroup {
  const float* X;     // [M][ldx] input rows (before the fused norm), rows 16-byte aligned
  const float* Rsd;   // residual rows [M][ldy] added in the epilogue, or null
  float* Y;           // [M][ldy]
  const void* P;      // repacked weights [NT][KT][64 lanes][8 bf16]
  const void* B[3];   // biases per row segment or null (paired: B[0] gate, B[1] up)
  const void* ng; const void* nb;  // gain / bias of the fused norm
  int M;              // rows, 1..16
};
struct MGemmArgs {
  MGemmGroup g[2];
  int K, KT, NT;    // reduction length (multiple of 8), its 32-column blocks, 16-row tiles
  int N[3];         // rows per segment (bias lookup)
  int ntot;         // logical output rows (paired: rows of one of the two matrices)
  int ldx, ldy;
  int norm;         // -1 none, 0 LayerNorm, 1 RMSNorm
  float eps;
  int act;          // 0 none, 1 GELU, 2 ReLU (paired launches apply SwiGLU)
  int topk; float* pk_val; int32_t* pk_idx;   // head launches: every workgroup leaves the top-k of each row's logits it made:
  int pk_stride;    // row m's list of workgroup b at ((m * pk_stride + b) * MAXM)
  int xrow;         // LDS bytes between two staged rows
  int tiles_wg;     // ceil(NT / gridDim.x); gridDim.x <= NT
  unsigned wbytes;  // NT * KT * 1024
  int passes;       // the reduction length is staged in LDS in this many passes (1: whole rows; > 1 only without a fused norm)
};

// LDS bytes between staged rows: the row itself, moved off a multiple of 256 so that neighbouring rows
// start in different banks
__host__ __device__ inline int mg_xrow(int KT) { int r = KT * 128; return (r & 255) ? r : r + 128; }
// Staging in passes: every wave's share of the reduction length (nb8 blocks) is cut into `passes` runs of
// nbp blocks (a multiple of the batch size); pass p stages, for each of the 8 waves, run p of its share.
__host__ __device__ inline int mg_nbp(int KT, int passes) {
  const int nb8 = (KT + MG_WAVES - 1) / MG_WAVES;
  if (passes <= 1) return (nb8 + MG_BATCH - 1) / MG_BATCH * MG_BATCH;
  return ((nb8 + passes - 1) / passes + MG_BATCH - 1) / MG_BATCH * MG_BATCH;
}
__host__ __device__ inline int mg_xrow_pass(int KT, int passes) { return passes <= 1 ? mg_xrow(KT) : mg_nbp(KT, passes) * 1024 + 128; }
// LDS map behind MG_LDS_G; returns the total
__host__ __device__ inline int mg_lds_layout(int K, int M, int norm, int tiles_wg, int xrow, int& off_b, int& off_part, int& off_x) {
  const int gsz = (K * 2 + 1023) & ~1023;
  off_b = MG_LDS_G + (norm >= 0 ? gsz : 0);
  off_part = off_b + (norm == 0 ? gsz : 0);
  off_x = off_part + tiles_wg * MG_WAVES * M * 64;
  return off_x + M * xrow;
}

// MP: the instance that can stage the reduction length in several passes (a.passes > 1); the other one
// keeps the single-pass loop free of that bookkeeping.
template <bool PAIRED, bool MP = false>
__global__ __launch_bounds__(MG_THREADS) void gemm_mfma_kernel(MGemmArgs a) {
  extern __shared__ float4 lds4[];
  char* lds = (char*)lds4;
  const MGemmGroup& G = a.g[blockIdx.y];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int M = G.M, K = a.K, KT = a.KT;
  const int grid = gridDim.x, xrow = a.xrow;
  const int ntiles = (int)blockIdx.x + (a.tiles_wg - 1) * grid < a.NT ? a.tiles_wg : a.tiles_wg - 1;
  int off_b, off_part, off_x;
  mg_lds_layout(K, M, a.norm, a.tiles_wg, xrow, off_b, off_part, off_x);
  float* stat = (float*)lds;                  // mu[16], rstd[16], redA[16][8], redB[16][8]
  float* redA = stat + 32;
  float* redB = stat + 32 + 16 * MG_WAVES;
  float* hlog = (float*)(lds + off_x);        // head launches: [M][HEAD_MAX_ROWS] logits, over the staged rows once those are done with

  // ---- 1. input rows (and the norm's gain and bias) into LDS, fp32 as they are: wave w takes the
  // kilobyte pieces w, w + 8, ... of every row.  These requests come first: a wave's loads return in order.
  // With passes, a staged row is 8 runs (one per wave) of nbp blocks; float f of the row belongs to wave
  // f / (32 nbp)'s share, block (pass * nbp + (f / 32) % nbp) of it.  pass_col gives the input column, or -1.
  const int npass = MP ? a.passes : 1;
  const int nb8_ = (KT + MG_WAVES - 1) / MG_WAVES, nbp_ = mg_nbp(KT, npass);
  auto pass_col = [&](int pass, int f) -> int {
    const int seg = f / (32 * nbp_), rem = f - seg * 32 * nbp_;
    const int s = pass * nbp_ + (rem >> 5);
    const int k0 = seg * nb8_ < KT ? seg * nb8_ : KT;
    const int nb = (k0 + nb8_ < KT ? k0 + nb8_ : KT) - k0;
    const int col = (k0 + s) * 32 + (rem & 31);
    return (s < nb && col < K) ? col : -1;
  };
  auto dma_pass = [&](int pass) {
    for (int u = wave; u < nbp_; u += MG_WAVES) {
      const int col = pass_col(pass, u * 256 + lane * 4);      // (the same for every row)
      if (col >= 0)
        for (int m = 0; m < M; ++m) dma16(G.X + (size_t)m * a.ldx + col, lds + off_x + m * xrow + u * 1024);
    }
  };
  {
    if (MP && npass > 1) dma_pass(0);
    else {
      const int U = (K + 255) >> 8;
      for (int m = 0; m < M; ++m)
        for (int u = wave; u < U; u += MG_WAVES) {
          const int kk = u * 256 + lane * 4;
          if (kk < K) dma16(G.X + (size_t)m * a.ldx + kk, lds + off_x + m * xrow + u * 1024);
        }
    }
    if (a.norm >= 0) {
      const int Ug = (K + 511) >> 9;
      for (int u = wave; u < Ug; u += MG_WAVES) {
        const int kk = u * 512 + lane * 8;
        if (kk < K) {
          dma16((const uint16_t*)G.ng + kk, lds + MG_LDS_G + u * 1024);
          if (a.norm == 0 && G.nb) dma16((const uint16_t*)G.nb + kk, lds + off_b + u * 1024);
        }
      }
    }
  }

  // ---- 2. bias and residual of the outputs this thread will finish (output e = tid + 512 i:
  // row = e % R inside the tile, then the input row, then the tile ordinal)
  constexpr int R = PAIRED ? 8 : 16;
  const int nout = ntiles * M * R;
  auto out_coord = [&](int e, int& ord, int& col, int& row, int& n) {
    row = e & (R - 1);
    const int f = e / R;
    ord = f / M; col = f - ord * M;
    n = ((int)blockIdx.x + ord * grid) * R + row;
  };
  // (the bf16 bias values stay raw until the epilogue: converting them here would wait for the loads)
  const uint16_t* const B0 = (const uint16_t*)G.B[0];
  const uint16_t* const B1 = (const uint16_t*)G.B[1];
  const uint16_t* const B2 = (const uint16_t*)G.B[2];
  auto out_operands = [&](int col, int n, uint32_t& b0, uint32_t& b1, float& rsd) {
    b0 = 0u; b1 = 0u; rsd = 0.f;
    if (PAIRED) {
      if (B0) b0 = B0[n];
      if (B1) b1 = B1[n];
    } else if (B0) {      // a model has either all linear biases or none
      int seg = 0, loc = n;
      if (loc >= a.N[0]) { loc -= a.N[0]; seg = 1; if (loc >= a.N[1]) { loc -= a.N[1]; seg = 2; } }
      const uint16_t* bp = seg == 0 ? B0 : (seg == 1 ? B1 : B2);
      b0 = bp[loc];
    }
    if (G.Rsd) rsd = G.Rsd[(size_t)col * a.ldy + n];
  };
  uint32_t p_b0[MG_EP], p_b1[MG_EP]; float p_rsd[MG_EP];
#pragma unroll
  for (int i = 0; i < MG_EP; ++i) {
    p_b0[i] = 0u; p_b1[i] = 0u; p_rsd[i] = 0.f;
    const int e = tid + i * MG_THREADS;
    if (e < nout) {
      int ord, col, row, n; out_coord(e, ord, col, row, n);
      if (n < a.ntot) out_operands(col, n, p_b0[i], p_b1[i], p_rsd[i]);
    }
  }

  // ---- 3. the weight stream: wave w owns k-blocks [kb0, kb0 + nblk) of every tile blockIdx.x,
  // + gridDim.x, ...; MG_BATCH blocks per batch, MG_RING batches in flight.  Every batch is always
  // requested in full: slots past the wave's share (or past the last tile) re-read the start of the
  // matrix, which is in the cache by then, and are never used.
  const int nb8 = (KT + MG_WAVES - 1) / MG_WAVES;
  const int kb0 = wave * nb8 < KT ? wave * nb8 : KT;
  const int nblk = (kb0 + nb8 < KT ? kb0 + nb8 : KT) - kb0;
  // Passes (P > 1 when the staged rows would not fit LDS at once): pass p covers blocks [p * nbp, (p + 1) * nbp)
  // of every wave's share, for all tiles, before the next pass starts.  A wave's accumulator of a tile is
  // parked in its partial-sum slot between passes and taken up again as the MFMA's C input, so the chain of
  // additions is exactly the one of a single pass.
  const int P = npass;
  const int nbp = mg_nbp(KT, P);                             // blocks of a wave's share per pass
  const int NBT = MP ? nbp / MG_BATCH : (nb8 + MG_BATCH - 1) / MG_BATCH;   // batches per tile (and pass), the same for every wave
  const int sst = P == 1 ? nb8 : nbp;                        // blocks between two waves' staged runs
  const int Q = P * ntiles * NBT;
  const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc((void*)G.P, 0, (int)a.wbytes, 0x00020000);
  const unsigned lane16 = lane * 16;
  int l_p = 0, l_tile = 0, l_b = 0;     // pass, tile ordinal and batch inside the tile of the next request
  auto issue = [&](u32x4 (&buf)[MG_BATCH]) {
    if constexpr (!MP) {
      const bool live = l_tile < ntiles;
      const unsigned base = (unsigned)(((int)blockIdx.x + l_tile * grid) * KT + kb0 + l_b * MG_BATCH) * 1024u;
#pragma unroll
      for (int j = 0; j < MG_BATCH; ++j) {
        const bool ok = live && l_b * MG_BATCH + j < nblk;
        buf[j] = __builtin_amdgcn_raw_buffer_load_b128(wres, lane16, ok ? base + j * 1024u : 0u, 2);   // 2: non-temporal
      }
      if (++l_b == NBT) { l_b = 0; ++l_tile; }
    } else {
      const bool live = l_p < P;
      const int s0 = l_p * nbp + l_b * MG_BATCH;
      const unsigned base = (unsigned)(((int)blockIdx.x + l_tile * grid) * KT + kb0 + s0) * 1024u;
#pragma unroll
      for (int j = 0; j < MG_BATCH; ++j) {
        const bool ok = live && s0 + j < nblk;
        buf[j] = __builtin_amdgcn_raw_buffer_load_b128(wres, lane16, ok ? base + j * 1024u : 0u, 2);
      }
      if (++l_b == NBT) { l_b = 0; if (++l_tile == ntiles) { l_tile = 0; ++l_p; } }
    }
  };
  // One batch per wave is what a compute unit keeps in flight: it goes out now, the rest of the ring
  // after the rows are staged (a wave that asked for more would sit in the request queue instead of
  // working on the rows).
  u32x4 ring[MG_RING][MG_BATCH];
  issue(ring[0]);

  // ---- 4. norm statistics and the split into two bf16 terms, in place: the 32 bytes that held the
  // floats k .. k+7 (k a multiple of 8) then hold hi(k..k+7) | lo(k..k+7).  One fixed order per row:
  // thread t sums the 8-element chunks t, t + 512, ... in turn, butterfly inside each wave, the eight
  // wave sums in index order.  LayerNorm: mean first, then the squared deviations.
  // everything requested before the weight stream has arrived once only the MG_BATCH newest loads
  // are outstanding; then the workgroup's rows are complete in LDS
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(MG_BATCH) : "memory");
  const int nchunk = KT * 4;                  // 32-byte chunks (8 elements) per staged row
  auto combine8 = [&](const float* r) { return ((((((r[0] + r[1]) + r[2]) + r[3]) + r[4]) + r[5]) + r[6]) + r[7]; };
  if (a.norm >= 0) {
    if (a.norm == 0) {
      for (int m = 0; m < M; ++m) {
        float sm = 0.f;
        for (int c = tid; c * 8 < K; c += MG_THREADS) {
          const float4* px = (const float4*)(lds + off_x + m * xrow + c * 32);
          const float4 v = px[0], w = px[1];
          sm += v.x; sm += v.y; sm += v.z; sm += v.w; sm += w.x; sm += w.y; sm += w.z; sm += w.w;
        }
        sm = wave_sum(sm);
        if (lane == 0) redA[m * MG_WAVES + wave] = sm;
      }
      __syncthreads();
    }
    for (int m = 0; m < M; ++m) {
      const float mu = a.norm == 0 ? combine8(redA + m * MG_WAVES) / (float)K : 0.f;
      float s2 = 0.f;
      for (int c = tid; c * 8 < K; c += MG_THREADS) {
        const float4* px = (const float4*)(lds + off_x + m * xrow + c * 32);
        const float4 v = px[0], w = px[1];
        const float d[8] = {v.x - mu, v.y - mu, v.z - mu, v.w - mu, w.x - mu, w.y - mu, w.z - mu, w.w - mu};
#pragma unroll
        for (int e = 0; e < 8; ++e) s2 = fmaf(d[e], d[e], s2);
      }
      s2 = wave_sum(s2);
      if (lane == 0) redB[m * MG_WAVES + wave] = s2;
    }
    __syncthreads();
    if (tid < M) {
      stat[tid] = a.norm == 0 ? combine8(redA + tid * MG_WAVES) / (float)K : 0.f;
      stat[16 + tid] = 1.0f / sqrtf(combine8(redB + tid * MG_WAVES) / (float)K + a.eps);
    }
    __syncthreads();
  }
  // (with passes: the same split, for the runs of one pass; chunks outside every wave's share become zeros)
  auto convert_rows = [&](int pass) {
  const int nch = (MP && npass > 1) ? nbp_ * 32 : nchunk;
  if constexpr (MP) {
    if (npass > 1) {
      // (no fused norm with passes; whether a chunk lies inside a wave's share is the same for every row)
      for (int c = tid; c < nch; c += MG_THREADS) {
        const bool inside = pass_col(pass, c * 8) >= 0;
        for (int m = 0; m < M; ++m) {
          char* px = lds + off_x + m * xrow + c * 32;
          float xv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          if (inside) {
            const float4 v = ((const float4*)px)[0], w = ((const float4*)px)[1];
            xv[0] = v.x; xv[1] = v.y; xv[2] = v.z; xv[3] = v.w; xv[4] = w.x; xv[5] = w.y; xv[6] = w.z; xv[7] = w.w;
          }
          uint32_t hp[4], lp[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            hp[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){xv[2 * e], xv[2 * e + 1]}, bf16x2));
            const float r0 = xv[2 * e] - __uint_as_float(hp[e] << 16), r1 = xv[2 * e + 1] - __uint_as_float(hp[e] & 0xffff0000u);
            lp[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){r0, r1}, bf16x2));
          }
          ((uint4*)px)[0] = make_uint4(hp[0], hp[1], hp[2], hp[3]);
          ((uint4*)px)[1] = make_uint4(lp[0], lp[1], lp[2], lp[3]);
        }
      }
      return;
    }
  }
  for (int m = 0; m < M; ++m) {
    const float mu = a.norm >= 0 ? stat[m] : 0.f, rs = a.norm >= 0 ? stat[16 + m] : 1.f;
    for (int c = tid; c < nch; c += MG_THREADS) {
      char* px = lds + off_x + m * xrow + c * 32;
      float xv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      if ((MP && npass > 1) ? pass_col(pass, c * 8) >= 0 : c * 8 < K) {
        const float4 v = ((const float4*)px)[0], w = ((const float4*)px)[1];
        xv[0] = v.x; xv[1] = v.y; xv[2] = v.z; xv[3] = v.w; xv[4] = w.x; xv[5] = w.y; xv[6] = w.z; xv[7] = w.w;
        if (a.norm >= 0) {
          const u32x4 gq = *(const u32x4*)(lds + MG_LDS_G + c * 16);
          float gf[8]; WTr<bf16_t>::unpack(gq, gf);
#pragma unroll
          for (int e = 0; e < 8; ++e) xv[e] = (xv[e] - mu) * rs * gf[e];
          if (a.norm == 0 && G.nb) {
            const u32x4 bq = *(const u32x4*)(lds + off_b + c * 16);
            float bf[8]; WTr<bf16_t>::unpack(bq, bf);
#pragma unroll
            for (int e = 0; e < 8; ++e) xv[e] += bf[e];
          }
        }
      }
      // hi = bf16(x) (the hardware's round-to-nearest-even pair conversion), lo = bf16(x - hi)
      uint32_t hp[4], lp[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        hp[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){xv[2 * e], xv[2 * e + 1]}, bf16x2));
        const float r0 = xv[2 * e] - __uint_as_float(hp[e] << 16), r1 = xv[2 * e + 1] - __uint_as_float(hp[e] & 0xffff0000u);
        lp[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){r0, r1}, bf16x2));
      }
      ((uint4*)px)[0] = make_uint4(hp[0], hp[1], hp[2], hp[3]);
      ((uint4*)px)[1] = make_uint4(lp[0], lp[1], lp[2], lp[3]);
    }
  }
  };
  convert_rows(0);
  __syncthreads();
#pragma unroll
  for (int r = 1; r < MG_RING; ++r) issue(ring[r]);

  // ---- 5. main loop.  B operand: lane l feeds column l % 16 (input row; lanes past M read row 0 and
  // their columns are never stored) and the eight k of chunk l / 16.
  const int bm = lane & 15, bc = lane >> 4;
  const char* xlane = lds + off_x + (bm < M ? bm : 0) * xrow + bc * 32 + ((!MP || P == 1) ? kb0 : wave * sst) * 128;
  float* plane = (float*)(lds + off_part) + (wave * M + bm) * 16 + bc * 4;   // + ord * 8 * M * 16
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  int c_p = 0, c_ord = 0, c_b = 0;
  auto consume = [&](u32x4 (&cur)[MG_BATCH]) {
    if constexpr (!MP) {
#pragma unroll
      for (int j = 0; j < MG_BATCH; ++j) {
        const int s = c_b * MG_BATCH + j;
        if (s < nblk) {                      // the same for the whole wave
          const u32x4* xp = (const u32x4*)(xlane + s * 128);
          const u32x4 bh = xp[0], bl = xp[1];
          const bf16x8 av = __builtin_bit_cast(bf16x8, cur[j]);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bh), acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bl), acc, 0, 0, 0);
        }
      }
      if (++c_b == NBT) {
        // this wave's partial sums of the tile: lane l holds rows 4 (l / 16) .. + 3 of column l % 16
        if (bm < M) *(f32x4*)(plane + c_ord * (MG_WAVES * 16) * M) = acc;
        acc = (f32x4){0.f, 0.f, 0.f, 0.f};
        c_b = 0; ++c_ord;
      }
    } else {
      if (c_b == 0 && c_p > 0) {
        if (c_ord == 0) {
          // next pass: every wave is done with the staged runs; bring in the next ones (the weight requests
          // already made for this pass keep flying meanwhile)
          __syncthreads();
          dma_pass(c_p);
          asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
          convert_rows(c_p);
          __syncthreads();
        }
        if (bm < M) acc = *(const f32x4*)(plane + c_ord * (MG_WAVES * 16) * M);    // the chain goes on where it stopped
      }
#pragma unroll
      for (int j = 0; j < MG_BATCH; ++j) {
        const int s = c_p * nbp + c_b * MG_BATCH + j;
        if (s < nblk) {
          const u32x4* xp = (const u32x4*)(xlane + (s - c_p * nbp) * 128);
          const u32x4 bh = xp[0], bl = xp[1];
          const bf16x8 av = __builtin_bit_cast(bf16x8, cur[j]);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bh), acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bl), acc, 0, 0, 0);
        }
      }
      if (++c_b == NBT) {
        if (bm < M) *(f32x4*)(plane + c_ord * (MG_WAVES * 16) * M) = acc;
        acc = (f32x4){0.f, 0.f, 0.f, 0.f};
        c_b = 0;
        if (++c_ord == ntiles) { c_ord = 0; ++c_p; }
      }
    }
  };
  for (int q = 0; q < Q; q += MG_RING) {
#pragma unroll
    for (int r = 0; r < MG_RING; ++r) {
      if (q + r < Q) consume(ring[r]);
      issue(ring[r]);
    }
  }
  __syncthreads();

  // ---- 6. epilogue: the eight partials of an output in wave order, bias, activation, residual
  auto finish = [&](int e, uint32_t rb0, uint32_t rb1, float rsd) {
    int ord, col, row, n; out_coord(e, ord, col, row, n);
    if (n >= a.ntot) return;
    const float b0 = __uint_as_float(rb0 << 16), b1 = __uint_as_float(rb1 << 16);
    const float* pp = (const float*)(lds + off_part) + (ord * MG_WAVES * M + col) * 16 + row;
    const int ws = M * 16;
    float s = pp[0];
#pragma unroll
    for (int w = 1; w < MG_WAVES; ++w) s += pp[w * ws];
    float y;
    if (PAIRED) {
      float u = pp[8];
#pragma unroll
      for (int w = 1; w < MG_WAVES; ++w) u += pp[w * ws + 8];
      y = silu(s + b0) * (u + b1);
    } else {
      y = s + b0;
      if (a.act == 1) y = gelu_erf(y);
      else if (a.act == 2) y = fmaxf(y, 0.f);
    }
    y += rsd;
    G.Y[(size_t)col * a.ldy + n] = y;
    if (a.topk > 0) hlog[col * HEAD_MAX_ROWS + ord * 16 + row] = y;
  };
#pragma unroll
  for (int i = 0; i < MG_EP; ++i) {
    const int e = tid + i * MG_THREADS;
    if (e < nout) finish(e, p_b0[i], p_b1[i], p_rsd[i]);
  }
  for (int e = tid + MG_EP * MG_THREADS; e < nout; e += MG_THREADS) {
    int ord, col, row, n; out_coord(e, ord, col, row, n);
    uint32_t b0 = 0u, b1 = 0u; float rsd = 0.f;
    if (n < a.ntot) out_operands(col, n, b0, b1, rsd);
    finish(e, b0, b1, rsd);
  }

  // ---- LM head: this workgroup's top-k of every row by (logit descending, id ascending); wave w takes rows w, w + 8, ...
  if (a.topk > 0) {
    __syncthreads();
    for (int col = wave; col < M; col += MG_WAVES) {
      constexpr int EPL = HEAD_MAX_ROWS / WAVE;
      float ev[EPL]; int ei[EPL];
#pragma unroll
      for (int u = 0; u < EPL; ++u) {
        const int e = lane + u * WAVE;       // entry e = tile ordinal * 16 + row
        ev[u] = -INFINITY; ei[u] = 0x7fffffff;
        const int id = ((int)blockIdx.x + (e >> 4) * grid) * 16 + (e & 15);
        if ((e >> 4) < ntiles && id < a.ntot) { ev[u] = hlog[col * HEAD_MAX_ROWS + e]; ei[u] = id; }
      }
      for (int r = 0; r < a.topk; ++r) {
        float v = -INFINITY; int i = 0x7fffffff;
#pragma unroll
        for (int u = 0; u < EPL; ++u) if (better(ev[u], ei[u], v, i)) { v = ev[u]; i = ei[u]; }
        wave_best(v, i);
#pragma unroll
        for (int u = 0; u < EPL; ++u) if (ei[u] == i) { ev[u] = -INFINITY; ei[u] = 0x7fffffff; }
        if (lane == 0) {
          const size_t o = ((size_t)col * a.pk_stride + blockIdx.x) * MAXM + r;
          a.pk_val[o] = v; a.pk_idx[o] = i;
        }
      }
    }
  }
}

// The norm of gemm_mfma_kernel's prologue on its own: Y = norm(X) row by row, with the same order of additions
// (thread t sums the 8-element pieces t, t + 512, ...; butterfly inside each wave; the eight wave sums in index
// order) and the same expression per element, so that a GEMM without a fused norm on Y gives the bits of the
// fused one on X.  For row groups whose rows do not fit LDS whole (prompt chunks): the GEMM then stages Y in passes.
#ifdef PPD_ENGINE_TU
struct NormRowsArgs {
  const float* X; float* Y;      // [M][ld]
  const void* g; const void* b;  // bf16 gain, bias (LayerNorm) or null
  int K, ld, norm;               // norm: 0 LayerNorm, 1 RMSNorm
  float eps;
};
__global__ __launch_bounds__(MG_THREADS) void norm_rows_kernel(NormRowsArgs a) {
  __shared__ float redA[MG_WAVES], redB[MG_WAVES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, K = a.K;
  const float* x = a.X + (size_t)blockIdx.x * a.ld;
  float* y = a.Y + (size_t)blockIdx.x * a.ld;
  auto combine8 = [&](const float* r) { return ((((((r[0] + r[1]) + r[2]) + r[3]) + r[4]) + r[5]) + r[6]) + r[7]; };
  float mu = 0.f;
  if (a.norm == 0) {
    float sm = 0.f;
    for (int c = tid; c * 8 < K; c += MG_THREADS) {
      const float4* px = (const float4*)(x + c * 8);
      const float4 v = px[0], w = px[1];
      sm += v.x; sm += v.y; sm += v.z; sm += v.w; sm += w.x; sm += w.y; sm += w.z; sm += w.w;
    }
    sm = wave_sum(sm);
    if (lane == 0) redA[wave] = sm;
    __syncthreads();
    mu = combine8(redA) / (float)K;
  }
  float s2 = 0.f;
  for (int c = tid; c * 8 < K; c += MG_THREADS) {
    const float4* px = (const float4*)(x + c * 8);
    const float4 v = px[0], w = px[1];
    const float d[8] = {v.x - mu, v.y - mu, v.z - mu, v.w - mu, w.x - mu, w.y - mu, w.z - mu, w.w - mu};
#pragma unroll
    for (int e = 0; e < 8; ++e) s2 = fmaf(d[e], d[e], s2);
  }
  s2 = wave_sum(s2);
  if (lane == 0) redB[wave] = s2;
  __syncthreads();
  const float rs = 1.0f / sqrtf(combine8(redB) / (float)K + a.eps);
  for (int c = tid; c * 8 < K; c += MG_THREADS) {
    const float4* px = (const float4*)(x + c * 8);
    const float4 v = px[0], w = px[1];
    float xv[8] = {v.x, v.y, v.z, v.w, w.x, w.y, w.z, w.w};
    const u32x4 gq = *(const u32x4*)((const char*)a.g + (size_t)c * 16);
    float gf[8]; WTr<bf16_t>::unpack(gq, gf);
#pragma unroll
    for (int e = 0; e < 8; ++e) xv[e] = (xv[e] - mu) * rs * gf[e];
    if (a.norm == 0 && a.b) {
      const u32x4 bq = *(const u32x4*)((const char*)a.b + (size_t)c * 16);
      float bf[8]; WTr<bf16_t>::unpack(bq, bf);
#pragma unroll
      for (int e = 0; e < 8; ++e) xv[e] += bf[e];
    }
    float4* py = (float4*)(y + c * 8);
    py[0] = make_float4(xv[0], xv[1], xv[2], xv[3]);
    py[1] = make_float4(xv[4], xv[5], xv[6], xv[7]);
  }
}
#endif

}  // namespace ppd
