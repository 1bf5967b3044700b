// Compute-bound prompt pass for bf16 models (gfx950).
//
// The method starts from a start token x_0 (Algorithm 1 / 2); a prompt is run through all d layers first to fill
// the key/value cache.  The decode kernels stream every weight once per 16 rows, which is the right shape for a
// handful of rows and the wrong one for a prompt: here the prompt's rows are a real matrix operand.
//
//   pack_rows_kernel    rows (after an optional norm) -> two bf16 terms x = hi + lo in MFMA operand blocks
//   pgemm_kernel        Y = epilogue(X W^T): register-tiled v_mfma_f32_32x32x16_bf16, weights in the repacked
//                       1 KiB blocks of the decode path (A operand), packed rows as B operand, both straight from
//                       memory (every wave-load is one contiguous kilobyte); products exact in fp32 as in decoding
//   pkv_pack_kernel     queries, keys, values of the prompt rows -> two-term operand blocks, and keys and values into
//                       the fp32 cache in the decode path's layout
//   pattn_kernel        causal attention of all prompt rows on the same MFMA (three products per pair of two-term
//                       operands), key/value steps staged through LDS for the four waves of a workgroup, running softmax
//
// Rounding order differs from the decode kernels (other tiles, other summation trees), so a cache filled here is
// close to, not bit-identical with, one filled row by row; every decode step after it is the same arithmetic
// whichever way the cache was filled, so PPD == plain greedy bit for bit still holds.
#pragma once
#include "ppd_kernels.h"

namespace ppd {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PG_WAVES = 4;                        // waves that multiply: each its own outputs against the workgroup's prompt rows
constexpr int PG_THREADS = (PG_WAVES + 1) * WAVE;  // and one wave that stages the rows in LDS for them
constexpr int PG_D = 2, PG_R = PG_D + 2;           // stages of rows in flight ahead of their use; ring slots in LDS
constexpr int PG_STAGE_BLKS = 16;                  // 1 KiB blocks per stage: KB 32-column blocks x 2 planes x TMB 16-row blocks
#ifndef PPD_PG_NBUF
#define PPD_PG_NBUF 6
#endif
constexpr int PG_NBUF = PPD_PG_NBUF;   // register buffers of operand blocks per wave
#ifndef PPD_PG_GROUP_M
#define PPD_PG_GROUP_M 8
#endif
#ifndef PPD_PG_GROUP_Q
#define PPD_PG_GROUP_Q 8
#endif
constexpr int PG_GROUP_M = PPD_PG_GROUP_M, PG_GROUP_Q = PPD_PG_GROUP_Q;   // launch-order groups on one XCD (row blocks x output blocks)

// ---- rows -> packed two-term operand blocks
// Block (mt, kt) holds rows 16 mt .. +15, columns 32 kt .. +31 as 64 lanes x 8 bf16: lane i + 16 c = row i, columns
// 8 c .. 8 c + 7 (the B operand of v_mfma_f32_16x16x32_bf16).  Plane 0: hi = bf16(x); plane 1: lo = bf16(x - hi).
// Rows past M and columns past K are zeros.
struct PackArgs {
  const float* X; int ld;        // [M][ld]
  int M, K, KT, MT;              // KT = ceil(K / 32), MT = ceil(M / 16)
  const void* g; const void* b;  // bf16 gain / bias of the norm (norm >= 0)
  int norm;                      // -1 none, 0 LayerNorm, 1 RMSNorm
  float eps;
  uint16_t* out;                 // [2][MT][KT][64][8]
};

__device__ __forceinline__ void split2(const float (&xv)[8], uint4& hi, uint4& lo) {
  uint32_t hp[4], lp[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    hp[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){xv[2 * e], xv[2 * e + 1]}, bf16x2));
    const float r0 = xv[2 * e] - __uint_as_float(hp[e] << 16), r1 = xv[2 * e + 1] - __uint_as_float(hp[e] & 0xffff0000u);
    lp[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){r0, r1}, bf16x2));
  }
  hi = make_uint4(hp[0], hp[1], hp[2], hp[3]);
  lo = make_uint4(lp[0], lp[1], lp[2], lp[3]);
}

#ifdef PPD_PREFILL_TU
// One workgroup per row (rows up to 16 MT: the padding rows write zeros).  The norm is the decode path's: thread t
// sums the 8-element pieces t, t + 512, ...; butterfly inside each wave; the eight wave sums in index order.
__global__ __launch_bounds__(MG_THREADS) void pack_rows_kernel(PackArgs a) {
  __shared__ float redA[MG_WAVES], redB[MG_WAVES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, K = a.K;
  const int m = blockIdx.x, mt = m >> 4, i = m & 15;
  const size_t plane = (size_t)a.MT * a.KT * 512;        // bf16 elements per plane
  const float* x = a.X + (size_t)m * a.ld;
  const bool live = m < a.M;
  auto combine8 = [&](const float* r) { return ((((((r[0] + r[1]) + r[2]) + r[3]) + r[4]) + r[5]) + r[6]) + r[7]; };
  float mu = 0.f, rs = 1.f;
  if (a.norm >= 0 && live) {
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
    rs = 1.0f / sqrtf(combine8(redB) / (float)K + a.eps);
  }
  for (int c = tid; c < a.KT * 4; c += MG_THREADS) {     // 8-element pieces of the padded row
    float xv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (live && c * 8 < K) {
      const float4* px = (const float4*)(x + c * 8);
      const float4 v = px[0], w = px[1];
      xv[0] = v.x; xv[1] = v.y; xv[2] = v.z; xv[3] = v.w; xv[4] = w.x; xv[5] = w.y; xv[6] = w.z; xv[7] = w.w;
      if (a.norm >= 0) {
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
      }
    }
    uint4 hi, lo;
    split2(xv, hi, lo);
    const size_t o = (((size_t)mt * a.KT + (c >> 2)) * 64 + i + 16 * (c & 3)) * 8;
    *(uint4*)(a.out + o) = hi;
    *(uint4*)(a.out + plane + o) = lo;
  }
}
#endif

// ---- tiled GEMM
struct PGemmArgs {
  const uint16_t* Xp;   // packed rows [2][MT][KT][64][8]
  const void* P;        // repacked weights [NT][KT][64][8]
  const void* B[3];     // biases per row segment or null (paired: B[0] gate, B[1] up)
  const float* Rsd;     // residual rows [M][ldy] or null
  float* Y;             // [M][ldy]
  int M, MT, KT, NT;
  int N[3], ntot;       // rows per segment (bias lookup); logical output rows
  int ldy;
  int act;              // 0 none, 1 GELU, 2 ReLU (paired launches apply SwiGLU)
  int NB, MB;           // workgroup grid: NB blocks of 4 * TN 16-row blocks along the outputs, MB blocks of TMB 16-row blocks along the rows
  int GQ, GM, MBG;      // launch order on one XCD: groups of GQ output blocks x GM row blocks, MBG = ceil(MB / GM) groups per output-block row
  // the outputs in packed two-term form instead of Y (they are the next GEMM's rows: the feed-forward activations):
  // [2][MT][KTp][64][8]; only outputs below ntot are written, the padding columns of the buffer stay as they are (zero)
  uint16_t* Yp; int KTp;
};

// four consecutive outputs n0 .. n0 + 3 (n0 a multiple of 4) of row m into the packed form: half of an 8-column piece
__device__ __forceinline__ void put_packed4(uint16_t* out, size_t plane_elems, int KT, int m, int n0, const float (&y)[4]) {
  uint32_t hp[2], lp[2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    hp[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){y[2 * e], y[2 * e + 1]}, bf16x2));
    const float r0 = y[2 * e] - __uint_as_float(hp[e] << 16), r1 = y[2 * e + 1] - __uint_as_float(hp[e] & 0xffff0000u);
    lp[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){r0, r1}, bf16x2));
  }
  const int c8 = n0 >> 3;
  const size_t o = (((size_t)(m >> 4) * KT + (c8 >> 2)) * 64 + (m & 15) + 16 * (c8 & 3)) * 8 + ((n0 >> 2) & 1) * 4;
  *(uint2*)(out + o) = make_uint2(hp[0], hp[1]);
  *(uint2*)(out + plane_elems + o) = make_uint2(lp[0], lp[1]);
}


// Workgroup b of the launch runs on XCD b % 8 (workgroups go round the XCDs in launch order), which owns every
// eighth output block.  Its workgroups come in groups of GQ output blocks x GM row blocks, about what the XCD's
// compute units work on at a time: the group reads GQ weight panels and GM row panels from memory once and serves
// the other uses from that XCD's L2 (one output block against all row blocks would re-read every row panel for
// every output block).  Measured on the 13B shape with 4095 rows: QKV projection 1.23 -> 1.06 ms.
// The MFMA is v_mfma_f32_32x32x16_bf16 (a 16x16x32 one issues at half its rate on this part).  Its operands
// come out of the 16-row blocks as they lie in memory: lane r + 32 h of a 32-row tile reads 16 bytes of the
// 16-row block r / 16 at lane position (r % 16) + 16 (2 w + h), w = 0, 1 being the two 16-column halves of the
// 32-column block, so one block pair feeds two MFMAs per operand pair, and weights and rows pair up column by
// column whatever order the hardware takes the 16 columns in.
// A workgroup is four multiplying waves and one staging wave.  Multiplying wave w holds TN / 2 x TMB / 2
// accumulator tiles of 32 x 32: its own TN 16-row weight blocks, straight from memory into PG_NBUF register
// buffers, against the workgroup's 16 TMB prompt rows, which the staging wave brings into LDS by direct loads (a
// ring of PG_R stages, PG_D in flight; one barrier per stage hands a stage over): a row block is fetched once per
// workgroup instead of once per wave, and the waits on the two kinds of loads do not mix in one wave's counter.
template <bool PAIRED, int TN, int TMB>
__global__ __launch_bounds__(PG_THREADS) void pgemm_kernel(PGemmArgs a) {
  constexpr int TW = TN / 2, TX = TMB / 2;                 // 32-row tiles per wave: weights, prompt rows
  constexpr int KB = PG_STAGE_BLKS / (2 * TMB);            // 32-column blocks per stage
  static_assert(TN % 2 == 0 && TMB % 2 == 0 && KB >= 1 && KB * 2 * TMB == PG_STAGE_BLKS && PG_NBUF % KB == 0, "tile shapes");
  static_assert(PG_D * PG_STAGE_BLKS < 64, "the staging wave's wait counts its requests in flight");
  extern __shared__ float4 pg_lds4[];
  char* const lds = (char*)pg_lds4;                        // [PG_R][PG_STAGE_BLKS] KiB
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = blockIdx.x, xcd = b & 7, r = b >> 3;
  const int per = a.GQ * a.GM, g = r / per, gi = r - g * per;
  const int gq = g / a.MBG, gm = g - gq * a.MBG;
  const int nb = (gq * a.GQ + gi / a.GM) * 8 + xcd, mb = gm * a.GM + gi % a.GM;
  if (nb >= a.NB || mb >= a.MB) return;
  const int KT = a.KT;
  const int mt0 = mb * TMB;                                // in 16-row blocks
  const size_t plane = (size_t)a.MT * KT * 1024;          // bytes per plane of the packed rows
  const int nstg = (KT + KB - 1) / KB;

  if (wave == PG_WAVES) {
    // ---- the staging wave: stage s = 32-column blocks KB s .. KB s + KB - 1 of the workgroup's rows, both planes
    const char* const src0 = (const char*)a.Xp + lane * 16;
    auto stage = [&](int s) {
      char* const dst = lds + (size_t)(s % PG_R) * PG_STAGE_BLKS * 1024;
#pragma unroll
      for (int kk = 0; kk < KB; ++kk) {
        const int kt = KB * s + kk < KT ? KB * s + kk : KT - 1;    // (a block past the end repeats the last one; unused)
#pragma unroll
        for (int pl = 0; pl < 2; ++pl)
#pragma unroll
          for (int tb = 0; tb < TMB; ++tb) {
            const int mt = mt0 + tb < a.MT ? mt0 + tb : a.MT - 1;  // (blocks past the prompt re-read its last block; never stored)
            dma16(src0 + pl * plane + ((size_t)mt * KT + kt) * 1024, dst + ((kk * 2 + pl) * TMB + tb) * 1024);
          }
      }
    };
    for (int s = 0; s < PG_D && s < nstg; ++s) stage(s);
    for (int s = 0; s < nstg; ++s) {
      // slot (s + PG_D) % PG_R was last read for stage s - 2: every wave is past that (it has met barrier s - 1)
      if (s + PG_D < nstg) {
        stage(s + PG_D);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PG_D * PG_STAGE_BLKS) : "memory");   // all but the PG_D youngest stages: stage s is in
      } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      }
      __syncthreads();
    }
    return;
  }

  // ---- the multiplying waves
  const int nt0 = (nb * PG_WAVES + wave) * TN;
  const int lr = lane & 31, lh = lane >> 5;
  const int lane_off = ((lr & 15) + 16 * lh) * 16;         // + 512 for the second 16-column half
  const char* wbase[TW];
#pragma unroll
  for (int t = 0; t < TW; ++t) {
    int nt = nt0 + 2 * t + (lr >> 4);
    if (nt >= a.NT) nt = a.NT - 1;                         // (blocks past the matrix re-read its last block; never stored)
    wbase[t] = (const char*)a.P + (size_t)nt * KT * 1024 + lane_off;
  }
  const char* const xlds = lds + (lr >> 4) * 1024 + lane_off;
  f32x16 acc[TW][TX];
#pragma unroll
  for (int i = 0; i < TW; ++i)
#pragma unroll
    for (int j = 0; j < TX; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  // PG_NBUF register buffers of weight blocks: those of the next PG_NBUF - 1 reduction steps are in flight while one is multiplied
  u32x4 wa[PG_NBUF][TW][2];
  auto fetch = [&](int kt, int buf) {
    const size_t o = (size_t)(kt < KT ? kt : KT - 1) * 1024;       // (requests past the end repeat the last block; unused)
#pragma unroll
    for (int t = 0; t < TW; ++t)
#pragma unroll
      for (int w = 0; w < 2; ++w) wa[buf][t][w] = *(const u32x4*)(wbase[t] + o + 512 * w);
  };
  // one 32-column block: the rows' two terms from LDS (all products with the first terms, then all with the second:
  // no MFMA waits for the one before it)
  auto mac = [&](int buf, int kt, int kk) {
    const char* const xs = xlds + ((size_t)((kt / KB) % PG_R) * PG_STAGE_BLKS + kk * 2 * TMB) * 1024;
    u32x4 xh[TX][2], xl[TX][2];
#pragma unroll
    for (int j = 0; j < TX; ++j)
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        xh[j][w] = *(const u32x4*)(xs + (2 * j) * 1024 + 512 * w);
        xl[j][w] = *(const u32x4*)(xs + (TMB + 2 * j) * 1024 + 512 * w);
      }
#pragma unroll
    for (int w = 0; w < 2; ++w)
#pragma unroll
      for (int i = 0; i < TW; ++i)
#pragma unroll
        for (int j = 0; j < TX; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wa[buf][i][w]), __builtin_bit_cast(bf16x8, xh[j][w]), acc[i][j], 0, 0, 0);
#pragma unroll
    for (int w = 0; w < 2; ++w)
#pragma unroll
      for (int i = 0; i < TW; ++i)
#pragma unroll
        for (int j = 0; j < TX; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wa[buf][i][w]), __builtin_bit_cast(bf16x8, xl[j][w]), acc[i][j], 0, 0, 0);
  };
#pragma unroll
  for (int p = 0; p < PG_NBUF - 1; ++p) fetch(p, p);
  int kt = 0;
  for (; kt + PG_NBUF <= KT; kt += PG_NBUF) {
#pragma unroll
    for (int p = 0; p < PG_NBUF; ++p) {
      if (p % KB == 0) __syncthreads();                    // the stage of this block is in LDS
      fetch(kt + p + PG_NBUF - 1, (p + PG_NBUF - 1) % PG_NBUF);
      mac(p, kt + p, p % KB);
    }
  }
#pragma unroll
  for (int p = 0; p < PG_NBUF - 1; ++p)
    if (kt + p < KT) {
      if (p % KB == 0) __syncthreads();
      fetch(kt + p + PG_NBUF - 1, (p + PG_NBUF - 1) % PG_NBUF);
      mac(p, kt + p, p % KB);
    }

  // ---- epilogue: registers 4 q .. 4 q + 3 of a tile are its rows 8 q + 4 (l / 32) .. + 3 (weight rows) for column l % 32
  // (prompt row)
  const uint16_t* const B0 = (const uint16_t*)a.B[0];
  const uint16_t* const B1 = (const uint16_t*)a.B[1];
  const uint16_t* const B2 = (const uint16_t*)a.B[2];
#pragma unroll
  for (int i = 0; i < TW; ++i) {
#pragma unroll
    for (int j = 0; j < TX; ++j) {
      const int m = (mt0 + 2 * j) * 16 + lr;
      if (m >= a.M) continue;
      if (PAIRED) {
        // a 16-row block holds the gate rows (0..7) and the up rows (8..15) of 8 outputs: register groups 0, 1 are
        // gate and up of the first block's outputs 4 (l / 32) .. + 3, groups 2, 3 of the second block's
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
          const int nt = nt0 + 2 * i + hb;
          if (nt >= a.NT) continue;
          const int n0 = nt * 8 + 4 * lh;
          if (n0 >= a.ntot) continue;
          float y[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int n = n0 + q < a.ntot ? n0 + q : a.ntot - 1;
            const float bg = B0 ? bf16_to_f32(B0[n]) : 0.f, bu = B1 ? bf16_to_f32(B1[n]) : 0.f;
            y[q] = n0 + q < a.ntot ? silu(acc[i][j][8 * hb + q] + bg) * (acc[i][j][8 * hb + 4 + q] + bu) : 0.f;
          }
          if (a.Yp) { put_packed4(a.Yp, (size_t)a.MT * a.KTp * 512, a.KTp, m, n0, y); continue; }
          float* py = a.Y + (size_t)m * a.ldy + n0;
          if (n0 + 3 < a.ntot) *(float4*)py = make_float4(y[0], y[1], y[2], y[3]);
          else for (int q = 0; q < 4; ++q) if (n0 + q < a.ntot) py[q] = y[q];
        }
      } else {
#pragma unroll
        for (int gq4 = 0; gq4 < 4; ++gq4) {
          const int n0 = (nt0 + 2 * i) * 16 + 8 * gq4 + 4 * lh;
          if (n0 >= a.ntot) continue;
          float y[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int n = n0 + q < a.ntot ? n0 + q : a.ntot - 1;
            float bv = 0.f;
            if (B0) {
              int seg = 0, loc = n;
              if (loc >= a.N[0]) { loc -= a.N[0]; seg = 1; if (loc >= a.N[1]) { loc -= a.N[1]; seg = 2; } }
              bv = bf16_to_f32((seg == 0 ? B0 : (seg == 1 ? B1 : B2))[loc]);
            }
            float tv = acc[i][j][4 * gq4 + q] + bv;
            if (a.act == 1) tv = gelu_erf(tv);
            else if (a.act == 2) tv = fmaxf(tv, 0.f);
            if (a.Rsd) tv += a.Rsd[(size_t)m * a.ldy + n];
            y[q] = n0 + q < a.ntot ? tv : 0.f;
          }
          if (a.Yp) { put_packed4(a.Yp, (size_t)a.MT * a.KTp * 512, a.KTp, m, n0, y); continue; }
          float* py = a.Y + (size_t)m * a.ldy + n0;
          if (n0 + 3 < a.ntot) *(float4*)py = make_float4(y[0], y[1], y[2], y[3]);
          else for (int q = 0; q < 4; ++q) if (n0 + q < a.ntot) py[q] = y[q];
        }
      }
    }
  }
}

// ---- causal attention of the prompt rows
// Row m of the prompt sits at position m (the prompt pass starts from an empty cache) and attends to rows 0 .. m.
// Queries (rotated, scaled), keys (rotated exactly as the cache holds them) and values are first put into two-term
// bf16 operand blocks, so that scores and outputs run on v_mfma_f32_16x16x32_bf16 with the three products
// hi.hi + hi.lo + lo.hi each (the lo.lo term is below 2^-16 of the result) instead of the fp32 MFMA, which
// is a sixteenth as fast:
//   Qp, Kp  [2][H][2 JP][HD / 32][64][8]   block (tile of 16 rows, 32 components): lane i + 16 c = row i, components 8 c .. + 7
//   Vp      [2][H][JP][HD / 16][64][8]     block (32 rows, 16 components): lane i + 16 c = component i, and its 8 values
//                                          are rows 4 c .. 4 c + 3 and 16 + 4 c .. 16 + 4 c + 3 of the 32
// (JP = ceil(M / 32); rows past M are zeros.)  The odd row order of Vp is the one in which a lane holds its scores
// after the two score MFMAs of a 32-row step: lane n + 16 c has, for query n, rows 4 c .. + 3 of either 16-row tile,
// so the probabilities are the B operand of the output MFMA as they stand, without any exchange between lanes.
struct PKvPackArgs {
  const float* qkv;     // [M][3 * d_model]: q | k | v as the projection left them
  const float2* rope;   // [max_ctx][hd / 2] or null
  uint16_t* Qp; uint16_t* Kp; uint16_t* Vp;
  float* Kc; float* Vc; // this layer's fp32 cache (the decode path's blocks): positions 0 .. M - 1 are filled as well
  int M, H, d_model, JP, max_ctx;
  float scale;          // factor on the queries: log2(e) / sqrt(hd), the softmax being evaluated as 2^(s - max)
};
struct PAttnArgs {
  const uint16_t* Qp; const uint16_t* Kp; const uint16_t* Vp;
  uint16_t* outp;       // the outputs in packed two-term form [2][MT][d_model / 32][64][8] (rows of the output projection)
  int M, H, d_model, JP;
};
// bytes of each of Qp, Kp, Vp
inline size_t pattn_stage_bytes(int M, int H, int HD) { return (size_t)2 * H * ((M + 31) / 32) * (HD / 16) * 1024; }

#ifdef PPD_PREFILL_TU
// One workgroup per (32 rows, head).
template <int HD>
__global__ __launch_bounds__(256) void pkv_pack_kernel(PKvPackArgs a) {
  constexpr int half = HD / 2, CB = HD / 32, CT = HD / 16, P8 = HD / 8;
  const int jp = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
  const size_t plane = (size_t)a.H * a.JP * CT * 512;      // bf16 elements per plane (the same for all three)
  // queries and keys: one 8-component piece of one row per item
  for (int it = tid; it < 32 * P8; it += 256) {
    const int rl = it / P8, c8 = it - rl * P8;             // row of the 32, piece
    const int m = 32 * jp + rl, i0 = 8 * c8;
    float q[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, k[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (m < a.M) {
      const float* r = a.qkv + (size_t)m * 3 * a.d_model + (size_t)h * HD;
      const float4 qa = *(const float4*)(r + i0), qb = *(const float4*)(r + i0 + 4);
      const float4 ka = *(const float4*)(r + a.d_model + i0), kb = *(const float4*)(r + a.d_model + i0 + 4);
      const float qv[8] = {qa.x, qa.y, qa.z, qa.w, qb.x, qb.y, qb.z, qb.w};
      const float kv[8] = {ka.x, ka.y, ka.z, ka.w, kb.x, kb.y, kb.z, kb.w};
      if (a.rope) {
        const int ip = i0 < half ? i0 + half : i0 - half;
        const float4 qc = *(const float4*)(r + ip), qd = *(const float4*)(r + ip + 4);
        const float4 kc = *(const float4*)(r + a.d_model + ip), kd = *(const float4*)(r + a.d_model + ip + 4);
        const float qo[8] = {qc.x, qc.y, qc.z, qc.w, qd.x, qd.y, qd.z, qd.w};
        const float ko[8] = {kc.x, kc.y, kc.z, kc.w, kd.x, kd.y, kd.z, kd.w};
        const float2* cz = a.rope + (size_t)m * half + (i0 < half ? i0 : i0 - half);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const float2 w = cz[u];
          if (i0 < half) { q[u] = fmaf(qv[u], w.x, -(qo[u] * w.y)); k[u] = fmaf(kv[u], w.x, -(ko[u] * w.y)); }
          else           { q[u] = fmaf(qv[u], w.x, qo[u] * w.y);    k[u] = fmaf(kv[u], w.x, ko[u] * w.y); }
        }
      } else {
#pragma unroll
        for (int u = 0; u < 8; ++u) { q[u] = qv[u]; k[u] = kv[u]; }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) q[u] *= a.scale;         // (scale carries log2(e): the attention kernel works with powers of two)
      // the cache takes the key as the decode path stores it: four components of one position are adjacent
      float* const kc = a.Kc + (size_t)h * kv_blocks(a.max_ctx) * (KV_BLOCK * HD);
      *(float4*)(kc + k_index(m, i0, HD)) = make_float4(k[0], k[1], k[2], k[3]);
      *(float4*)(kc + k_index(m, i0 + 4, HD)) = make_float4(k[4], k[5], k[6], k[7]);
    }
    const size_t o = ((((size_t)h * 2 * a.JP + 2 * jp + (rl >> 4)) * CB + (c8 >> 2)) * 64 + (rl & 15) + 16 * (c8 & 3)) * 8;
    uint4 hi, lo;
    split2(q, hi, lo);
    *(uint4*)(a.Qp + o) = hi; *(uint4*)(a.Qp + plane + o) = lo;
    split2(k, hi, lo);
    *(uint4*)(a.Kp + o) = hi; *(uint4*)(a.Kp + plane + o) = lo;
  }
  // values: one lane of one component tile per item
  for (int it = tid; it < CT * 64; it += 256) {
    const int ct = it >> 6, ln = it & 63, i = ln & 15, c = ln >> 4;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int m = 32 * jp + (e < 4 ? 4 * c + e : 16 + 4 * c + (e - 4));
      v[e] = m < a.M ? a.qkv[(size_t)m * 3 * a.d_model + 2 * (size_t)a.d_model + (size_t)h * HD + 16 * ct + i] : 0.f;
    }
    const size_t o = ((((size_t)h * a.JP + jp) * CT + ct) * 64 + ln) * 8;
    uint4 hi, lo;
    split2(v, hi, lo);
    *(uint4*)(a.Vp + o) = hi; *(uint4*)(a.Vp + plane + o) = lo;
    // the cache holds four consecutive positions of one component side by side: the lane's two quadruples
    float* const vc = a.Vc + (size_t)h * kv_blocks(a.max_ctx) * (KV_BLOCK * HD);
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const int m0 = 32 * jp + 16 * x + 4 * c;
      float* const dst = vc + v_index(m0, 16 * ct + i, HD);
      if (m0 + 3 < a.M) *(float4*)dst = make_float4(v[4 * x], v[4 * x + 1], v[4 * x + 2], v[4 * x + 3]);
      else for (int u = 0; u < 4; ++u) if (m0 + u < a.M) dst[u] = v[4 * x + u];
    }
  }
}

// A workgroup is 4 waves of one head; a wave owns QT consecutive 16-row query tiles (the columns of its MFMAs),
// the workgroup 64 QT consecutive rows.  The workgroup walks the 32-row steps of keys and values up to its last
// row: a step's blocks (keys hi, lo; values hi, lo: 4 HD / 16 KiB) come into LDS by direct loads, a step ahead of
// their use, two buffers; every wave reads them from there (a fourth of the traffic of four waves loading for
// themselves) and keeps a running maximum and sum per row.
template <int HD, int QT>
__global__ __launch_bounds__(256, (QT <= 2 ? 2 : 1)) void pattn_kernel(PAttnArgs a) {
  constexpr int CB = HD / 32, CT = HD / 16;
  constexpr int STEP_BLKS = 4 * CB + 2 * CT;               // 1 KiB blocks per step: K hi (2 CB), K lo (2 CB), V hi (CT), V lo (CT)
  extern __shared__ float4 pattn_lds4[];
  char* const lds = (char*)pattn_lds4;                     // [2][STEP_BLKS] KiB
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = blockIdx.y;
  const int wg = (int)gridDim.x - 1 - (int)blockIdx.x;     // the longest rows first
  const int MT2 = 2 * a.JP;
  const int qt0 = (wg * 4 + wave) * QT;                    // this wave's first tile (may lie past the prompt: then it only helps to load)
  const int bn = lane & 15, bc = lane >> 4;
  const size_t plane = (size_t)a.H * a.JP * CT * 1024;     // bytes per plane
  u32x4 qh[QT][CB], ql[QT][CB];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int tile = qt0 + t < MT2 ? qt0 + t : MT2 - 1;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      const char* src = (const char*)a.Qp + (((size_t)h * MT2 + tile) * CB + cb) * 1024 + lane * 16;
      qh[t][cb] = *(const u32x4*)src;
      ql[t][cb] = *(const u32x4*)(src + plane);
    }
  }
  f32x4 oacc[QT][CT];
  float mx[QT], l[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    mx[t] = -INFINITY; l[t] = 0.f;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) oacc[t][ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }
  int wg_last = (wg * 4 + 3) * QT + QT - 1;
  if (wg_last > MT2 - 1) wg_last = MT2 - 1;
  const int nsteps = wg_last / 2 + 1;                      // steps the workgroup walks (<= JP)
  auto stage = [&](int jp, int buf) {
    for (int b = wave; b < STEP_BLKS; b += 4) {
      const char* src;
      if (b < 4 * CB) {
        const int pl = b / (2 * CB), idx = b - pl * 2 * CB;
        src = (const char*)a.Kp + pl * plane + (((size_t)h * MT2 + 2 * jp) * CB + idx) * 1024;
      } else {
        const int bb = b - 4 * CB, pl = bb / CT, idx = bb - pl * CT;
        src = (const char*)a.Vp + pl * plane + (((size_t)h * a.JP + jp) * CT + idx) * 1024;
      }
      dma16(src + lane * 16, lds + ((size_t)buf * STEP_BLKS + b) * 1024);
    }
  };
  stage(0, 0);
  // the queries are waited for here, once: the compiler's own count of outstanding loads knows nothing of the
  // direct-to-LDS requests, and a wait for a query register inside the loop would drain the step in flight
#pragma unroll
  for (int t = 0; t < QT; ++t)
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) asm volatile("" : "+v"(qh[t][cb]), "+v"(ql[t][cb]));
  for (int jp = 0; jp < nsteps; ++jp) {
    // this step's blocks have arrived (this wave's requests, then everybody's); everybody is done with the other buffer
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (jp + 1 < nsteps) stage(jp + 1, (jp + 1) & 1);
    const char* const kb = lds + (size_t)(jp & 1) * STEP_BLKS * 1024 + lane * 16;
    const char* const vb = kb + 4 * CB * 1024;
    // the wave takes part while the step begins at or before the last row of its last tile; a tile that lies
    // wholly before the step is computed all the same and masked (its weights come out as exact zeros)
    if (2 * jp > qt0 + QT - 1) continue;
    f32x4 s[QT][2];
#pragma unroll
    for (int t = 0; t < QT; ++t) { s[t][0] = (f32x4){0.f, 0.f, 0.f, 0.f}; s[t][1] = (f32x4){0.f, 0.f, 0.f, 0.f}; }
    // (consecutive MFMAs go to different accumulators: none waits for the one before it)
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      bf16x8 kh[2], kl[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        kh[x] = __builtin_bit_cast(bf16x8, *(const u32x4*)(kb + (x * CB + cb) * 1024));
        kl[x] = __builtin_bit_cast(bf16x8, *(const u32x4*)(kb + ((2 + x) * CB + cb) * 1024));
      }
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int t = 0; t < QT; ++t) s[t][x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kh[x], __builtin_bit_cast(bf16x8, qh[t][cb]), s[t][x], 0, 0, 0);
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int t = 0; t < QT; ++t) s[t][x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kl[x], __builtin_bit_cast(bf16x8, qh[t][cb]), s[t][x], 0, 0, 0);
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int t = 0; t < QT; ++t) s[t][x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kh[x], __builtin_bit_cast(bf16x8, ql[t][cb]), s[t][x], 0, 0, 0);
    }
    // s[t][x][r]: row 32 jp + 16 x + 4 bc + r against query row 16 (qt0 + t) + bn
    const bool diag = 32 * jp + 31 > 16 * qt0;             // the step reaches past the first row of the wave's first tile
    u32x4 ph[QT], plo[QT];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      const int qrow = 16 * (qt0 + t) + bn;
      float sv[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) sv[e] = s[t][e >> 2][e & 3];
      if (diag) {                                          // mask what lies after each row
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (32 * jp + 16 * (e >> 2) + 4 * bc + (e & 3) > qrow) sv[e] = -INFINITY;
      }
      float bm = sv[0];
#pragma unroll
      for (int e = 1; e < 8; ++e) bm = fmaxf(bm, sv[e]);
      // the running maximum of a query is the same in its four lanes; it moves only when some lane of the wave has
      // met a larger score (rare after the first steps), and only then are the lanes compared and the sums rescaled
      if (__any(bm > mx[t])) {
        bm = fmaxf(bm, __shfl_xor(bm, 16, WAVE));
        bm = fmaxf(bm, __shfl_xor(bm, 32, WAVE));
        const float mnew = fmaxf(mx[t], bm);               // finite from the first step on: row 0 is visible to every query
        const float resc = __builtin_amdgcn_exp2f(mx[t] - mnew);
        mx[t] = mnew;
        l[t] *= resc;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
          for (int r = 0; r < 4; ++r) oacc[t][ct][r] *= resc;
      }
      float pv[8], ps = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) { pv[e] = __builtin_amdgcn_exp2f(sv[e] - mx[t]); ps += pv[e]; }
      l[t] += ps;                                          // this lane's 8 rows of the step; the four lanes of a query are added at the end
      uint4 hi, lo;
      split2(pv, hi, lo);
      ph[t] = (u32x4){hi.x, hi.y, hi.z, hi.w}; plo[t] = (u32x4){lo.x, lo.y, lo.z, lo.w};
    }
    // outputs: rows = components 16 ct + 4 bc + r, reduction over the step's 32 rows in the order Vp holds them
#pragma unroll
    for (int c2 = 0; c2 < CT; c2 += 2) {
      bf16x8 vh[2], vl[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        vh[x] = __builtin_bit_cast(bf16x8, *(const u32x4*)(vb + (c2 + x) * 1024));
        vl[x] = __builtin_bit_cast(bf16x8, *(const u32x4*)(vb + (CT + c2 + x) * 1024));
      }
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int t = 0; t < QT; ++t) oacc[t][c2 + x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vh[x], __builtin_bit_cast(bf16x8, ph[t]), oacc[t][c2 + x], 0, 0, 0);
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int t = 0; t < QT; ++t) oacc[t][c2 + x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vl[x], __builtin_bit_cast(bf16x8, ph[t]), oacc[t][c2 + x], 0, 0, 0);
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int t = 0; t < QT; ++t) oacc[t][c2 + x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vh[x], __builtin_bit_cast(bf16x8, plo[t]), oacc[t][c2 + x], 0, 0, 0);
    }
  }
  const int MT = (a.M + 15) / 16, KT = a.d_model / 32;
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int mrow = 16 * (qt0 + t) + bn;
    float lt = l[t];                                       // lanes bc = 0, 1, 2, 3 of the query, in that order
    {
      const float l1 = __shfl(lt, bn + 16, WAVE), l2 = __shfl(lt, bn + 32, WAVE), l3 = __shfl(lt, bn + 48, WAVE);
      lt = ((__shfl(lt, bn, WAVE) + l1) + l2) + l3;
    }
    if (mrow >= a.M) continue;
    const float inv = 1.0f / lt;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      const float y[4] = {oacc[t][ct][0] * inv, oacc[t][ct][1] * inv, oacc[t][ct][2] * inv, oacc[t][ct][3] * inv};
      put_packed4(a.outp, (size_t)MT * KT * 512, KT, mrow, h * HD + 16 * ct + 4 * bc, y);
    }
  }
}
#endif

// launchers (ppd_prefill.hip)
hipError_t launch_pack_rows(hipStream_t stream, const PackArgs& a);
hipError_t launch_pgemm(hipStream_t stream, PGemmArgs a, bool paired);
hipError_t launch_pkv_pack(hipStream_t stream, const PKvPackArgs& a, int head_dim);
hipError_t launch_pattn(hipStream_t stream, const PAttnArgs& a, int head_dim);
// bytes of the packed form of M rows of K columns
inline size_t packed_bytes(int M, int K) { return (size_t)2 * ((M + 15) / 16) * ((K + 31) / 32) * 1024; }

}  // namespace ppd
