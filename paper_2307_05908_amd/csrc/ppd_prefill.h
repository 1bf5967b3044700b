// Compute-bound prompt pass for bf16 models (gfx950).
//
// The method starts from a start token x_0 (Algorithm 1 / 2); a prompt is run through all d layers first to fill
// the key/value cache.  The decode kernels stream every weight once per 16 rows, which is the right shape for a
// handful of rows and the wrong one for a prompt: here the prompt's rows are a real matrix operand.
//
//   pack_rows_kernel    rows (after an optional norm) -> two bf16 terms x = hi + lo in MFMA operand blocks
//   pgemm_kernel        Y = epilogue(X W^T): register-tiled v_mfma_f32_16x16x32_bf16, weights in the repacked
//                       1 KiB blocks of the decode path (A operand), packed rows as B operand, both straight from
//                       memory (every wave-load is one contiguous kilobyte); products exact in fp32 as in decoding
//   pattn_kernel        causal attention of all prompt rows over the fp32 key/value cache (blocks that are
//                       v_mfma_f32_16x16x4_f32 operands), one wave per 16 query rows, running softmax
//
// Rounding order differs from the decode kernels (other tiles, other summation trees), so a cache filled here is
// close to, not bit-identical with, one filled row by row; every decode step after it is the same arithmetic
// whichever way the cache was filled, so PPD == plain greedy bit for bit still holds.
#pragma once
#include "ppd_kernels.h"

namespace ppd {

constexpr int PG_THREADS = 256;     // 4 waves
constexpr int PG_WAVES = PG_THREADS / WAVE;
constexpr int PG_TM = 4;            // 16-row tiles of the prompt per wave: 64 rows per workgroup
#ifndef PPD_PG_NBUF
#define PPD_PG_NBUF 4
#endif
constexpr int PG_NBUF = PPD_PG_NBUF;   // register buffers of operand blocks per wave

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
  int NB, MB;           // workgroup grid: NB blocks of 4 * TN tiles along the outputs, MB blocks of PG_TM tiles along the rows
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


// Workgroup b of the launch: an eighth of the output blocks per XCD (workgroups go round the XCDs in launch
// order), and all row blocks of an output block one after the other on the same XCD, so that a weight block is
// fetched from memory once and served to the other row blocks from that XCD's L2.
template <bool PAIRED, int TN>
__global__ __launch_bounds__(PG_THREADS) void pgemm_kernel(PGemmArgs a) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = blockIdx.x, xcd = b & 7, r = b >> 3;
  const int nb = (r / a.MB) * 8 + xcd, mb = r - (r / a.MB) * a.MB;
  if (nb >= a.NB) return;
  const int KT = a.KT;
  const int nt0 = (nb * PG_WAVES + wave) * TN, mt0 = mb * PG_TM;
  const size_t plane = (size_t)a.MT * KT * 1024;          // bytes per plane of the packed rows
  const char* wbase[TN]; const char* xbase[PG_TM];
#pragma unroll
  for (int t = 0; t < TN; ++t) {
    const int nt = nt0 + t < a.NT ? nt0 + t : a.NT - 1;   // (tiles past the matrix re-read its last tile; never stored)
    wbase[t] = (const char*)a.P + (size_t)nt * KT * 1024 + lane * 16;
  }
#pragma unroll
  for (int t = 0; t < PG_TM; ++t) {
    const int mt = mt0 + t < a.MT ? mt0 + t : a.MT - 1;
    xbase[t] = (const char*)a.Xp + (size_t)mt * KT * 1024 + lane * 16;
  }
  f32x4 acc[TN][PG_TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < PG_TM; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};
  // PG_NBUF register buffers: the blocks of the next PG_NBUF - 1 reduction steps are in flight while one is multiplied
  u32x4 wa[PG_NBUF][TN], xh[PG_NBUF][PG_TM], xl[PG_NBUF][PG_TM];
  auto fetch = [&](int kt, int buf) {
    const size_t o = (size_t)(kt < KT ? kt : KT - 1) * 1024;       // (requests past the end repeat the last block; unused)
#pragma unroll
    for (int t = 0; t < TN; ++t) wa[buf][t] = *(const u32x4*)(wbase[t] + o);
#pragma unroll
    for (int t = 0; t < PG_TM; ++t) { xh[buf][t] = *(const u32x4*)(xbase[t] + o); xl[buf][t] = *(const u32x4*)(xbase[t] + plane + o); }
  };
  // (all products with the first terms, then all with the second: no MFMA waits for the one before it)
  auto mac = [&](int buf) {
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int j = 0; j < PG_TM; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wa[buf][i]), __builtin_bit_cast(bf16x8, xh[buf][j]), acc[i][j], 0, 0, 0);
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int j = 0; j < PG_TM; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wa[buf][i]), __builtin_bit_cast(bf16x8, xl[buf][j]), acc[i][j], 0, 0, 0);
  };
#pragma unroll
  for (int p = 0; p < PG_NBUF - 1; ++p) fetch(p, p);
  int kt = 0;
  for (; kt + PG_NBUF <= KT; kt += PG_NBUF) {
#pragma unroll
    for (int p = 0; p < PG_NBUF; ++p) {
      fetch(kt + p + PG_NBUF - 1, (p + PG_NBUF - 1) % PG_NBUF);
      mac(p);
    }
  }
#pragma unroll
  for (int p = 0; p < PG_NBUF - 1; ++p)
    if (kt + p < KT) {
      fetch(kt + p + PG_NBUF - 1, (p + PG_NBUF - 1) % PG_NBUF);
      mac(p);
    }

  // ---- epilogue: lane l holds outputs 4 (l / 16) .. + 3 of the tile for row l % 16 of the row tile
  const int c = lane >> 4, mi = lane & 15;
  const uint16_t* const B0 = (const uint16_t*)a.B[0];
  const uint16_t* const B1 = (const uint16_t*)a.B[1];
  const uint16_t* const B2 = (const uint16_t*)a.B[2];
#pragma unroll
  for (int i = 0; i < TN; ++i) {
    const int nt = nt0 + i;
    if (nt >= a.NT) continue;
#pragma unroll
    for (int j = 0; j < PG_TM; ++j) {
      const int m = (mt0 + j) * 16 + mi;
      f32x4 v = acc[i][j];
      if (PAIRED) {
        // the tile's rows 0..7 are gate rows, 8..15 the up rows of the same 8 outputs: lanes c = 0, 1 take the
        // up values of lanes c + 2
        f32x4 u;
#pragma unroll
        for (int q = 0; q < 4; ++q) u[q] = __shfl(v[q], (lane + 32) & 63, WAVE);
        if (c >= 2 || mt0 + j >= a.MT || m >= a.M) continue;
        const int n0 = nt * 8 + c * 4;
        float y[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n0 + q < a.ntot ? n0 + q : a.ntot - 1;
          const float bg = B0 ? bf16_to_f32(B0[n]) : 0.f, bu = B1 ? bf16_to_f32(B1[n]) : 0.f;
          y[q] = silu(v[q] + bg) * (u[q] + bu);
        }
        if (a.Yp) {
          if (n0 >= a.ntot) continue;
#pragma unroll
          for (int q = 0; q < 4; ++q) if (n0 + q >= a.ntot) y[q] = 0.f;
          put_packed4(a.Yp, (size_t)a.MT * a.KTp * 512, a.KTp, m, n0, y);
          continue;
        }
        float* py = a.Y + (size_t)m * a.ldy + n0;
        if (n0 + 3 < a.ntot) *(float4*)py = make_float4(y[0], y[1], y[2], y[3]);
        else for (int q = 0; q < 4; ++q) if (n0 + q < a.ntot) py[q] = y[q];
      } else {
        if (mt0 + j >= a.MT || m >= a.M) continue;
        const int n0 = nt * 16 + c * 4;
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
          float t = v[q] + bv;
          if (a.act == 1) t = gelu_erf(t);
          else if (a.act == 2) t = fmaxf(t, 0.f);
          if (a.Rsd) t += a.Rsd[(size_t)m * a.ldy + n];
          y[q] = t;
        }
        if (a.Yp) {
          if (n0 >= a.ntot) continue;
#pragma unroll
          for (int q = 0; q < 4; ++q) if (n0 + q >= a.ntot) y[q] = 0.f;
          put_packed4(a.Yp, (size_t)a.MT * a.KTp * 512, a.KTp, m, n0, y);
          continue;
        }
        float* py = a.Y + (size_t)m * a.ldy + n0;
        if (n0 + 3 < a.ntot) *(float4*)py = make_float4(y[0], y[1], y[2], y[3]);
        else for (int q = 0; q < 4; ++q) if (n0 + q < a.ntot) py[q] = y[q];
      }
    }
  }
}

// ---- causal attention over the cache
// Row m of the prompt sits at position p0 + m and attends to cached positions [0, p0 + m]: the keys (rotated) and
// values of all rows are in the cache before this kernel runs (chunk_kv_kernel).  A wave owns 16 consecutive rows
// (the columns of its MFMAs) and walks the 16-position cache blocks up to its last row's position with a running
// maximum and sum; a workgroup is 4 such waves of one head.
struct PAttnArgs {
  const float* qkv;     // [M][3 * d_model]: q | k | v as the projection left them (q not yet rotated)
  const float* Kc; const float* Vc;   // this layer's cache
  const float2* rope;   // [max_ctx][hd / 2] or null
  const DevState* ds;   // row 0 sits at position ds->pos
  uint16_t* outp;       // the outputs in packed two-term form [2][MT][d_model / 32][64][8] (rows of the output projection)
  int M, H, d_model, max_ctx;
  float scale;
};

template <int HD>
__global__ __launch_bounds__(256) void pattn_kernel(PAttnArgs a) {
  constexpr int NS = HD / 16, half = HD / 2;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = blockIdx.y;
  const int qt = ((int)gridDim.x - 1 - (int)blockIdx.x) * 4 + wave;     // the longest rows first
  if (qt * 16 >= a.M) return;
  const int p0 = a.ds->pos;
  const int bn = lane & 15, bc = lane >> 4;
  const int mrow = qt * 16 + bn;                         // this lane's column: prompt row (may lie past M: computed, not stored)
  const int mq = mrow < a.M ? mrow : a.M - 1;
  const int pq = p0 + mq;                                // its position
  // the row's query, rotated and scaled: components 16 s + 4 bc + u
  f32x4 q4[NS];
  {
    const float* qr = a.qkv + (size_t)mq * 3 * a.d_model + (size_t)h * HD;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int i0 = 16 * s + 4 * bc;
      const float4 v = *(const float4*)(qr + i0);
      float x[4] = {v.x, v.y, v.z, v.w};
      if (a.rope) {
        const int ip = i0 < half ? i0 + half : i0 - half;
        const float4 o = *(const float4*)(qr + ip);
        const float xo[4] = {o.x, o.y, o.z, o.w};
        const float2* cz = a.rope + (size_t)pq * half + (i0 < half ? i0 : i0 - half);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float2 t = cz[u];
          x[u] = i0 < half ? fmaf(x[u], t.x, -(xo[u] * t.y)) : fmaf(x[u], t.x, xo[u] * t.y);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) q4[s][u] = x[u] * a.scale;
    }
  }
  const int plast = p0 + (qt * 16 + 15 < a.M ? qt * 16 + 15 : a.M - 1);      // last position any column of this wave sees
  const int nblk = plast / KV_BLOCK + 1;
  const size_t hb = (size_t)h * kv_blocks(a.max_ctx);
  const char* kb = (const char*)a.Kc + hb * (NS * 1024) + lane * 16;
  const char* vb = (const char*)a.Vc + hb * (NS * 1024) + lane * 16;
  f32x4 kreg[NS], vreg[NS], oacc[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) oacc[s] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float mx = -INFINITY, l = 0.f;
#pragma unroll
  for (int s = 0; s < NS; ++s) kreg[s] = *(const f32x4*)(kb + s * 1024);
#pragma unroll
  for (int s = 0; s < NS; ++s) vreg[s] = *(const f32x4*)(vb + s * 1024);
  for (int jb = 0; jb < nblk; ++jb) {
    // scores of the block's 16 positions for the wave's 16 rows: sacc[jj] = position 16 jb + 4 bc + jj, row bn
    f32x4 sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int u = 0; u < 4; ++u) sacc = __builtin_amdgcn_mfma_f32_16x16x4f32(kreg[s][u], q4[s][u], sacc, 0, 0, 0);
    const int jn = jb + 1 < nblk ? jb + 1 : jb;          // next block's keys (the last iteration repeats its own: unused)
#pragma unroll
    for (int s = 0; s < NS; ++s) kreg[s] = *(const f32x4*)(kb + ((size_t)jn * NS + s) * 1024);
    float bm = -INFINITY;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int j = jb * KV_BLOCK + 4 * bc + jj;
      if (j > pq) sacc[jj] = -INFINITY;
      bm = fmaxf(bm, sacc[jj]);
    }
    bm = fmaxf(bm, __shfl_xor(bm, 16, WAVE));
    bm = fmaxf(bm, __shfl_xor(bm, 32, WAVE));
    const float mnew = fmaxf(mx, bm);                    // finite from the first block on: position 0 is visible to every row
    const float resc = expf(mx - mnew);
    f32x4 p4;
    float ps = 0.f;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) { p4[jj] = expf(sacc[jj] - mnew); ps += p4[jj]; }
    ps += __shfl_xor(ps, 16, WAVE);
    ps += __shfl_xor(ps, 32, WAVE);
    l = fmaf(l, resc, ps);
    mx = mnew;
    // outputs: rows = components 16 s + 4 bc + jj, reduction over the block's positions 4 bc + u (p4 is the B operand as it stands)
#pragma unroll
    for (int s = 0; s < NS; ++s) {
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) oacc[s][jj] *= resc;
#pragma unroll
      for (int u = 0; u < 4; ++u) oacc[s] = __builtin_amdgcn_mfma_f32_16x16x4f32(vreg[s][u], p4[u], oacc[s], 0, 0, 0);
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) vreg[s] = *(const f32x4*)(vb + ((size_t)jn * NS + s) * 1024);
  }
  if (mrow < a.M) {
    const float inv = 1.0f / l;
    const int MT = (a.M + 15) / 16, KT = a.d_model / 32;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const float y[4] = {oacc[s][0] * inv, oacc[s][1] * inv, oacc[s][2] * inv, oacc[s][3] * inv};
      put_packed4(a.outp, (size_t)MT * KT * 512, KT, mrow, h * HD + 16 * s + 4 * bc, y);
    }
  }
}

// launchers (ppd_prefill.hip)
hipError_t launch_pack_rows(hipStream_t stream, const PackArgs& a);
hipError_t launch_pgemm(hipStream_t stream, PGemmArgs a, bool paired);
hipError_t launch_pattn(hipStream_t stream, const PAttnArgs& a, int head_dim);
// bytes of the packed form of M rows of K columns
inline size_t packed_bytes(int M, int K) { return (size_t)2 * ((M + 15) / 16) * ((K + 31) / 32) * 1024; }

}  // namespace ppd
