/* Seeded synthetic inputs: counter-based normal / uniform generators.
 *
 * This file holds no arithmetic of the decoding method.  It only turns
 * (seed, stream, index) into reproducible numbers, so that the CPU oracle and
 * the GPU library can be handed the very same bytes.
 *
 * Element i of stream s under seed z is a pure function of (z, s, i): a
 * 64-bit mixing hash of the pair index gives two uniforms, Box-Muller turns
 * them into two standard normals, element i takes the (i & 1)-th of them.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

static inline uint64_t key_of(uint64_t seed, uint64_t stream) {
  return mix64(mix64(seed) ^ (stream * 0xD6E8FEB86659FD93ull));
}

/* two standard normals for pair index p */
static inline void normal_pair(uint64_t key, uint64_t p, double *z0, double *z1) {
  uint64_t a = mix64(key ^ (2 * p));
  uint64_t b = mix64(key ^ (2 * p + 1));
  /* u1 in (0,1], u2 in [0,1): 53-bit mantissas */
  double u1 = ((double)(a >> 11) + 1.0) * (1.0 / 9007199254740992.0);
  double u2 = (double)(b >> 11) * (1.0 / 9007199254740992.0);
  double r = sqrt(-2.0 * log(u1));
  double th = 6.283185307179586476925286766559 * u2;
  *z0 = r * cos(th);
  *z1 = r * sin(th);
}

static inline uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40); /* NaN */
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

/* out[i] = (float)(mean + std * z_i) * scale, rounded once more to bf16 when
 * as_bf16 != 0 (round-to-nearest-even).  scale is applied in fp32. */
void ppd_inputs_fill_normal(void *out, size_t n, uint64_t seed, uint64_t stream,
                            double mean, double std, float scale, int as_bf16) {
  uint64_t key = key_of(seed, stream);
  size_t npairs = (n + 1) / 2;
#pragma omp parallel for schedule(static)
  for (size_t p = 0; p < npairs; ++p) {
    double z[2];
    normal_pair(key, p, &z[0], &z[1]);
    for (int j = 0; j < 2; ++j) {
      size_t i = 2 * p + j;
      if (i >= n) break;
      float v = (float)(mean + std * z[j]) * scale;
      if (as_bf16) ((uint16_t *)out)[i] = f32_to_bf16_rne(v);
      else ((float *)out)[i] = v;
    }
  }
}

/* out[i] uniform on [0, vocab) */
void ppd_inputs_fill_tokens(int32_t *out, size_t n, uint64_t seed, uint64_t stream,
                            int32_t vocab) {
  uint64_t key = key_of(seed, stream);
  for (size_t i = 0; i < n; ++i) {
    uint64_t h = mix64(key ^ i);
    out[i] = (int32_t)(((unsigned __int128)h * (uint64_t)vocab) >> 64);
  }
}

/* 64-bit FNV-1a over raw bytes: used to label a generated model in stored
 * fixtures so a fixture is never compared against different weights. */
uint64_t ppd_inputs_checksum(const void *buf, size_t nbytes, uint64_t h) {
  const unsigned char *p = (const unsigned char *)buf;
  if (h == 0) h = 0xcbf29ce484222325ull;
  for (size_t i = 0; i < nbytes; ++i) { h ^= p[i]; h *= 0x100000001b3ull; }
  return h;
}
