// Counter probe: a short PPD run through the C ABI without Python, for `rocprofv3 --pmc ... -- ./ppd_pmc_probe`.
//
// Builds a model of the 7B (or 13B) shape's widths with a few layers and cheap synthetic weights, feeds a prompt,
// runs some PPD rounds and plain steps, and one 1 GiB device-to-device copy (a kernel of known traffic against which
// the byte counters are scaled).  Every launch shape of a full-depth run occurs (a pipelined step does not depend on
// the depth), so FETCH_SIZE / WRITE_SIZE per dispatch can be read per kernel and launch shape.  Prints what it ran.
//
//   ppd_pmc_probe [shape: 7b | 13b] [layers] [prompt] [rounds]
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../../include/ppd.h"
#include "../../include/ppd_measure.h"

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)

static uint16_t bf16_of(float f) { uint32_t u; memcpy(&u, &f, 4); u += 0x7fffu + ((u >> 16) & 1u); return (uint16_t)(u >> 16); }

int main(int argc, char** argv) {
  const bool big = argc > 1 && !strcmp(argv[1], "13b");
  const int L = argc > 2 ? atoi(argv[2]) : 4, n_prompt = argc > 3 ? atoi(argv[3]) : 512, rounds = argc > 4 ? atoi(argv[4]) : 8;
  ppd_model_dims d; memset(&d, 0, sizeof d);
  d.n_layers = L; d.d_model = big ? 5120 : 4096; d.n_heads = big ? 40 : 32; d.head_dim = 128; d.d_ff = big ? 13824 : 11008;
  d.vocab = 32000; d.max_ctx = n_prompt + 2 * rounds + 64; d.norm = 1; d.act = 2; d.pos = 1; d.has_bias = 0; d.wdtype = 1;
  d.norm_eps = 1e-5f; d.rope_theta = 1e4f; d.eos_id = -1;
  if (L < 2 || L % 2 || n_prompt < 2 || rounds < 1) { fprintf(stderr, "usage: ppd_pmc_probe [7b|13b] [layers, even] [prompt] [rounds]\n"); return 1; }
  const size_t dm = d.d_model, F = d.d_ff, V = d.vocab;
  // one host pattern, as large as the largest tensor: values of standard deviation about 0.02
  const size_t nmax = V * dm > F * dm ? V * dm : F * dm;
  std::vector<uint16_t> pat(nmax);
  uint64_t x = 0x9E3779B97F4A7C15ull;
  for (size_t i = 0; i < nmax; ++i) { x = x * 6364136223846793005ull + 1442695040888963407ull; pat[i] = bf16_of(((int)((x >> 33) % 2001) - 1000) * 3.5e-5f); }
  std::vector<uint16_t> ones(dm, 0x3F80);
  std::vector<void*> owned;
  auto dev = [&](const uint16_t* src, size_t n, size_t shift) -> void* {
    void* p = nullptr;
    if (hipMalloc(&p, n * 2) != hipSuccess) return nullptr;
    owned.push_back(p);
    if (hipMemcpy(p, src + (shift % 4096), n * 2, hipMemcpyHostToDevice) != hipSuccess) return nullptr;   // (a shifted view: tensors differ)
    return p;
  };
  pat.resize(nmax + 4096, 0x3c00);
  ppd_weights w; memset(&w, 0, sizeof w);
  std::vector<const void*> ln1(L), ln2(L), wq(L), wk(L), wv(L), wo(L), win(L), wup(L), wout(L);
  for (int l = 0; l < L; ++l) {
    ln1[l] = dev(ones.data(), dm, 0); ln2[l] = dev(ones.data(), dm, 0);
    wq[l] = dev(pat.data(), dm * dm, 7 * l + 1); wk[l] = dev(pat.data(), dm * dm, 7 * l + 2); wv[l] = dev(pat.data(), dm * dm, 7 * l + 3);
    wo[l] = dev(pat.data(), dm * dm, 7 * l + 4); win[l] = dev(pat.data(), F * dm, 7 * l + 5); wup[l] = dev(pat.data(), F * dm, 7 * l + 6);
    wout[l] = dev(pat.data(), dm * F, 7 * l + 7);
    if (!ln1[l] || !ln2[l] || !wq[l] || !wk[l] || !wv[l] || !wo[l] || !win[l] || !wup[l] || !wout[l]) { fprintf(stderr, "allocation failed\n"); return 2; }
  }
  w.tok_emb = dev(pat.data(), V * dm, 11); w.lm_head = dev(pat.data(), V * dm, 13); w.lnf_g = dev(ones.data(), dm, 0);
  if (!w.tok_emb || !w.lm_head || !w.lnf_g) { fprintf(stderr, "allocation failed\n"); return 2; }
  w.ln1_g = ln1.data(); w.ln2_g = ln2.data(); w.wq = wq.data(); w.wk = wk.data(); w.wv = wv.data(); w.wo = wo.data();
  w.w_in = win.data(); w.w_up = wup.data(); w.w_out = wout.data();
  CK(hipDeviceSynchronize());
  ppd_ctx* c = nullptr;
  int rc = ppd_create(&d, &w, 3, L / 2, nullptr, &c);
  if (rc) { fprintf(stderr, "ppd_create: %s (hip %d)\n", ppd_strerror(rc), ppd_last_hip_error(nullptr)); return 2; }
  std::vector<int32_t> prompt(n_prompt);
  for (int i = 0; i < n_prompt; ++i) { x = x * 6364136223846793005ull + 1442695040888963407ull; prompt[i] = (int32_t)((x >> 33) % V); }
  if ((rc = ppd_prefill(c, prompt.data(), n_prompt))) { fprintf(stderr, "ppd_prefill: %s\n", ppd_strerror(rc)); return 2; }
  int32_t tok = 0; int hits = 0;
  for (int r = 0; r < rounds; ++r) {
    ppd_step_info info;
    if ((rc = ppd_step(c, &tok, 1, &info)) < 0) { fprintf(stderr, "ppd_step: %s\n", ppd_strerror(rc)); return 2; }
    hits += info.matched;
  }
  for (int r = 0; r < rounds; ++r)
    if ((rc = plain_greedy_step(c, &tok)) < 0) { fprintf(stderr, "plain_greedy_step: %s\n", ppd_strerror(rc)); return 2; }
  ppd_destroy(c);
  // the kernel of known traffic: 1 GiB read, 1 GiB written
  void *a = nullptr, *b = nullptr;
  CK(hipMalloc(&a, (size_t)1 << 30)); CK(hipMalloc(&b, (size_t)1 << 30));
  CK(hipMemset(a, 1, (size_t)1 << 30));
  CK(hipMemcpy(b, a, (size_t)1 << 30, hipMemcpyDeviceToDevice));
  CK(hipDeviceSynchronize());
  CK(hipFree(a)); CK(hipFree(b));
  for (void* p : owned) (void)hipFree(p);
  printf("ppd_pmc_probe: %s widths, %d layers, prompt %d, %d PPD rounds (%d matched) + %d plain steps, 1 GiB copy\n",
         big ? "13b" : "7b", L, n_prompt, rounds, hits, rounds);
  return 0;
}
