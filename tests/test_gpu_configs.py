"""GPU parity at the benchmark configurations' own sizes.

opt125m runs the oracle live.  The 7B / 13B shapes compare against oracle outputs stored by
tests/golden/make_golden.py (tokens, and per generated position the final and early logits at 256
sampled vocabulary ids plus the oracle's top-8), and check PPD against plain greedy on the GPU bit
for bit.  A stored file is only used with the weights it was made from (checksum)."""
import os

import numpy as np
import pytest

import oracle
import ppd_inputs as pi
from gpu_common import TOL, gpu_generate, run_against_oracle, tripwire
from paper_2307_05908_amd import binding, tradeoff

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")
_cache = {}


def model_on_gpu(name):
    """One full-size model at a time on the host and on the GPU."""
    if _cache.get("name") != name:
        _cache.clear()
        import gc
        gc.collect()
        import torch
        torch.cuda.empty_cache()
        cfg = pi.CONFIGS[name]
        print("generating", name, flush=True)
        m = pi.make_model(cfg)
        _cache.update(name=name, cfg=cfg, m=m, dev=binding.upload_model(m))
    return _cache["cfg"], _cache["m"], _cache["dev"]


def test_opt125m_full_config_against_live_oracle():
    cfg, m, dev = model_on_gpu("opt125m")
    prompt = pi.make_prompt(cfg)
    o = oracle.Oracle(m, ctx_cap=cfg.n_prompt + cfg.n_gen + 1)
    ro = o.ppd(prompt, cfg.n_gen, cfg.k, cfg.exit_layer, want_logits=True)
    P = binding.PPD(cfg, dev)
    r = run_against_oracle(P, prompt, "ppd", ro["tokens"], ro["final_logits"], ro["early_logits"], tol=TOL[cfg.wdtype])
    print("opt125m ppd: max|dlogit|", r["max_err"], r["max_err_early"], "resyncs", r["resyncs"], "matches", r["matches"], flush=True)
    r = run_against_oracle(P, prompt, "plain", ro["tokens"], ro["final_logits"], tol=TOL[cfg.wdtype])
    print("opt125m plain: max|dlogit|", r["max_err"], "resyncs", r["resyncs"], flush=True)
    toks, z, infos = gpu_generate(P, prompt, cfg.n_gen, "ppd")
    ptoks, pz, _ = gpu_generate(P, prompt, cfg.n_gen, "plain")
    np.testing.assert_array_equal(toks, ptoks)
    np.testing.assert_array_equal(z, pz)


def test_llama7b_width_short_context_against_live_oracle():
    """Full 7B width and depth, short prompt: the oracle runs in the test (a few dozen token passes)."""
    cfg, m, dev = model_on_gpu("llama7b")
    prompt = pi.make_prompt(cfg, 20)
    o = oracle.Oracle(m, ctx_cap=40)
    ro = o.ppd(prompt, 8, 3, cfg.exit_layer, want_logits=True)
    P = binding.PPD(cfg, dev, k=3)
    r = run_against_oracle(P, prompt, "ppd", ro["tokens"], ro["final_logits"], ro["early_logits"], tol=2e-2)
    print("llama7b short: max|dlogit|", r["max_err"], r["max_err_early"], "resyncs", r["resyncs"], flush=True)
    o.close()


def check_against_golden(name, gname, ks):
    cfg, m, dev = model_on_gpu(name)
    g = np.load(os.path.join(GOLD, gname + ".npz"))
    if int(g["weights_checksum"]) != m.checksum():
        pytest.skip("stored oracle outputs were made from other weight bytes (different libm?); "
                    "regenerate with tests/golden/make_golden.py")
    prompt = pi.make_prompt(cfg)
    np.testing.assert_array_equal(prompt, g["prompt"])
    otoks, ids = g["tokens"], g["sample_ids"]
    ell, tol = len(otoks), 2e-2
    e = cfg.exit_layer
    # every logit of the vocabulary at a few positions, where such a file was stored
    full, fpath = {}, os.path.join(GOLD, gname + "_full.npz")
    if os.path.exists(fpath):
        gf = np.load(fpath)
        if int(gf["weights_checksum"]) == m.checksum() and np.array_equal(gf["tokens"], otoks):
            full = {int(p): (gf["final_logits"][i], gf["early_logits"][i]) for i, p in enumerate(gf["positions"])}
    worst_full = 0.0
    # plain greedy along the oracle's sequence: sampled logits, top-8, tokens
    P = binding.PPD(cfg, dev, k=ks[0])
    P.ppd_prefill(prompt)
    worst, resyncs = 0.0, 0
    plain_tokens, plain_logits = [], []
    for t in range(ell):
        tok = P.plain_greedy_step()
        z = P.ppd_get_logits()
        plain_tokens.append(tok)
        plain_logits.append(z)
        err = max(np.abs(z[ids] - g["final_samples"][t]).max(), np.abs(z[g["final_top_ids"][t]] - g["final_top_vals"][t]).max())
        worst = max(worst, float(err))
        assert err <= tol, f"{name}: final logits off by {err} at step {t}"
        if t in full and resyncs == 0:
            worst_full = max(worst_full, float(np.abs(z - full[t][0]).max()))
        if tok != int(otoks[t]):
            top_ids, top_vals = list(g["final_top_ids"][t]), g["final_top_vals"][t]
            assert tok in top_ids and top_vals[0] - top_vals[top_ids.index(tok)] < tol, f"{name}: token differs beyond margin at step {t}"
            resyncs += 1
            P.ppd_prefill(list(prompt) + [int(x) for x in otoks[:t + 1]])
    print(name, "plain vs stored oracle: max|dlogit|", worst, "resyncs", resyncs, flush=True)
    assert worst <= tripwire(cfg), f"{name}: {worst:.3g} is within the tolerance but past the regression tripwire"
    if full:
        print(name, "all", cfg.vocab, "logits at positions", sorted(full), ": max|dlogit|", worst_full, flush=True)
        assert worst_full <= tripwire(cfg)
    for k in ks:
        Pk = binding.PPD(cfg, dev, k=k) if k != ks[0] else P
        Pk.ppd_prefill(prompt)
        matches, resynced = 0, False
        for t in range(ell):
            tok, info = Pk.ppd_step()
            ze = Pk.ppd_get_early_logits()
            err = max(np.abs(ze[ids] - g["early_samples"][t]).max(), np.abs(ze[g["early_top_ids"][t]] - g["early_top_vals"][t]).max())
            assert err <= tol, f"{name} k={k}: early logits off by {err} at step {t}"
            if t in full and not resynced:
                assert np.abs(ze - full[t][1]).max() <= tripwire(cfg), f"{name} k={k}: an early logit outside the stored sample is off at step {t}"
            cand = list(info.cand)[:k]
            kth = g["early_top_vals"][t][k - 1]
            for c in cand:      # every candidate is within tol of making the oracle's top-k
                ov = g["early_top_vals"][t][list(g["early_top_ids"][t]).index(c)] if c in g["early_top_ids"][t] else None
                assert ov is not None and ov >= kth - tol
            assert info.match_idx == (cand.index(tok) if tok in cand else -1)
            matches += info.matched
            if not resynced:
                # PPD on the GPU is plain greedy on the GPU, bit for bit
                assert tok == plain_tokens[t]
                np.testing.assert_array_equal(Pk.ppd_get_logits(), plain_logits[t])
            if tok != int(otoks[t]):
                resynced = True
                Pk.ppd_prefill(list(prompt) + [int(x) for x in otoks[:t + 1]])
        st = Pk.ppd_get_stats()
        if not resynced:
            N = st["runs"]
            assert st["main_layer_rows"] == tradeoff.latency_of_runs(cfg.n_layers, e, ell, N)
            assert st["main_layer_rows"] + st["branch_layer_rows"] == tradeoff.compute_of_runs(cfg.n_layers, e, ell, k, N)
        print(name, "k", k, "p_correct", matches / ell, flush=True)
        if Pk is not P:
            Pk.close()
    P.close()
    return


def test_llama7b_full_config_k135():
    check_against_golden("llama7b", "llama7b", (3, 1, 5))


@pytest.mark.parametrize("mode,ks,p", [(oracle.TOP_K, 3, 1.0), (oracle.TOP_P, 0, 0.95)])
def test_llama7b_sampling_full_config(mode, ks, p):
    """Appendix B at the benchmark's own size (32000 logits, prompt 512, the launch configuration bench.py
    times): PPD draws the tokens of plain sampling bit for bit, and every token is the oracle's sampler's
    choice on the GPU's own logits with that position's uniform (both decide in fp64)."""
    cfg, m, dev = model_on_gpu("llama7b")
    prompt = pi.make_prompt(cfg)
    P = binding.PPD(cfg, dev)
    P.ppd_set_sampling(mode, ks, p, 77)
    n = 24
    toks, z, _ = gpu_generate(P, prompt, n, "ppd")
    ptoks, pz, _ = gpu_generate(P, prompt, n, "plain")
    np.testing.assert_array_equal(toks, ptoks)
    np.testing.assert_array_equal(z.view(np.uint32), pz.view(np.uint32))
    for t in range(n):
        u = oracle.uniform(77, len(prompt) + t)
        assert int(toks[t]) == oracle.sample(z[t].astype(np.float64), mode, ks, p, u), (t, u)
    P.close()


def test_llama7b_speculative_early_prediction_full_config(monkeypatch):
    """The (1 + k)-row final head of the 7B shape with a high match rate (alpha = 0.02 variant is not needed:
    the check is bit equality with rounds that run their own early head, whatever the rate)."""
    cfg, m, dev = model_on_gpu("llama7b")
    prompt = pi.make_prompt(cfg)

    def run():
        P = binding.PPD(cfg, dev, k=5)
        P.ppd_prefill(prompt)
        out = []
        for _ in range(32):
            tok, info = P.ppd_step(want_info=True)
            out.append((tok, info.matched, info.match_idx, tuple(info.cand[:5]),
                        P.ppd_get_logits().tobytes(), P.ppd_get_early_logits().tobytes()))
        st = P.ppd_get_stats()
        P.close()
        return out, st

    monkeypatch.setenv("PPD_SPEC", "1")
    a, sa = run()
    monkeypatch.setenv("PPD_SPEC", "2")
    b, sb = run()
    assert a == b
    follow = sum(1 for j in range(1, len(a)) if a[j - 1][1])
    assert sb["weight_bytes"] - sa["weight_bytes"] == follow * cfg.head_weight_bytes()


def test_llama7b_prompt_chunks_full_config(monkeypatch):
    """Prompt chunks at the 7B shape's own widths (16 rows staged in 2, 4 and 6 passes by the four GEMMs of a
    layer, causal attention over two 64-position chunks): the cache equals the token-by-token prefill's, so the
    rounds decoded from it are the same bit for bit."""
    cfg, m, dev = model_on_gpu("llama7b")
    prompt = pi.make_prompt(cfg, 100)

    def run():
        P = binding.PPD(cfg, dev, k=3)
        toks, z, _ = gpu_generate(P, prompt, 4, "ppd")
        P.close()
        return toks, z

    monkeypatch.setenv("PPD_PREFILL_TILED", "2")     # (the default for this prompt is the compute-bound pass)
    t16, z16 = run()
    monkeypatch.setenv("PPD_PREFILL_CHUNK", "1")
    t1, z1 = run()
    np.testing.assert_array_equal(t16, t1)
    np.testing.assert_array_equal(z16.view(np.uint32), z1.view(np.uint32))


@pytest.mark.parametrize("name", ["llama7b_a1", "llama7b_a0p1", "llama7b_a0p02"])
def test_llama7b_controlled_match_rate(name):
    if not os.path.exists(os.path.join(GOLD, name + ".npz")):
        pytest.skip("no stored oracle outputs for " + name)
    check_against_golden(name, name, (3,))


def test_llama13b_long_context():
    if not os.path.exists(os.path.join(GOLD, "llama13b.npz")):
        pytest.skip("no stored oracle outputs for llama13b")
    check_against_golden("llama13b", "llama13b", (3,))


def test_llama7b_width_exit_layer_24_against_live_oracle():
    """General exit layer (Algorithm 2) at full width: dbar = 24 of 32.  The candidates run layers 1..8; after a
    match the main token resumes at layer 9 and runs alone to layer 24 before the next early prediction.  The
    controlled-match-rate variant (late blocks damped) makes nearly every round match, so that path runs in
    every round; the oracle runs live (short context), all logits compared."""
    cfg, m, dev = model_on_gpu("llama7b_a0p1")
    prompt = pi.make_prompt(cfg, 20)
    o = oracle.Oracle(m, ctx_cap=40)
    ro = o.ppd(prompt, 8, 3, 24, want_logits=True)
    P = binding.PPD(cfg, dev, k=3, exit_layer=24)
    r = run_against_oracle(P, prompt, "ppd", ro["tokens"], ro["final_logits"], ro["early_logits"], tol=2e-2)
    print("llama7b dbar 24: max|dlogit|", r["max_err"], r["max_err_early"], "resyncs", r["resyncs"], "matches", r["matches"], flush=True)
    assert r["matches"] >= 6 and ro["stats"]["matches"] >= 6
    st = P.ppd_get_stats()
    if r["resyncs"] == 0:
        assert st["main_layer_rows"] == tradeoff.latency_of_runs(32, 24, 8, st["runs"])
    Q = binding.PPD(cfg, dev, k=3)
    ptoks, pz, _ = gpu_generate(Q, prompt, 8, "plain")
    toks, z, _ = gpu_generate(P, prompt, 8, "ppd")
    np.testing.assert_array_equal(toks, ptoks)
    np.testing.assert_array_equal(z.view(np.uint32), pz.view(np.uint32))
    o.close()
