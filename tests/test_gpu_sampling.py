"""GPU parity of the sampling-based final prediction (Appendix B): PPD against plain sampling on the GPU bit
for bit, every drawn token against the oracle's sampler on the GPU's own logits (both decide in fp64), and the
logits along the oracle's sampled sequence."""
import numpy as np
import pytest

import oracle
import ppd_inputs as pi
from gpu_common import TOL, gpu_generate
from helpers import small_cfg
from paper_2307_05908_amd import binding

pytestmark = pytest.mark.gpu

SEED = 20230713
MODES = [(oracle.TOP_K, 3, 1.0), (oracle.TOP_P, 0, 0.95), (oracle.TOP_P, 0, 0.3), (oracle.TOP_K, 8, 1.0)]


@pytest.fixture(scope="module", params=["tiny", "opt", "llama"])
def setup(request):
    cfg = small_cfg(request.param)
    m = pi.make_model(cfg)
    return cfg, m, binding.upload_model(m), oracle.Oracle(m)


@pytest.mark.parametrize("mode,ks,p", MODES)
def test_ppd_sampling_is_plain_sampling_bit_exact(setup, mode, ks, p):
    cfg, m, dev, o = setup
    prompt = pi.make_prompt(cfg)
    P = binding.PPD(cfg, dev, k=3)
    gtoks, _, _ = gpu_generate(P, prompt, cfg.n_gen, "plain", want_logits=False)
    P.ppd_set_sampling(mode, ks, p, SEED)
    ptoks, pz, _ = gpu_generate(P, prompt, cfg.n_gen, "plain")
    toks, z, infos = gpu_generate(P, prompt, cfg.n_gen, "ppd")
    np.testing.assert_array_equal(toks, ptoks)
    np.testing.assert_array_equal(z.view(np.uint32), pz.view(np.uint32))
    assert not np.array_equal(ptoks, gtoks)
    # every token is what the oracle's sampler draws from these very logits with that position's uniform
    for t in range(cfg.n_gen):
        u = oracle.uniform(SEED, len(prompt) + t)
        assert int(toks[t]) == oracle.sample(z[t].astype(np.float64), mode, ks, p, u), (t, u)
    # the match flag of a round compares the drawn token with the early candidates
    for t, (matched, midx, cand) in enumerate(infos):
        assert midx == (cand[:3].index(toks[t]) if toks[t] in cand[:3] else -1)
    # another seed draws another sequence; back to the arg max afterwards
    P.ppd_set_sampling(mode, ks, p, SEED + 1)
    other, _, _ = gpu_generate(P, prompt, cfg.n_gen, "ppd", want_logits=False)
    assert not np.array_equal(other, toks)
    P.ppd_set_sampling(0)
    back, _, _ = gpu_generate(P, prompt, cfg.n_gen, "ppd", want_logits=False)
    np.testing.assert_array_equal(back, gtoks)
    P.close()


def _kept_cdf(z, mode, ks, p):
    """Ranking and cumulative probabilities of the kept tokens (fp64, from the definition)."""
    order = np.lexsort((np.arange(len(z)), -z))
    w = np.exp(z[order] - z[order[0]])
    c = np.cumsum(w)
    keep = min(max(ks, 1), len(z)) if mode == oracle.TOP_K else int(np.argmax(c >= p * c[-1])) + 1
    return order[:keep], c[:keep] / c[keep - 1]


@pytest.mark.parametrize("mode,ks,p", MODES[:2])
def test_sampled_sequence_against_oracle(setup, mode, ks, p):
    """Along the oracle's own sampled sequence the logits agree within the tolerance; a token may differ from
    the oracle's only where that position's uniform falls within the tolerance of an edge of the token's
    interval of the cumulative distribution (then the GPU is put back on the oracle's sequence)."""
    cfg, m, dev, o = setup
    tol = TOL[cfg.wdtype]
    prompt = [int(x) for x in pi.make_prompt(cfg)]
    o.set_selection(mode, ks, p, SEED)
    ro = o.ppd(prompt, cfg.n_gen, 3, cfg.exit_layer, want_logits=True)
    o.set_selection(oracle.GREEDY)
    otoks, oz = ro["tokens"], ro["final_logits"]
    P = binding.PPD(cfg, dev, k=3)
    P.ppd_set_sampling(mode, ks, p, SEED)
    P.ppd_prefill(prompt)
    resyncs = 0
    for t in range(cfg.n_gen):
        tok, _ = P.ppd_step()
        z = P.ppd_get_logits().astype(np.float64)
        assert np.abs(z - oz[t]).max() <= tol
        if tok != int(otoks[t]):
            u = oracle.uniform(SEED, len(prompt) + t)
            kept, cdf = _kept_cdf(oz[t], mode, ks, p)
            where = np.nonzero(kept == tok)[0]
            # logits off by at most tol move every cumulative probability by less than 2 tol
            if len(where):
                j = int(where[0])
                lo, hi = (cdf[j - 1] if j else 0.0), cdf[j]
                assert lo - 2 * tol <= u <= hi + 2 * tol, (t, tok, int(otoks[t]), u, lo, hi)
            else:   # the token sits just outside the oracle's kept set: only possible at its very end
                assert oz[t][tok] >= oz[t][kept[-1]] - 2 * tol
            resyncs += 1
            P.ppd_prefill(prompt + [int(x) for x in otoks[:t + 1]])
    print(cfg.name, "mode", mode, "resyncs", resyncs)
    P.close()


@pytest.mark.parametrize("family", ["llama", "opt"])
def test_equal_logits_and_limits(family):
    """A zero LM head makes all logits equal: the ranking is by id and every mass is the same, so the draw is
    token floor(u n) (top-p with p = 1), floor(u ks) (top-k).  Also ks beyond the vocabulary and bad arguments."""
    cfg = small_cfg(family)
    m = pi.make_model(cfg)
    m.g["lm_head"] = np.zeros_like(m.g["lm_head"])
    if m.g.get("lnf_b") is not None:
        m.g["lnf_b"] = np.zeros_like(m.g["lnf_b"])
    dev = binding.upload_model(m)
    prompt = pi.make_prompt(cfg)
    P = binding.PPD(cfg, dev, k=3)
    for mode, ks, p in [(oracle.TOP_P, 0, 1.0), (oracle.TOP_P, 0, 0.5), (oracle.TOP_K, 5, 1.0), (oracle.TOP_K, cfg.vocab + 7, 1.0)]:
        P.ppd_set_sampling(mode, ks, p, SEED)
        P.ppd_prefill(prompt)
        for t in range(8):
            tok = P.plain_greedy_step() if t % 2 else P.ppd_step()[0]
            z = P.ppd_get_logits().astype(np.float64)
            assert np.all(z == 0.0)
            u = oracle.uniform(SEED, len(prompt) + t)
            assert tok == oracle.sample(z, mode, ks, p, u)
            n_kept = cfg.vocab if mode == oracle.TOP_P and p == 1.0 else (
                (cfg.vocab + 1) // 2 if mode == oracle.TOP_P else min(ks, cfg.vocab))
            assert tok == int(u * n_kept), (mode, ks, p, t, u, tok)
    for bad in [(3, 0, 1.0), (1, 0, 1.0), (2, 0, 0.0), (2, 0, 1.5)]:
        with pytest.raises(binding.PPDError) as ei:
            P.ppd_set_sampling(*bad, 0)
        assert ei.value.code == -1
    P.close()


@pytest.mark.parametrize("mode,ks,p", MODES[:3])
def test_vocabulary_beyond_the_on_chip_path(mode, ks, p):
    """More than 32768 logits do not fit the sampling kernel's registers and LDS: it then re-reads keys and
    weights from memory in every pass.  Same checks as above on a model with 33001 tokens."""
    cfg = small_cfg("opt", vocab=33001, n_gen=12)
    m = pi.make_model(cfg)
    dev = binding.upload_model(m)
    prompt = pi.make_prompt(cfg)
    P = binding.PPD(cfg, dev, k=3)
    P.ppd_set_sampling(mode, ks, p, SEED)
    ptoks, pz, _ = gpu_generate(P, prompt, cfg.n_gen, "plain")
    toks, z, _ = gpu_generate(P, prompt, cfg.n_gen, "ppd")
    np.testing.assert_array_equal(toks, ptoks)
    np.testing.assert_array_equal(z.view(np.uint32), pz.view(np.uint32))
    for t in range(cfg.n_gen):
        u = oracle.uniform(SEED, len(prompt) + t)
        assert int(toks[t]) == oracle.sample(z[t].astype(np.float64), mode, ks, p, u), (t, u)
    # equal logits through this path too: token floor(u n)
    m.g["lm_head"] = np.zeros_like(m.g["lm_head"])
    if m.g.get("lnf_b") is not None:
        m.g["lnf_b"] = np.zeros_like(m.g["lnf_b"])
    P2 = binding.PPD(cfg, binding.upload_model(m), k=3)
    P2.ppd_set_sampling(oracle.TOP_P, 0, 1.0, SEED)
    P2.ppd_prefill(prompt)
    for t in range(4):
        tok, _ = P2.ppd_step()
        assert tok == int(oracle.uniform(SEED, len(prompt) + t) * cfg.vocab)
    P.close()
    P2.close()
