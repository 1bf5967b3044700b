"""Pins of the oracle's sampling-based final prediction (Appendix B): the generator against its published
known-answer vectors, the samplers against closed forms and a library softmax, the decoding loops against
the exactness invariant (PPD draws the tokens non-PPD decoding draws from the same random stream)."""
import os

import numpy as np
import pytest
from scipy.special import softmax

import oracle
import ppd_inputs as pi
from helpers import small_cfg

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        out = oracle.philox4x32_10(w[0:4], w[4:6])
        assert [int(x) for x in out] == w[6:10]


def test_uniform_is_the_top_24_bits_of_the_first_word():
    for seed, idx in [(0, 0), (1234567890123, 17), (2**64 - 1, 2**40 + 5)]:
        out = oracle.philox4x32_10([idx & 0xffffffff, idx >> 32, 0, 0], [seed & 0xffffffff, seed >> 32])
        u = oracle.uniform(seed, idx)
        assert u == (int(out[0]) >> 8) / 2.0**24 and 0.0 <= u < 1.0
    # different positions and seeds give different numbers; mean of many is near 1/2
    us = np.array([oracle.uniform(7, i) for i in range(4000)])
    assert len(set(us)) > 3990 and abs(us.mean() - 0.5) < 0.02
    assert oracle.uniform(7, 3) != oracle.uniform(8, 3)


def test_two_token_closed_form():
    z = np.array([np.log(3.0), 0.0])             # probabilities 3/4, 1/4
    for u in np.linspace(0.0, 0.999, 50):
        assert oracle.sample(z, oracle.TOP_K, 2, 1.0, u) == (0 if u < 0.75 else 1)
        assert oracle.sample(z, oracle.TOP_P, 0, 1.0, u) == (0 if u < 0.75 else 1)
        assert oracle.sample(z, oracle.TOP_P, 0, 0.7, u) == 0      # the nucleus is token 0 alone
        assert oracle.sample(z, oracle.TOP_K, 1, 1.0, u) == 0
    # order of the ranking, not of the ids: the likelier token comes first
    z = np.array([0.0, np.log(3.0)])
    assert oracle.sample(z, oracle.TOP_K, 2, 1.0, 0.5) == 1 and oracle.sample(z, oracle.TOP_K, 2, 1.0, 0.8) == 0


def test_degenerate_cases_reduce_to_arg_max_or_uniform():
    rng = np.random.default_rng(3)
    z = rng.standard_normal(500)
    am = int(np.argmax(z))
    for u in (0.0, 0.3, 0.999999):
        assert oracle.sample(z, oracle.TOP_K, 1, 1.0, u) == am
        assert oracle.sample(z, oracle.TOP_P, 0, 1e-9, u) == am
        assert oracle.sample(z, oracle.GREEDY, 0, 0.0, u) == am
    assert oracle.sample(z, oracle.TOP_K, 50, 1.0, 0.0) == am and oracle.sample(z, oracle.TOP_P, 0, 0.9, 0.0) == am
    # equal logits: ranking by id, equal masses -> token floor(u n) (top-k: floor(u ks))
    z = np.zeros(64)
    for u in (0.0, 0.26, 0.5, 0.99):
        assert oracle.sample(z, oracle.TOP_P, 0, 1.0, u) == int(u * 64)
        assert oracle.sample(z, oracle.TOP_K, 8, 1.0, u) == int(u * 8)
    # p = 1/2 over equal logits keeps the first half of the ids
    assert oracle.sample(z, oracle.TOP_P, 0, 0.5, 0.99) == 31


@pytest.mark.parametrize("mode,ks,p", [(oracle.TOP_K, 3, 1.0), (oracle.TOP_K, 40, 1.0), (oracle.TOP_P, 0, 0.95),
                                       (oracle.TOP_P, 0, 0.5)])
def test_inversion_reproduces_the_truncated_softmax(mode, ks, p):
    """On an even grid of N values of u the number of draws of a token is N times its probability under the
    truncated, renormalised softmax (library softmax, truncation written out here), up to rounding."""
    rng = np.random.default_rng(11)
    z = rng.standard_normal(200) * 2.0
    prob = softmax(z)
    order = np.lexsort((np.arange(len(z)), -z))
    if mode == oracle.TOP_K:
        kept = order[:ks]
    else:
        c = np.cumsum(prob[order])
        kept = order[:int(np.searchsorted(c, p - 1e-15)) + 1]
    q = np.zeros_like(prob)
    q[kept] = prob[kept] / prob[kept].sum()
    N = 20000
    counts = np.bincount([oracle.sample(z, mode, ks, p, (i + 0.5) / N) for i in range(N)], minlength=len(z))
    assert counts[q == 0].sum() == 0
    assert np.abs(counts - q * N).max() <= 1.0 + 1e-6
    # and the draws walk the ranking: u increasing never moves to a likelier token
    ranks = np.empty(len(z), dtype=int)
    ranks[order] = np.arange(len(z))
    seq = [ranks[oracle.sample(z, mode, ks, p, (i + 0.5) / 50)] for i in range(50)]
    assert seq == sorted(seq)


@pytest.mark.parametrize("family", ["tiny", "opt", "llama"])
@pytest.mark.parametrize("mode,ks,p", [(oracle.TOP_K, 3, 1.0), (oracle.TOP_P, 0, 0.95)])
def test_ppd_with_sampling_draws_the_tokens_of_plain_sampling(family, mode, ks, p):
    """Appendix B changes only the final prediction; the exactness of Sec. 3 then reads: the same tokens as
    decoding without PPD from the same random stream.  Also against the cache-free whole-sequence forward."""
    cfg = small_cfg(family)
    m = pi.make_model(cfg)
    o = oracle.Oracle(m)
    prompt = pi.make_prompt(cfg)
    greedy = o.plain_greedy(prompt, 10)
    o.set_selection(mode, ks, p, seed=99)
    plain, z = o.plain_greedy(prompt, 10, want_logits=True)
    assert not np.array_equal(plain, greedy)            # random-init logits are nearly flat: sampling moves away
    np.testing.assert_array_equal(o.plain_recompute(prompt, 10), plain)
    for k in (1, 3):
        r = o.ppd(prompt, 10, k, cfg.exit_layer, want_logits=True)
        np.testing.assert_array_equal(r["tokens"], plain)
        np.testing.assert_allclose(r["final_logits"], z, rtol=0, atol=1e-9)
    # every token is the sampler's choice at that step's logits and that position's uniform
    for t in range(10):
        u = oracle.uniform(99, len(prompt) + t)
        assert plain[t] == oracle.sample(z[t], mode, ks, p, u)
    # another seed, another sequence
    o.set_selection(mode, ks, p, seed=100)
    assert not np.array_equal(o.plain_greedy(prompt, 10), plain)
    o.set_selection(oracle.GREEDY)
    np.testing.assert_array_equal(o.plain_greedy(prompt, 10), greedy)


def test_sampler_invariants_on_random_inputs():
    """Properties that hold for every input: the draw lies in the kept set; it does not move when a constant
    is added to all logits (large ones included: no overflow in the weights); it walks down the ranking as u
    grows; top-k sampling with everything kept is top-p sampling with p = 1."""
    rng = np.random.default_rng(5)
    for trial in range(60):
        n = int(rng.integers(2, 300))
        z = rng.standard_normal(n) * float(rng.choice([0.1, 1.0, 8.0]))
        if trial % 3 == 0:
            z[rng.integers(0, n, size=n // 2)] = z[0]            # ties
        order = np.lexsort((np.arange(n), -z))
        rank = np.empty(n, dtype=int)
        rank[order] = np.arange(n)
        ks = int(rng.integers(1, n + 1))
        p = float(rng.uniform(0.05, 1.0))
        prob = softmax(z)[order]
        m_p = int(np.searchsorted(np.cumsum(prob), p * (1 - 1e-12))) + 1
        last = {}
        for u in np.linspace(0.0, 0.9999, 23):
            tk = oracle.sample(z, oracle.TOP_K, ks, 1.0, u)
            tp = oracle.sample(z, oracle.TOP_P, 0, p, u)
            assert rank[tk] < ks
            assert rank[tp] < min(m_p + 1, n)                    # (+1: p S may fall on a cumulative sum's rounding)
            for shift in (1000.0, -1000.0):
                assert oracle.sample(z + shift, oracle.TOP_K, ks, 1.0, u) == tk
                assert oracle.sample(z + shift, oracle.TOP_P, 0, p, u) == tp
            for name, t in (("k", tk), ("p", tp)):
                assert rank[t] >= last.get(name, 0)
                last[name] = rank[t]
            assert oracle.sample(z, oracle.TOP_K, n, 1.0, u) == oracle.sample(z, oracle.TOP_P, 0, 1.0, u)
