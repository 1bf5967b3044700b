"""Pins of the CPU oracle against things other than itself: library routines
(numpy / torch CPU fp64), closed forms, the paper's exactness invariant and
its counter identities, brute force on tiny inputs."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import ppd_inputs as pi
from helpers import small_cfg
from paper_2307_05908_amd import tradeoff

FAMILIES = ["tiny", "opt", "llama"]


def _t(a):
    return torch.from_numpy(pi.to_float64(a)) if a is not None else None


@pytest.fixture(scope="module", params=FAMILIES)
def fam(request):
    cfg = small_cfg(request.param)
    m = pi.make_model(cfg)
    return cfg, m, oracle.Oracle(m)


# ---------------------------------------------------------------- sub-ops
def test_linear_is_numpy_matvec(fam):
    cfg, m, o = fam
    rng = np.random.default_rng(1)
    W, b = m.layers["w_in"][1], m.layers["b_in"][1]
    x = rng.standard_normal(cfg.d_model)
    ref = pi.to_float64(W) @ x + (pi.to_float64(b) if b is not None else 0.0)
    np.testing.assert_allclose(o.linear(W, b, x), ref, rtol=0, atol=1e-12)
    # transposed-operand mistake would need a square matrix to even run: check one
    Wq = m.layers["wq"][0]
    x = rng.standard_normal(cfg.d_model)
    np.testing.assert_allclose(o.linear(Wq, None, x), pi.to_float64(Wq) @ x, rtol=0, atol=1e-12)
    assert np.abs(pi.to_float64(Wq).T @ x - pi.to_float64(Wq) @ x).max() > 1e-3


def test_norm_is_torch_norm(fam):
    cfg, m, o = fam
    x = np.random.default_rng(2).standard_normal(cfg.d_model) * 3 + 0.5
    g, b = m.layers["ln2_g"][0], m.layers["ln2_b"][0]
    if cfg.norm == pi.NORM_LAYERNORM:
        ref = F.layer_norm(torch.from_numpy(x), (cfg.d_model,), _t(g), _t(b), cfg.norm_eps)
    else:
        ref = F.rms_norm(torch.from_numpy(x), (cfg.d_model,), _t(g), cfg.norm_eps)
    np.testing.assert_allclose(o.norm(g, b, x), ref.numpy(), rtol=0, atol=1e-12)


def test_activations_are_torch_activations():
    u = torch.linspace(-6, 6, 241, dtype=torch.float64)
    for kind, ref in ((pi.ACT_GELU, F.gelu(u)), (pi.ACT_RELU, F.relu(u)), (pi.ACT_SWIGLU, F.silu(u))):
        got = np.array([oracle.act(kind, float(v)) for v in u])
        np.testing.assert_allclose(got, ref.numpy(), rtol=0, atol=1e-13)


def test_rope_is_complex_rotation_and_relative():
    cfg = small_cfg("llama")
    m = pi.make_model(cfg)
    o = oracle.Oracle(m)
    rng = np.random.default_rng(3)
    hd, H, half = cfg.head_dim, cfg.n_heads, cfg.head_dim // 2
    q, k = rng.standard_normal(cfg.d_model), rng.standard_normal(cfg.d_model)
    np.testing.assert_array_equal(o.rope(q, 0), q)          # position 0: identity
    for pos in (1, 7, 95):
        r = o.rope(q, pos).reshape(H, hd)
        z = q.reshape(H, hd)[:, :half] + 1j * q.reshape(H, hd)[:, half:]
        ang = pos * cfg.rope_theta ** (-2.0 * np.arange(half) / hd)
        zr = z * np.exp(1j * ang)                            # textbook form: complex multiplication
        np.testing.assert_allclose(r[:, :half], zr.real, atol=1e-12)
        np.testing.assert_allclose(r[:, half:], zr.imag, atol=1e-12)
        np.testing.assert_allclose(np.linalg.norm(r, axis=1), np.linalg.norm(q.reshape(H, hd), axis=1), rtol=1e-12)
    # the score of a (query, key) pair depends on the position difference only
    s1 = (o.rope(q, 9).reshape(H, hd) * o.rope(k, 4).reshape(H, hd)).sum(1)
    s2 = (o.rope(q, 40).reshape(H, hd) * o.rope(k, 35).reshape(H, hd)).sum(1)
    np.testing.assert_allclose(s1, s2, atol=1e-10)


# ------------------------------------------------- whole forward vs torch
def torch_forward(cfg, m, tokens):
    """The same transformer written with torch's library routines, fp64, matrix form."""
    n, dm, H, hd = len(tokens), cfg.d_model, cfg.n_heads, cfg.head_dim
    tok = torch.as_tensor(np.asarray(tokens), dtype=torch.long)
    x = _t(m.g["tok_emb"])[tok]
    if cfg.pos == pi.POS_LEARNED:
        x = x + _t(m.g["pos_emb"])[:n]

    def norm(v, g, b):
        if cfg.norm == pi.NORM_LAYERNORM:
            return F.layer_norm(v, (dm,), _t(g), _t(b), cfg.norm_eps)
        return F.rms_norm(v, (dm,), _t(g), cfg.norm_eps)

    def rope(v):  # v: [n, H, hd]
        if cfg.pos != pi.POS_ROPE:
            return v
        half = hd // 2
        inv = cfg.rope_theta ** (-torch.arange(half, dtype=torch.float64) * 2.0 / hd)
        ang = torch.arange(n, dtype=torch.float64)[:, None] * inv[None, :]
        rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]
        z = torch.complex(v[..., :half], v[..., half:]) * rot
        return torch.cat([z.real, z.imag], dim=-1)

    L = m.layers
    for l in range(cfg.n_layers):
        a = norm(x, L["ln1_g"][l], L["ln1_b"][l])
        q = F.linear(a, _t(L["wq"][l]), _t(L["bq"][l])).view(n, H, hd)
        k = F.linear(a, _t(L["wk"][l]), _t(L["bk"][l])).view(n, H, hd)
        v = F.linear(a, _t(L["wv"][l]), _t(L["bv"][l])).view(n, H, hd)
        q, k = rope(q), rope(k)
        att = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1), is_causal=True)
        x = x + F.linear(att.transpose(0, 1).reshape(n, dm), _t(L["wo"][l]), _t(L["bo"][l]))
        a = norm(x, L["ln2_g"][l], L["ln2_b"][l])
        u = F.linear(a, _t(L["w_in"][l]), _t(L["b_in"][l]))
        if cfg.act == pi.ACT_SWIGLU:
            u = F.silu(u) * F.linear(a, _t(L["w_up"][l]))
        elif cfg.act == pi.ACT_GELU:
            u = F.gelu(u)
        else:
            u = F.relu(u)
        x = x + F.linear(u, _t(L["w_out"][l]), _t(L["b_out"][l]))
    return F.linear(norm(x, m.g["lnf_g"], m.g["lnf_b"]), _t(m.g["lm_head"])).numpy()


def test_full_forward_is_torch_forward(fam):
    cfg, m, o = fam
    toks = pi.make_prompt(cfg, 23)
    np.testing.assert_allclose(o.full_forward(toks), torch_forward(cfg, m, toks), rtol=0, atol=1e-10)


def test_uniform_attention_closed_form():
    """With W_q = 0 every score is 0, so attention is the plain mean of the values."""
    cfg = small_cfg("tiny", n_layers=1, has_bias=0)
    m = pi.make_model(cfg)
    m.layers["wq"][0][:] = 0
    for b in ("bq", "bk", "bv", "bo", "b_in", "b_out"):
        m.layers[b][0] = None
    o = oracle.Oracle(m)
    toks = pi.make_prompt(cfg, 5)
    f64 = pi.to_float64
    x = f64(m.g["tok_emb"])[toks] + f64(m.g["pos_emb"])[:5]

    def ln(v, g, b):
        return (v - v.mean(-1, keepdims=True)) / np.sqrt(v.var(-1, keepdims=True) + cfg.norm_eps) * f64(g) + f64(b)

    v = ln(x, m.layers["ln1_g"][0], m.layers["ln1_b"][0]) @ f64(m.layers["wv"][0]).T
    att = np.cumsum(v, 0) / np.arange(1, 6)[:, None]
    x = x + att @ f64(m.layers["wo"][0]).T
    u = ln(x, m.layers["ln2_g"][0], m.layers["ln2_b"][0]) @ f64(m.layers["w_in"][0]).T
    from scipy.special import erf
    x = x + (0.5 * u * (1 + erf(u / np.sqrt(2)))) @ f64(m.layers["w_out"][0]).T
    z = ln(x, m.g["lnf_g"], m.g["lnf_b"]) @ f64(m.g["lm_head"]).T
    np.testing.assert_allclose(o.full_forward(toks), z, rtol=0, atol=1e-10)


# -------------------------------------------------- cache, PPD, counters
def test_cached_greedy_equals_recompute(fam):
    cfg, m, o = fam
    p = pi.make_prompt(cfg, 9)
    t1, z1 = o.plain_greedy(p, 10, want_logits=True)
    t2, z2 = o.plain_recompute(p, 10, want_logits=True)
    np.testing.assert_array_equal(t1, t2)
    np.testing.assert_allclose(z1, z2, rtol=0, atol=1e-10)
    # and the greedy choice is the brute-force arg max of those logits
    np.testing.assert_array_equal(t1, z2.argmax(1))


def test_teacher_forced_reproduces_greedy_logits(fam):
    cfg, m, o = fam
    p = pi.make_prompt(cfg, 9)
    t1, z1 = o.plain_greedy(p, 6, want_logits=True)
    seq = np.concatenate([p, t1[:-1]])
    zf, ze = o.teacher_forced(seq, len(p) - 1, dbar=cfg.exit_layer)
    np.testing.assert_array_equal(zf, z1)
    r = o.ppd(p, 6, 2, cfg.exit_layer, want_logits=True)
    np.testing.assert_array_equal(ze, r["early_logits"])


@pytest.mark.parametrize("k", [1, 3, 5])
def test_ppd_output_is_greedy_output_and_counters_hold(fam, k):
    """Sec. 1 / Sec. 3: PPD keeps the exact decoding result.  Proof of Theorem 4.1:
    latency = dbar*l + (d-dbar)*N, compute = (dbar + k(d-dbar))*l + (d-dbar)*N,
    N - 1 = number of failed early predictions among the first l-1."""
    cfg, m, o = fam
    d, ell = cfg.n_layers, cfg.n_gen
    p = pi.make_prompt(cfg)
    plain, zp = o.plain_greedy(p, ell, want_logits=True)
    for dbar in range((d + 1) // 2, d + 1):
        r = o.ppd(p, ell, k, dbar, want_logits=True)
        np.testing.assert_array_equal(r["tokens"], plain)
        np.testing.assert_array_equal(r["final_logits"], zp)
        st = r["stats"]
        hit = r["match_idx"] >= 0
        # a candidate matches iff the final token is among the early top-k, at the reported index
        for t in range(ell):
            where = np.nonzero(r["cand"][t] == plain[t])[0]
            assert (r["match_idx"][t] == (where[0] if len(where) else -1))
            assert len(set(r["cand"][t])) == k
        N = 1 + int((~hit[:ell - 1]).sum())
        assert st["runs"] == N and st["rounds"] == ell and st["matches"] == int(hit.sum())
        assert st["main_layer_rows"] == tradeoff.latency_of_runs(d, dbar, ell, N)
        assert st["main_layer_rows"] + st["branch_layer_rows"] == tradeoff.compute_of_runs(d, dbar, ell, k, N)


def test_ppd_odd_depth():
    cfg = small_cfg("llama", n_layers=5, exit_layer=3)
    m = pi.make_model(cfg)
    o = oracle.Oracle(m)
    p = pi.make_prompt(cfg)
    plain = o.plain_greedy(p, 12)
    for dbar in (3, 4, 5):
        np.testing.assert_array_equal(o.ppd(p, 12, 2, dbar)["tokens"], plain)
    with pytest.raises(ValueError):
        o.ppd(p, 12, 2, 2)  # dbar < d/2 is outside Theorem 4.1's range


def test_match_nesting_in_k(fam):
    """Sec. 4.3: a larger k can only raise the match rate; per position the
    top-1 set is inside the top-3 set inside the top-5 set."""
    cfg, m, o = fam
    p = pi.make_prompt(cfg)
    hits = {k: o.ppd(p, cfg.n_gen, k, cfg.exit_layer)["match_idx"] >= 0 for k in (1, 3, 5)}
    assert not (hits[1] & ~hits[3]).any() and not (hits[3] & ~hits[5]).any()


@pytest.mark.parametrize("family", ["opt", "llama"])
def test_alpha_zero_gives_match_rate_one_and_fig2(family):
    """If the blocks after the exit layer add nothing, the early logits are the final
    logits, every round matches at index 0, and the whole text is one run.
    Fig. 2: run length 3, k = 3, p = 1: latency d + 2*dbar, 4 units busy for 3(d-dbar)."""
    cfg = small_cfg(family, alpha=0.0)
    m = pi.make_model(cfg)
    d, dbar = cfg.n_layers, cfg.exit_layer
    for l in range(dbar, d):          # alpha scales the two output matrices; silence their biases too
        for b in ("bo", "b_out"):
            if m.layers[b][l] is not None:
                m.layers[b][l][:] = 0
    o = oracle.Oracle(m)
    p = pi.make_prompt(cfg)
    r = o.ppd(p, 3, 3, dbar, want_logits=True)
    assert (r["match_idx"] == 0).all()
    np.testing.assert_array_equal(r["early_logits"], r["final_logits"])
    assert r["stats"]["runs"] == 1
    assert r["stats"]["main_layer_rows"] == d + 2 * dbar == tradeoff.run_time(d, dbar, 3)
    assert r["stats"]["branch_layer_rows"] == 3 * 3 * (d - dbar)


def test_k_equal_vocab_always_matches():
    cfg = small_cfg("tiny", vocab=48)
    m = pi.make_model(cfg)
    o = oracle.Oracle(m)
    r = o.ppd(pi.make_prompt(cfg), 8, 48, 2)
    assert (r["match_idx"] >= 0).all()
    np.testing.assert_array_equal(r["tokens"], o.plain_greedy(pi.make_prompt(cfg), 8))


def test_topk_and_argmax_bruteforce():
    rng = np.random.default_rng(5)
    for trial in range(20):
        z = np.round(rng.standard_normal(200), 1)  # many exact ties
        order = np.lexsort((np.arange(200), -z))    # (value desc, id asc): full sort
        for k in (1, 3, 8):
            np.testing.assert_array_equal(oracle.topk(z, k), order[:k])
        assert oracle.argmax(z) == order[0]


def test_eos_stops_both():
    cfg = small_cfg("tiny")
    m = pi.make_model(cfg)
    o = oracle.Oracle(m)
    p = pi.make_prompt(cfg)
    full = o.plain_greedy(p, 12)
    eos = int(full[4])
    first = int(np.nonzero(full == eos)[0][0])
    a = o.plain_greedy(p, 12, eos=eos)
    b = o.ppd(p, 12, 3, 2, eos=eos)["tokens"]
    np.testing.assert_array_equal(a, full[:first + 1])
    np.testing.assert_array_equal(b, a)


# ------------------------------------------------ separate early classifier
class _Shallow:
    """The first `n` blocks of a model with another classifier matrix (for torch_forward)."""

    def __init__(self, m, n, head):
        self.cfg = m.cfg.replace(n_layers=n)
        self.g = dict(m.g, lm_head=head)
        self.layers = m.layers


def test_early_head_is_the_classifier_of_the_truncated_model(fam):
    """Sec. 4.3: the early prediction may use a classifier trained for the exit layer.  With such a matrix E
    the early logits of round t are E . Norm_f(h_dbar), i.e. the output of the same transformer cut after dbar
    blocks with E as its classifier (library forward, fp64); the candidates are their top-k by a full sort;
    the emitted tokens and final logits stay those of plain greedy decoding."""
    cfg, m, o = fam
    E = pi.make_early_head(cfg)
    oe = oracle.Oracle(m, early_head=E)
    p, ell, k = pi.make_prompt(cfg, 9), 8, 3
    plain, zp = o.plain_greedy(p, ell, want_logits=True)
    seq = np.concatenate([p, plain[:-1]])
    d = cfg.n_layers
    for dbar in sorted({(d + 1) // 2, d - 1}):
        r = oe.ppd(p, ell, k, dbar, want_logits=True)
        np.testing.assert_array_equal(r["tokens"], plain)
        np.testing.assert_array_equal(r["final_logits"], zp)
        zt = torch_forward(cfg.replace(n_layers=dbar), _Shallow(m, dbar, E), seq)[len(p) - 1:]
        np.testing.assert_allclose(r["early_logits"], zt, rtol=0, atol=1e-10)
        for t in range(ell):
            order = np.lexsort((np.arange(cfg.vocab), -r["early_logits"][t]))
            np.testing.assert_array_equal(r["cand"][t], order[:k])
            where = np.nonzero(r["cand"][t] == plain[t])[0]
            assert r["match_idx"][t] == (where[0] if len(where) else -1)
        # the default (no separate matrix) reads the LM head instead: the two must differ visibly
        rd = o.ppd(p, ell, k, dbar, want_logits=True)
        zd = torch_forward(cfg.replace(n_layers=dbar), _Shallow(m, dbar, m.g["lm_head"]), seq)[len(p) - 1:]
        np.testing.assert_allclose(rd["early_logits"], zd, rtol=0, atol=1e-10)
        assert np.abs(zd - zt).max() > 0.1
        # teacher-forced early logits take the same classifier
        _, ze = oe.teacher_forced(seq, len(p) - 1, dbar=dbar)
        np.testing.assert_array_equal(ze, r["early_logits"])
    # handing over the LM head itself as the early classifier is the default
    osame = oracle.Oracle(m, early_head=m.g["lm_head"])
    np.testing.assert_array_equal(osame.ppd(p, ell, k, cfg.exit_layer, want_logits=True)["early_logits"],
                                  o.ppd(p, ell, k, cfg.exit_layer, want_logits=True)["early_logits"])


@pytest.mark.parametrize("family", ["opt", "llama"])
def test_early_head_close_to_lm_head_matches_and_adopts(family):
    """An early classifier near the LM head on a model whose late blocks add little: most rounds match, the
    matching sub-process is adopted (rounds that start mid-stack), and the output is still plain greedy's."""
    cfg = small_cfg(family, alpha=0.05)
    m = pi.make_model(cfg)
    E = pi.make_early_head(cfg, m, mix=0.3)
    o, oe = oracle.Oracle(m), oracle.Oracle(m, early_head=E)
    p = pi.make_prompt(cfg)
    plain, zp = o.plain_greedy(p, cfg.n_gen, want_logits=True)
    r = oe.ppd(p, cfg.n_gen, 3, cfg.exit_layer, want_logits=True)
    np.testing.assert_array_equal(r["tokens"], plain)
    np.testing.assert_array_equal(r["final_logits"], zp)
    hits = int((r["match_idx"] >= 0).sum())
    assert 0 < hits and r["stats"]["matches"] == hits
    assert r["stats"]["runs"] == 1 + int((r["match_idx"][:cfg.n_gen - 1] < 0).sum())
    rd = o.ppd(p, cfg.n_gen, 3, cfg.exit_layer, want_logits=True)
    assert np.abs(r["early_logits"] - rd["early_logits"]).max() > 1e-2
