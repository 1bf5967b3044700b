"""GPU parity: the HIP library (through the C ABI) against the CPU oracle, element by
element, and PPD-on-GPU against plain-greedy-on-GPU bit for bit."""
import numpy as np
import pytest

import oracle
import ppd_inputs as pi
from gpu_common import TOL, gpu_generate, run_against_oracle
from helpers import small_cfg
from paper_2307_05908_amd import binding, tradeoff

pytestmark = pytest.mark.gpu

SMALL = {
    "tiny": small_cfg("tiny"),
    "opt": small_cfg("opt"),
    "llama": small_cfg("llama"),
    # several attention chunks (64 positions each) and a ragged last one
    "llama_long": small_cfg("llama", max_ctx=420, n_prompt=300, n_gen=24),
    "opt_long": small_cfg("opt", max_ctx=300, n_prompt=250, n_gen=16),
}
# prompts past 1024 rows: the prompt attention's two-tiles-per-wave instances, ragged last tiles
XLONG = {
    "llama_xlong": small_cfg("llama", max_ctx=1160, n_prompt=1102, n_gen=6),
    "opt_xlong": small_cfg("opt", max_ctx=1100, n_prompt=1038, n_gen=6),
}


@pytest.fixture(scope="module", params=list(SMALL))
def setup(request):
    cfg = SMALL[request.param]
    m = pi.make_model(cfg)
    dev = binding.upload_model(m)
    return cfg, m, dev, oracle.Oracle(m)


def test_plain_greedy_matches_oracle(setup):
    cfg, m, dev, o = setup
    prompt = pi.make_prompt(cfg)
    otoks, oz = o.plain_greedy(prompt, cfg.n_gen, want_logits=True)
    P = binding.PPD(cfg, dev)
    r = run_against_oracle(P, prompt, "plain", otoks, oz, tol=TOL[cfg.wdtype])
    print(cfg.name, "plain max|dlogit|", r["max_err"], "resyncs", r["resyncs"])


@pytest.mark.parametrize("k", [1, 3, 5, 8])
def test_ppd_matches_oracle(setup, k):
    cfg, m, dev, o = setup
    prompt = pi.make_prompt(cfg)
    d = cfg.n_layers
    for dbar in sorted({(d + 1) // 2, cfg.exit_layer, d - 1}):
        ro = o.ppd(prompt, cfg.n_gen, k, dbar, want_logits=True)
        P = binding.PPD(cfg, dev, k=k, exit_layer=dbar)
        r = run_against_oracle(P, prompt, "ppd", ro["tokens"], ro["final_logits"], ro["early_logits"], tol=TOL[cfg.wdtype])
        print(cfg.name, "k", k, "dbar", dbar, "max|dlogit|", r["max_err"], r["max_err_early"], "resyncs", r["resyncs"],
              "matches", r["matches"], "oracle matches", ro["stats"]["matches"])
        # (per round, run_against_oracle has checked the match index against the GPU's own candidates and the
        # candidates against the oracle's early logits; the totals agree whenever no candidate set differed)
        if r["resyncs"] == 0 and r["cand_sets_equal"]:
            assert r["matches"] == ro["stats"]["matches"]
        P.close()


@pytest.mark.parametrize("k", [1, 3, 5])
def test_ppd_gpu_is_plain_gpu_bit_exact(setup, k):
    """Sec. 1 / Sec. 3: PPD keeps the exact decoding result.  Tokens and final logits of every
    round equal plain greedy decoding on the same kernels; the counters obey the identities
    in the proof of Theorem 4.1."""
    cfg, m, dev, o = setup
    prompt = pi.make_prompt(cfg)
    d, ell = cfg.n_layers, cfg.n_gen
    P0 = binding.PPD(cfg, dev)
    ptoks, pz, _ = gpu_generate(P0, prompt, ell, "plain")
    P0.close()
    for dbar in sorted({(d + 1) // 2, cfg.exit_layer, d - 1}):
        P = binding.PPD(cfg, dev, k=k, exit_layer=dbar)
        toks, z, infos = gpu_generate(P, prompt, ell, "ppd")
        np.testing.assert_array_equal(toks, ptoks)
        np.testing.assert_array_equal(z, pz)
        st = P.ppd_get_stats()
        hit = np.array([i[0] for i in infos], dtype=bool)
        N = 1 + int((~hit[:ell - 1]).sum())
        assert st["runs"] == N and st["rounds"] == ell and st["matches"] == int(hit.sum())
        assert st["main_layer_rows"] == tradeoff.latency_of_runs(d, dbar, ell, N)
        assert st["main_layer_rows"] + st["branch_layer_rows"] == tradeoff.compute_of_runs(d, dbar, ell, k, N)
        P.close()


def test_graph_replay_equals_eager_launches(setup):
    """Rounds replayed from captured HIP graphs give the bits of eagerly issued launches, on every
    replay (the program's own copies and synchronisations run between replays)."""
    cfg, m, dev, o = setup
    prompt = pi.make_prompt(cfg)
    ell = min(cfg.n_gen, 16)
    res = []
    for graphs in (True, False):
        P = binding.PPD(cfg, dev, k=3)
        P.ppd_set_graphs(graphs)
        toks, z, infos = gpu_generate(P, prompt, ell, "ppd")
        ptoks, pz, _ = gpu_generate(P, prompt, ell, "plain")
        res.append((toks, z, infos, ptoks, pz))
        P.close()
    np.testing.assert_array_equal(res[0][0], res[1][0])
    np.testing.assert_array_equal(res[0][1], res[1][1])
    assert res[0][2] == res[1][2]
    np.testing.assert_array_equal(res[0][3], res[1][3])
    np.testing.assert_array_equal(res[0][4], res[1][4])


def test_mixing_plain_and_ppd_steps(setup):
    cfg, m, dev, o = setup
    prompt = pi.make_prompt(cfg)
    P0 = binding.PPD(cfg, dev)
    ptoks, _, _ = gpu_generate(P0, prompt, 12, "plain", want_logits=False)
    P = binding.PPD(cfg, dev)
    P.ppd_prefill(prompt)
    got = []
    for t in range(12):
        got.append(P.ppd_step()[0] if (t // 2) % 2 == 0 else P.plain_greedy_step())
    np.testing.assert_array_equal(got, ptoks)


def test_edge_cases():
    cfg = small_cfg("llama", max_ctx=40)
    m = pi.make_model(cfg)
    dev = binding.upload_model(m)
    o = oracle.Oracle(m)
    P = binding.PPD(cfg, dev, k=3)
    # step before prefill
    with pytest.raises(binding.PPDError) as ei:
        P.ppd_step()
    assert ei.value.code == -4
    # prompt of one token: nothing to prefill, x_0 is the prompt
    prompt = pi.make_prompt(cfg, 1)
    otoks, oz = o.plain_greedy(prompt, 6, want_logits=True)
    run_against_oracle(P, prompt, "ppd", otoks, oz, tol=2e-2)
    # bad token id, over-long prompt
    with pytest.raises(binding.PPDError) as ei:
        P.ppd_prefill([0, cfg.vocab])
    assert ei.value.code == -1
    with pytest.raises(binding.PPDError) as ei:
        P.ppd_prefill([1] * 41)
    assert ei.value.code == -3
    # run into the end of the context window: PPD needs position t+1 for its candidates
    prompt = pi.make_prompt(cfg, 30)
    P.ppd_prefill(prompt)
    n = 0
    with pytest.raises(binding.PPDError) as ei:
        for _ in range(20):
            P.ppd_step()
            n += 1
    assert ei.value.code == -3 and n == 10        # positions 29..38 emit, 39 has no room for t+1
    tok = P.plain_greedy_step()                    # the plain step still fits position 39
    assert tok is not None
    with pytest.raises(binding.PPDError):
        P.plain_greedy_step()
    # EOS stops both kinds of step
    otoks = o.plain_greedy(prompt, 8)
    eos = int(otoks[3])
    first = int(np.nonzero(otoks == eos)[0][0])
    Pe = binding.PPD(cfg, dev, k=3, eos_id=eos)
    Pe.ppd_prefill(prompt)
    got = []
    while True:
        tok, _ = Pe.ppd_step()
        if tok is None:
            break
        got.append(tok)
    np.testing.assert_array_equal(got, otoks[:first + 1])
    assert Pe.plain_greedy_step() is None


@pytest.mark.gpu
def test_stream_read_probe_reports_a_plausible_rate():
    """The library's measurement aid: 256 MiB read, between 1 and 8 TB/s on an MI355X."""
    import torch
    buf = torch.zeros(1 << 28, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    rate = binding.ppd_stream_read_probe(buf, iters=4)
    assert 1000.0 < rate < 8000.0, rate


@pytest.mark.gpu
def test_ffn_in_burst_timing_invalidates_the_sequence():
    cfg = small_cfg("llama")
    dev = binding.upload_model(pi.make_model(cfg))
    P = binding.PPD(cfg, dev, k=3)
    with pytest.raises(binding.PPDError) as ei:     # needs a prefilled context
        P.ppd_time_ffn_in(4)
    assert ei.value.code == -4
    prompt = pi.make_prompt(cfg)
    P.ppd_prefill(prompt)
    ref = [P.ppd_step()[0] for _ in range(4)]
    P.ppd_prefill(prompt)
    ms = P.ppd_time_ffn_in(8)
    assert 0.0 < ms < 1.0
    P.ppd_prefill(prompt)
    ms2 = P.ppd_time_ffn_in(8, groups=2)             # the two-group launch of a pipelined step
    assert 0.0 < ms2 < 1.0
    with pytest.raises(binding.PPDError) as ei:     # the activations were overwritten
        P.ppd_step()
    assert ei.value.code == -4
    P.ppd_prefill(prompt)                            # and a new prefill restores everything
    assert [P.ppd_step()[0] for _ in range(4)] == ref
    P.close()


@pytest.mark.gpu
@pytest.mark.parametrize("family", ["llama", "opt"])
def test_staging_in_passes_is_bit_identical(family, monkeypatch):
    """Rows too long for LDS are staged in several passes with the accumulators parked in between; forced on
    here (PPD_MGPASSES), every token and logit equals the single-pass run bit for bit.  The feed-forward width
    is large enough (2056: nine 32-column blocks per wave, the last one ragged) for every forced pass to carry
    part of the reduction."""
    cfg = small_cfg(family, d_ff=2056)
    dev = binding.upload_model(pi.make_model(cfg))
    prompt = pi.make_prompt(cfg)

    def run():
        P = binding.PPD(cfg, dev, k=5)
        P.ppd_prefill(prompt)
        toks, zs = [], []
        for _ in range(cfg.n_gen):
            toks.append(P.ppd_step()[0])
            zs.append(P.ppd_get_logits().copy())
        P.close()
        return toks, np.stack(zs)

    ref_t, ref_z = run()
    for passes in (2, 3):
        monkeypatch.setenv("PPD_MGPASSES", str(passes))
        t, z = run()
        assert t == ref_t
        np.testing.assert_array_equal(z.view(np.uint32), ref_z.view(np.uint32))


@pytest.mark.gpu
@pytest.mark.parametrize("family", ["llama", "opt", "llama_long"])
@pytest.mark.parametrize("k", [1, 3, 5])
def test_speculative_early_prediction_changes_nothing_but_the_traffic(family, k, monkeypatch):
    """With the exit layer at d/2 the final head also runs on the candidate rows, and after a match the
    matching row's top-k are the next round's candidates (no early head pass in that round).  Tokens, final
    and early logits, candidates and match indices equal the rounds that run their own early head, bit for
    bit; only the LM-head traffic drops, by one matrix per matching round."""
    cfg = SMALL[family].replace(alpha=0.05)          # late layers damped: most early predictions hold
    assert 2 * cfg.exit_layer == cfg.n_layers
    dev = binding.upload_model(pi.make_model(cfg))
    prompt = pi.make_prompt(cfg)

    def run():
        P = binding.PPD(cfg, dev, k=k)
        P.ppd_prefill(prompt)
        toks, zs, es, infos = [], [], [], []
        for t in range(cfg.n_gen):
            if t == cfg.n_gen // 2:                  # a plain step in between: the next round starts from layer 1 again
                toks.append(P.plain_greedy_step())
                continue
            tok, info = P.ppd_step(want_info=True)
            toks.append(tok)
            infos.append((info.matched, info.match_idx, tuple(info.cand[:k])))
            zs.append(P.ppd_get_logits().copy())
            es.append(P.ppd_get_early_logits().copy())
        st = P.ppd_get_stats()
        P.close()
        return toks, np.stack(zs), np.stack(es), infos, st

    monkeypatch.setenv("PPD_SPEC", "1")
    t1, z1, e1, i1, st1 = run()
    monkeypatch.setenv("PPD_SPEC", "2")
    t0, z0, e0, i0, st0 = run()
    assert t1 == t0 and i1 == i0
    np.testing.assert_array_equal(z1.view(np.uint32), z0.view(np.uint32))
    np.testing.assert_array_equal(e1.view(np.uint32), e0.view(np.uint32))
    assert st1["matches"] == st0["matches"] and st1["main_layer_rows"] == st0["main_layer_rows"]
    if cfg.wdtype == pi.WD_BF16:
        # rounds that follow a match (not the one after the plain step, not past the end) skipped their early head
        hits = [m for m, _, _ in i1]
        follow = sum(1 for j in range(1, len(hits)) if hits[j - 1] and j != cfg.n_gen // 2)
        head_bytes = cfg.vocab * cfg.d_model * cfg.wbytes
        assert st0["weight_bytes"] - st1["weight_bytes"] == follow * head_bytes
        assert follow > 0


@pytest.mark.gpu
@pytest.mark.parametrize("name", list(SMALL))
def test_prompt_in_chunks_is_token_by_token_bit_exact(name, monkeypatch):
    """ppd_prefill feeds the prompt a chunk of positions at a time (one pass over the weights per chunk, rows of a
    chunk attend causally to each other); every row's arithmetic is that of a one-token pass, so the cache and
    everything decoded from it equal the token-by-token prefill (PPD_PREFILL_CHUNK=1) bit for bit.  Prompt
    lengths leave ragged last chunks and cross the 64-position attention chunks; the full 16-row chunk as well."""
    cfg = SMALL[name]
    dev = binding.upload_model(pi.make_model(cfg))

    def run(n_prompt):
        prompt = pi.make_prompt(cfg, n_prompt)
        P = binding.PPD(cfg, dev, k=3)
        toks, z, _ = gpu_generate(P, prompt, 6, "ppd")
        ptoks, pz, _ = gpu_generate(P, prompt, 3, "plain")
        P.close()
        return toks, z, ptoks, pz

    lengths = sorted({2, 3, 9, 10, cfg.n_prompt, min(cfg.max_ctx - 8, 70), min(cfg.max_ctx - 8, 130)})
    monkeypatch.setenv("PPD_PREFILL_TILED", "2")     # (longer prompts of bf16 models would take the compute-bound pass)
    got = {n: run(n) for n in lengths}
    monkeypatch.setenv("PPD_PREFILL_CHUNK", "16")
    got16 = {n: run(n) for n in lengths}
    monkeypatch.setenv("PPD_PREFILL_CHUNK", "1")
    for n in lengths:
        ref = run(n)
        for a, b in list(zip(got[n], ref)) + list(zip(got16[n], ref)):
            np.testing.assert_array_equal(np.asarray(a).view(np.uint32) if np.asarray(a).dtype == np.float32 else a,
                                          np.asarray(b).view(np.uint32) if np.asarray(b).dtype == np.float32 else b)


@pytest.mark.gpu
@pytest.mark.parametrize("family", ["tiny", "opt", "llama"])
@pytest.mark.parametrize("near", [False, True])
def test_separate_early_head_matches_oracle_and_keeps_the_output(family, near):
    """Sec. 4.3: a classifier of its own for the exit layer (`early_head`).  The early logits follow the oracle
    run with the same matrix, the candidates are their top-k, tokens and final logits stay those of plain greedy
    decoding on the GPU bit for bit.  near = False: an unrelated random matrix (no round matches); near = True:
    the LM head plus noise on a model with damped late blocks, so that most rounds match and the rounds after a
    match start mid-stack and run their own early head (no speculative prediction with a separate classifier).
    Exit layers d/2 and d-1."""
    cfg = small_cfg(family, alpha=0.05) if near else small_cfg(family)
    m = pi.make_model(cfg)
    E = pi.make_early_head(cfg, m, mix=0.3) if near else pi.make_early_head(cfg)
    dev = binding.upload_model(m)
    import torch
    Et = torch.from_numpy(E.view(np.int16) if E.dtype == np.uint16 else E).to("cuda:0")
    if E.dtype == np.uint16:
        Et = Et.view(torch.bfloat16)
    o = oracle.Oracle(m, early_head=E)
    prompt = pi.make_prompt(cfg)
    d, ell, k = cfg.n_layers, cfg.n_gen, 3
    P0 = binding.PPD(cfg, dev)
    ptoks, pz, _ = gpu_generate(P0, prompt, ell, "plain")
    P0.close()
    for dbar in sorted({(d + 1) // 2, d - 1}):
        ro = o.ppd(prompt, ell, k, dbar, want_logits=True)
        P = binding.PPD(cfg, dev, k=k, exit_layer=dbar, early_head=Et)
        r = run_against_oracle(P, prompt, "ppd", ro["tokens"], ro["final_logits"], ro["early_logits"], tol=TOL[cfg.wdtype])
        print(cfg.name, "early_head near", near, "dbar", dbar, "max|dlogit|", r["max_err"], r["max_err_early"],
              "matches", r["matches"], "oracle", ro["stats"]["matches"], flush=True)
        if near:
            assert r["matches"] > ell // 4
        elif r["resyncs"] == 0 and r["cand_sets_equal"]:
            assert r["matches"] == ro["stats"]["matches"]
        toks, z, infos = gpu_generate(P, prompt, ell, "ppd")
        np.testing.assert_array_equal(toks, ptoks)
        np.testing.assert_array_equal(z.view(np.uint32), pz.view(np.uint32))
        # the default context (LM head as the early classifier) predicts something else
        Pd = binding.PPD(cfg, dev, k=k, exit_layer=dbar)
        Pd.ppd_prefill(prompt); P.ppd_prefill(prompt)
        Pd.ppd_step(); P.ppd_step()
        assert np.abs(Pd.ppd_get_early_logits() - P.ppd_get_early_logits()).max() > 1e-2
        Pd.close()
        P.close()


@pytest.mark.gpu
@pytest.mark.parametrize("name", ["llama_xlong", "opt_xlong"])
def test_compute_bound_prompt_pass_beyond_1024_rows(name, monkeypatch):
    """Prompts of 1024 rows and more take the attention instance with two query tiles per wave (head dimensions 128
    and 64 here), with a ragged last tile, a ragged last 32-row step and a last workgroup that is partly empty.
    Checked as for shorter prompts: next-token logits against the oracle, and against the row-chunk path."""
    cfg = XLONG[name]
    m = pi.make_model(cfg)
    dev = binding.upload_model(m)
    o = oracle.Oracle(m)
    for n_prompt in (1025, cfg.n_prompt):
        prompt = pi.make_prompt(cfg, n_prompt)
        ro = o.ppd(prompt, 4, 3, cfg.exit_layer, want_logits=True)
        monkeypatch.setenv("PPD_PREFILL_TILED", "1")
        P = binding.PPD(cfg, dev, k=3)
        r = run_against_oracle(P, prompt, "ppd", ro["tokens"], ro["final_logits"], ro["early_logits"], tol=TOL[cfg.wdtype])
        toks, z, _ = gpu_generate(P, prompt, 4, "ppd")
        P.close()
        monkeypatch.setenv("PPD_PREFILL_TILED", "2")
        Q = binding.PPD(cfg, dev, k=3)
        qtoks, qz, _ = gpu_generate(Q, prompt, 4, "ppd")
        Q.close()
        print(name, n_prompt, "worst |dlogit| vs oracle", r["max_err"], "vs row chunks", float(np.abs(z - qz).max()), flush=True)
        assert np.abs(z - qz).max() <= 1e-4


@pytest.mark.gpu
@pytest.mark.parametrize("name", ["llama_long", "opt_long"])
def test_compute_bound_prompt_pass_against_oracle_and_row_chunks(name, monkeypatch):
    """Prompts of bf16 models from 32 rows on go through tiled MFMA GEMMs and causal attention over the cache, all
    rows at once.  Other tiles and summation trees than the decode kernels: the cache is close to, not identical
    with, the row-chunk path's.  Checked: the logits of the next tokens against the oracle (teacher-forced, tolerance
    2e-2 and the tripwire) for prompt lengths with ragged 16- and 64-row tiles, against the row-chunk path (a few
    1e-5 apart at most), and PPD == plain greedy bit for bit from either cache."""
    cfg = SMALL[name]
    m = pi.make_model(cfg)
    dev = binding.upload_model(m)
    o = oracle.Oracle(m)
    worst = 0.0
    for n_prompt in (33, 64, 65, 81, 128, 129, cfg.n_prompt):
        prompt = pi.make_prompt(cfg, n_prompt)
        ro = o.ppd(prompt, 6, 3, cfg.exit_layer, want_logits=True)
        monkeypatch.setenv("PPD_PREFILL_TILED", "1")
        P = binding.PPD(cfg, dev, k=3)
        r = run_against_oracle(P, prompt, "ppd", ro["tokens"], ro["final_logits"], ro["early_logits"], tol=TOL[cfg.wdtype])
        toks, z, _ = gpu_generate(P, prompt, 6, "ppd")
        ptoks, pz, _ = gpu_generate(P, prompt, 6, "plain")
        np.testing.assert_array_equal(toks, ptoks)
        np.testing.assert_array_equal(z.view(np.uint32), pz.view(np.uint32))
        P.close()
        monkeypatch.setenv("PPD_PREFILL_TILED", "2")
        Q = binding.PPD(cfg, dev, k=3)
        qtoks, qz, _ = gpu_generate(Q, prompt, 6, "ppd")
        Q.close()
        worst = max(worst, float(np.abs(z - qz).max()), r["max_err"])
        assert np.abs(z - qz).max() <= 1e-4
    print(name, "compute-bound prompt pass: worst |dlogit| vs oracle / row chunks", worst, flush=True)
