"""The stand-alone early prediction (`ppd_early_topk`) against the oracle's own pieces: final norm, classifier
matrix product, top-k by (logit descending, id ascending).  Shapes span several workgroups, a ragged last weight
row set, reduction lengths above and below the staged tile, both weight types and both norms."""
import numpy as np
import pytest
import torch

import oracle
import ppd_inputs as pi
from helpers import small_cfg
from paper_2307_05908_amd import binding

pytestmark = pytest.mark.gpu

CASES = {
    "tiny_fp32_ln": small_cfg("tiny"),
    "opt_bf16_ln": small_cfg("opt"),
    "llama_bf16_rms": small_cfg("llama"),
    # vocabulary not a multiple of anything, more rows than one wave pass, reduction length beyond one staged tile
    "wide_rms": small_cfg("llama", d_model=16384 + 512, n_heads=132, vocab=3001, n_layers=2, exit_layer=1, d_ff=64),
    "big_vocab_ln": small_cfg("opt", vocab=50272, d_model=64, n_heads=1, n_layers=2, exit_layer=1, d_ff=64),
}


def dev_tensor(a):
    if a is None:
        return None
    t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to("cuda:0")
    return t.view(torch.bfloat16) if a.dtype == np.uint16 else t


def oracle_logits(o, m, E, h):
    a = o.norm(m.g["lnf_g"], m.g.get("lnf_b"), h.astype(np.float64))
    return o.linear(E, None, a)


def check_against_oracle(ids, vals, z_gpu, zo, k, tol):
    if z_gpu is not None:
        assert np.abs(z_gpu - zo).max() <= tol
        order = np.lexsort((np.arange(len(z_gpu)), -z_gpu.astype(np.float64)))
        np.testing.assert_array_equal(ids, order[:k])           # exactly the top-k of the kernel's own logits
        np.testing.assert_array_equal(vals, z_gpu[ids])
    assert len(set(ids.tolist())) == k
    kth = np.sort(zo)[-k]
    assert (zo[ids] >= kth - tol).all()                          # and within tolerance of the oracle's
    assert np.abs(vals - zo[ids]).max() <= tol


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("k", [1, 3, 8])
def test_early_topk_matches_oracle(name, k):
    cfg = CASES[name]
    # only the final norm and the classifier are needed: a model of the shape without its layers
    m = pi.make_model(cfg.replace(n_layers=1, exit_layer=1, d_ff=8))
    E = pi.make_early_head(cfg)
    o = oracle.Oracle(m)
    rng = np.random.default_rng(7)
    h = (rng.standard_normal(cfg.d_model) * 1.5 + 0.2).astype(np.float32)
    zo = oracle_logits(o, m, E, h)
    tol = 1e-4 if cfg.wdtype == pi.WD_FP32 else 2e-2
    ids, vals, z = binding.ppd_early_topk(dev_tensor(h), dev_tensor(m.g["lnf_g"]), dev_tensor(m.g.get("lnf_b")),
                                          dev_tensor(E), k, cfg.norm, cfg.norm_eps, want_logits=True)
    check_against_oracle(ids.cpu().numpy(), vals.cpu().numpy(), z.cpu().numpy(), zo, k, tol)
    # without a logits buffer of the caller's the result is the same
    ids2, vals2, _ = binding.ppd_early_topk(dev_tensor(h), dev_tensor(m.g["lnf_g"]), dev_tensor(m.g.get("lnf_b")),
                                            dev_tensor(E), k, cfg.norm, cfg.norm_eps, want_logits=False)
    np.testing.assert_array_equal(ids2.cpu().numpy(), ids.cpu().numpy())
    np.testing.assert_array_equal(vals2.cpu().numpy().view(np.uint32), vals.cpu().numpy().view(np.uint32))


def test_early_topk_ties_go_to_the_lowest_id():
    """Equal classifier rows give equal logits: the ranking falls back on the id."""
    cfg = small_cfg("tiny", vocab=600)
    m = pi.make_model(cfg.replace(n_layers=1, exit_layer=1, d_ff=8))
    E = pi.make_early_head(cfg)
    E[1::2] = E[0::2]                       # ids 2j and 2j+1 tie exactly
    h = np.random.default_rng(3).standard_normal(cfg.d_model).astype(np.float32)
    ids, vals, z = binding.ppd_early_topk(dev_tensor(h), dev_tensor(m.g["lnf_g"]), dev_tensor(m.g.get("lnf_b")),
                                          dev_tensor(E), 6, cfg.norm, cfg.norm_eps, want_logits=True)
    ids, z = ids.cpu().numpy(), z.cpu().numpy()
    np.testing.assert_array_equal(z[0::2], z[1::2])
    np.testing.assert_array_equal(ids, np.lexsort((np.arange(cfg.vocab), -z.astype(np.float64)))[:6])
    assert (ids[0::2] % 2 == 0).all() and (ids[1::2] == ids[0::2] + 1).all()
