"""`ppd_early_topk_noalloc` (fixed scratch array inside the library, no allocation, asynchronous) against
`ppd_early_topk` through the C ABI: same ids bit for bit, same logits bit for bit, on two calls in a row, the
second with a smaller input (the array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

import ppd_inputs as pi
from helpers import small_cfg
from paper_2307_05908_amd import binding

pytestmark = pytest.mark.gpu


def dev_tensor(a):
    if a is None:
        return None
    t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to("cuda:0")
    return t.view(torch.bfloat16) if a.dtype == np.uint16 else t


def case(cfg, seed):
    m = pi.make_model(cfg.replace(n_layers=1, exit_layer=1, d_ff=8))
    E = pi.make_early_head(cfg)
    h = (np.random.default_rng(seed).standard_normal(cfg.d_model) * 1.5 + 0.2).astype(np.float32)
    return dev_tensor(h), dev_tensor(m.g["lnf_g"]), dev_tensor(m.g.get("lnf_b")), dev_tensor(E), cfg.norm, cfg.norm_eps


@pytest.mark.parametrize("family", ["llama", "opt", "tiny"])
def test_noalloc_equals_allocating_entry_point_twice_in_a_row(family):
    big = small_cfg(family, vocab=40000 if family != "tiny" else 3000)
    small = small_cfg(family, vocab=777, d_model=128, n_heads=2 if family != "llama" else 1)
    for cfg, k, want_logits in ((big, 8, False), (small, 3, False), (big, 5, True), (small, 2, True)):
        h, g, b, E, norm, eps = case(cfg, 11)
        ref = binding.ppd_early_topk(h, g, b, E, k, norm, eps, want_logits=True)
        got = binding.ppd_early_topk_noalloc(h, g, b, E, k, norm, eps, want_logits=want_logits)
        torch.cuda.synchronize()       # the call only queues work: its outputs are complete after the stream's work
        np.testing.assert_array_equal(got[0].cpu().numpy(), ref[0].cpu().numpy())
        np.testing.assert_array_equal(got[1].cpu().numpy().view(np.uint32), ref[1].cpu().numpy().view(np.uint32))
        if want_logits:
            np.testing.assert_array_equal(got[2].cpu().numpy().view(np.uint32), ref[2].cpu().numpy().view(np.uint32))


def test_noalloc_rejects_sizes_beyond_its_array():
    lib = binding.load_library()
    cfg = small_cfg("llama", vocab=65536 + 16, d_model=64, n_heads=1)
    h, g, b, E, norm, eps = case(cfg, 5)
    with pytest.raises(binding.PPDError) as ei:
        binding.ppd_early_topk_noalloc(h, g, b, E, 3, norm, eps)
    assert ei.value.code == -6 and b"maximum" in lib.ppd_strerror(-6)
    ids, vals, _ = binding.ppd_early_topk(h, g, b, E, 3, norm, eps)      # the allocating entry point takes it
    assert len(set(ids.cpu().tolist())) == 3
    # the largest size it takes
    cfg = small_cfg("llama", vocab=65536, d_model=64, n_heads=1)
    h, g, b, E, norm, eps = case(cfg, 6)
    ref = binding.ppd_early_topk(h, g, b, E, 8, norm, eps, want_logits=True)
    got = binding.ppd_early_topk_noalloc(h, g, b, E, 8, norm, eps)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got[0].cpu().numpy(), ref[0].cpu().numpy())
    np.testing.assert_array_equal(got[1].cpu().numpy().view(np.uint32), ref[1].cpu().numpy().view(np.uint32))
