"""The C-ABI library without a GPU: it loads, exports what include/*.h declare,
and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2307_05908_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ppd_[a-z_]+|plain_greedy_step)\s*\(", text)))


def test_header_symbols_are_exported():
    lib = binding.load_library()
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_strerror():
    lib = binding.load_library()
    assert lib.ppd_strerror(0) == b"ok"
    assert b"context" in lib.ppd_strerror(-3)


def _dims(**kw):
    base = dict(n_layers=4, d_model=256, n_heads=4, head_dim=64, d_ff=1024, vocab=1024, max_ctx=128,
                norm=0, act=0, pos=0, has_bias=1, wdtype=0, norm_eps=1e-5, rope_theta=1e4, eos_id=-1)
    base.update(kw)
    return binding.ModelDims(**base)


@pytest.mark.parametrize("kw,k,e", [
    (dict(d_model=250), 3, 2),          # d_model not a multiple of 8
    (dict(head_dim=32, n_heads=8), 3, 2),
    (dict(n_heads=3), 3, 2),            # heads * head_dim != d_model
    (dict(norm=2), 3, 2),
    (dict(), 0, 2), (dict(), 9, 2),     # k outside [1, 8]
    (dict(), 3, 1),                     # exit layer below d/2 (Theorem 4.1 needs dbar >= d/2)
    (dict(), 3, 4),                     # exit layer == d
])
def test_create_rejects_bad_arguments(kw, k, e):
    lib = binding.load_library()
    d = _dims(**kw)
    w = binding.Weights()
    h = ctypes.c_void_p()
    assert lib.ppd_create(ctypes.byref(d), ctypes.byref(w), k, e, None, ctypes.byref(h)) == -1
    assert not h.value


def test_create_rejects_a_matrix_beyond_32_bit_offsets():
    """The kernels address one weight matrix with 32-bit byte offsets: a model whose LM head (or fused projection)
    reaches 4 GiB is refused with PPD_ELIMIT before anything is allocated or read."""
    lib = binding.load_library()
    h = ctypes.c_void_p()
    w = binding.Weights()
    big_head = _dims(d_model=8192, n_heads=64, head_dim=128, d_ff=8192, vocab=200000)      # 200000 x 8192 x 4 B = 6.5 GB
    assert lib.ppd_create(ctypes.byref(big_head), ctypes.byref(w), 3, 2, None, ctypes.byref(h)) == -6
    big_ffn = _dims(d_model=16384, n_heads=128, head_dim=128, d_ff=65536, act=2, vocab=1024)   # gate|up: 2 x 65536 x 16384 x 4 B
    assert lib.ppd_create(ctypes.byref(big_ffn), ctypes.byref(w), 3, 2, None, ctypes.byref(h)) == -6
    assert not h.value


def test_null_arguments():
    lib = binding.load_library()
    assert lib.ppd_create(None, None, 3, 2, None, None) == -1
    assert lib.ppd_reset(None) == -1
    assert lib.ppd_step(None, None, 1, None) == -1
    assert lib.plain_greedy_step(None, None) == -1
    out = ctypes.c_double(0.0)
    assert lib.ppd_time_ffn_in(None, 4, 1, ctypes.byref(out)) == -1
    assert lib.ppd_set_sampling(None, 1, 3, 1.0, 0) == -1
    assert lib.ppd_stream_read_probe(None, 1 << 20, 1, ctypes.byref(out)) == -1      # no buffer
    assert lib.ppd_stream_read_probe(ctypes.c_void_p(16), 24, 1, ctypes.byref(out)) == -1   # not a multiple of 16
    assert lib.ppd_stream_read_probe(ctypes.c_void_p(16), 1 << 20, 0, ctypes.byref(out)) == -1
    # weights table with missing tensors
    d = _dims()
    w = binding.Weights()
    h = ctypes.c_void_p()
    assert lib.ppd_create(ctypes.byref(d), ctypes.byref(w), 3, 2, None, ctypes.byref(h)) == -1


def test_early_topk_rejects_bad_arguments():
    lib = binding.load_library()
    p = ctypes.c_void_p(256)      # never dereferenced: every case fails the argument checks
    ok = dict(d_model=256, vocab=1000, norm=1, eps=1e-5, wdtype=1, k=3)

    def call(**kw):
        a = dict(ok, **kw)
        return lib.ppd_early_topk(a["d_model"], a["vocab"], a["norm"], a["eps"], a["wdtype"], a.get("g", p), None,
                                  a.get("head", p), a.get("h", p), a["k"], a.get("ids", p), None, None, None)

    assert call(d_model=250) == -1 and call(vocab=0) == -1 and call(norm=2) == -1 and call(wdtype=3) == -1
    assert call(k=0) == -1 and call(k=9) == -1 and call(vocab=2, k=3) == -1
    assert call(norm=0) == -1                      # LayerNorm without its bias
    assert call(g=None) == -1 and call(head=None) == -1 and call(h=None) == -1 and call(ids=None) == -1
    assert call(h=ctypes.c_void_p(260)) == -1      # misaligned row
