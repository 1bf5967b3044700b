"""ctypes front-end of the CPU oracle (oracle/ppd_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  Nothing on the product path may import it, and
it imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libppd_oracle.so")
_lib = None

_LAYER_FIELDS = ("ln1_g", "ln1_b", "wq", "wk", "wv", "wo", "bq", "bk", "bv", "bo",
                 "ln2_g", "ln2_b", "w_in", "w_up", "w_out", "b_in", "b_out")


class OrcDims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "d_model", "n_heads", "head_dim", "d_ff", "vocab", "max_ctx",
                 "norm", "act", "pos", "has_bias", "wdtype")] + \
               [("norm_eps", ctypes.c_double), ("rope_theta", ctypes.c_double)]


class OrcWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("tok_emb", "pos_emb", "lnf_g", "lnf_b", "lm_head", "early_head")] + \
               [(n, ctypes.POINTER(ctypes.c_void_p)) for n in _LAYER_FIELDS]


class OrcStats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in
                ("rounds", "matches", "runs", "main_layer_rows", "branch_layer_rows")]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (CPU only; OpenMP across output rows and heads)."""
    src = os.path.join(_HERE, "ppd_oracle.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O3", "-mavx2", "-mfma", "-fPIC", "-shared", "-fopenmp", "-std=c11",
                               "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        lib.orc_create.argtypes = [ctypes.POINTER(OrcDims), ctypes.POINTER(OrcWeights), ci]
        lib.orc_create.restype = vp
        lib.orc_destroy.argtypes = [vp]
        lib.orc_destroy.restype = None
        lib.orc_plain_greedy.argtypes = [vp, vp, ci, ci, ci, vp, vp]
        lib.orc_plain_recompute.argtypes = [vp, vp, ci, ci, vp, vp]
        lib.orc_full_forward.argtypes = [vp, vp, ci, vp]
        lib.orc_ppd.argtypes = [vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, ctypes.POINTER(OrcStats), vp, vp]
        lib.orc_teacher_forced.argtypes = [vp, vp, ci, ci, ci, vp, vp]
        lib.orc_linear.argtypes = [vp, vp, vp, ci, ci, vp, vp]
        lib.orc_linear.restype = None
        lib.orc_norm.argtypes = [vp, vp, vp, vp, vp]
        lib.orc_norm.restype = None
        lib.orc_rope.argtypes = [vp, vp, ci]
        lib.orc_rope.restype = None
        lib.orc_act.argtypes = [ci, ctypes.c_double]
        lib.orc_act.restype = ctypes.c_double
        lib.orc_topk.argtypes = [vp, ci, ci, vp]
        lib.orc_topk.restype = None
        lib.orc_argmax.argtypes = [vp, ci]
        lib.orc_argmax.restype = ci
        lib.orc_set_selection.argtypes = [vp, ci, ci, ctypes.c_double, ctypes.c_uint64]
        lib.orc_set_selection.restype = None
        lib.orc_philox4x32_10.argtypes = [vp, vp, vp]
        lib.orc_philox4x32_10.restype = None
        lib.orc_uniform.argtypes = [ctypes.c_uint64, ctypes.c_int64]
        lib.orc_uniform.restype = ctypes.c_double
        lib.orc_sample.argtypes = [vp, ci, ci, ci, ctypes.c_double, ctypes.c_double]
        lib.orc_sample.restype = ci
        _lib = lib
    return _lib


GREEDY, TOP_K, TOP_P = 0, 1, 2


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


class Oracle:
    """The oracle bound to one synthetic model (a ``ppd_inputs.SynthModel``-like
    object with ``cfg``, ``g`` and ``layers``).  Keeps the model's arrays alive."""

    def __init__(self, model, ctx_cap: Optional[int] = None, early_head: Optional[np.ndarray] = None):
        lib = _load()
        cfg = model.cfg
        self.model, self.cfg = model, cfg
        self.ctx_cap = int(ctx_cap if ctx_cap is not None else cfg.max_ctx)
        d = OrcDims(cfg.n_layers, cfg.d_model, cfg.n_heads, cfg.head_dim, cfg.d_ff, cfg.vocab, cfg.max_ctx,
                    cfg.norm, cfg.act, cfg.pos, cfg.has_bias, cfg.wdtype, cfg.norm_eps, cfg.rope_theta)
        w = OrcWeights()
        g = model.g
        w.tok_emb, w.pos_emb = _ptr(g["tok_emb"]), _ptr(g.get("pos_emb"))
        w.lnf_g, w.lnf_b, w.lm_head = _ptr(g["lnf_g"]), _ptr(g.get("lnf_b")), _ptr(g["lm_head"])
        self._early = early_head
        w.early_head = _ptr(early_head)
        self._arrs = []
        for f in _LAYER_FIELDS:
            arr = (ctypes.c_void_p * cfg.n_layers)(*[_ptr(t) for t in model.layers[f]])
            self._arrs.append(arr)
            setattr(w, f, arr)
        self._d, self._w = d, w
        self._h = lib.orc_create(ctypes.byref(d), ctypes.byref(w), self.ctx_cap)
        if not self._h:
            raise MemoryError("orc_create failed")

    def close(self):
        if self._h:
            _load().orc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- decoding ---------------------------------------------------------
    def set_selection(self, mode=GREEDY, top_k=0, top_p=1.0, seed=0):
        """Rule for the final prediction of every decoding loop of this object (Appendix B):
        GREEDY, TOP_K sampling or TOP_P sampling with the counter-based uniform of (seed, position)."""
        _load().orc_set_selection(self._h, int(mode), int(top_k), float(top_p), int(seed))

    def plain_greedy(self, prompt, ell, want_logits=False, eos=-1):
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        toks = np.zeros(ell, dtype=np.int32)
        z = np.zeros((ell, self.cfg.vocab)) if want_logits else None
        n = _load().orc_plain_greedy(self._h, prompt.ctypes.data, len(prompt), ell, eos, toks.ctypes.data, _ptr(z))
        if n < 0:
            raise ValueError("orc_plain_greedy: bad arguments")
        return (toks[:n], z[:n]) if want_logits else toks[:n]

    def plain_recompute(self, prompt, ell, want_logits=False):
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        toks = np.zeros(ell, dtype=np.int32)
        z = np.zeros((ell, self.cfg.vocab)) if want_logits else None
        _load().orc_plain_recompute(self._h, prompt.ctypes.data, len(prompt), ell, toks.ctypes.data, _ptr(z))
        return (toks, z) if want_logits else toks

    def full_forward(self, tokens):
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        z = np.zeros((len(tokens), self.cfg.vocab))
        _load().orc_full_forward(self._h, tokens.ctypes.data, len(tokens), z.ctypes.data)
        return z

    def ppd(self, prompt, ell, k, dbar, want_logits=False, eos=-1):
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        toks = np.zeros(ell, dtype=np.int32)
        cand = np.zeros((ell, k), dtype=np.int32)
        midx = np.zeros(ell, dtype=np.int32)
        st = OrcStats()
        ze = np.zeros((ell, self.cfg.vocab)) if want_logits else None
        zf = np.zeros((ell, self.cfg.vocab)) if want_logits else None
        n = _load().orc_ppd(self._h, prompt.ctypes.data, len(prompt), ell, k, dbar, eos, toks.ctypes.data,
                            cand.ctypes.data, midx.ctypes.data, ctypes.byref(st), _ptr(ze), _ptr(zf))
        if n < 0:
            raise ValueError("orc_ppd: bad arguments")
        out = dict(tokens=toks[:n], cand=cand[:n], match_idx=midx[:n],
                   stats={f: int(getattr(st, f)) for f, _ in OrcStats._fields_})
        if want_logits:
            out["early_logits"], out["final_logits"] = ze[:n], zf[:n]
        return out

    def teacher_forced(self, tokens, first, dbar=0):
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        n = len(tokens)
        zf = np.zeros((n - first, self.cfg.vocab))
        ze = np.zeros((n - first, self.cfg.vocab)) if dbar > 0 else None
        rc = _load().orc_teacher_forced(self._h, tokens.ctypes.data, n, first, dbar, zf.ctypes.data, _ptr(ze))
        if rc < 0:
            raise ValueError("orc_teacher_forced: sequence longer than ctx_cap")
        return (zf, ze) if dbar > 0 else zf

    # -- primitives for the pin tests -----------------------------------------
    def linear(self, W, b, x):
        x = np.ascontiguousarray(x, dtype=np.float64)
        y = np.zeros(W.shape[0])
        _load().orc_linear(self._h, W.ctypes.data, _ptr(b), W.shape[0], W.shape[1], x.ctypes.data, y.ctypes.data)
        return y

    def norm(self, g, b, x):
        x = np.ascontiguousarray(x, dtype=np.float64)
        y = np.zeros_like(x)
        _load().orc_norm(self._h, g.ctypes.data, _ptr(b), x.ctypes.data, y.ctypes.data)
        return y

    def rope(self, v, pos):
        v = np.array(v, dtype=np.float64, copy=True)
        _load().orc_rope(self._h, v.ctypes.data, int(pos))
        return v


def act(kind: int, u: float) -> float:
    return float(_load().orc_act(kind, u))


def topk(z, k):
    z = np.ascontiguousarray(z, dtype=np.float64)
    ids = np.zeros(k, dtype=np.int32)
    _load().orc_topk(z.ctypes.data, len(z), k, ids.ctypes.data)
    return ids


def argmax(z):
    z = np.ascontiguousarray(z, dtype=np.float64)
    return int(_load().orc_argmax(z.ctypes.data, len(z)))


def philox4x32_10(ctr, key):
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    _load().orc_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


def uniform(seed: int, index: int) -> float:
    """u in [0, 1) of the token chosen at sequence position ``index``."""
    return float(_load().orc_uniform(int(seed), int(index)))


def sample(z, mode, top_k, top_p, u):
    """Token drawn from the truncated softmax of the logits z by inversion at u."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    return int(_load().orc_sample(z.ctypes.data, len(z), int(mode), int(top_k), float(top_p), float(u)))
