"""ctypes binding of libppd (include/ppd.h, include/ppd_measure.h): argument marshalling only.

Every step of the decode path runs in the HIP kernels behind the C ABI; this
module turns torch device tensors into the pointer tables the library takes
and mirrors its entry points under the same names.  There is no CPU fallback:
if the library cannot be loaded, importing the symbols raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional

import numpy as np

from . import build as _build

PPD_MAX_K = 8
KERNEL_CLASSES = ("embed", "gemm_qkv", "attn", "attn_merge", "gemm_o", "gemm_ffn_in", "gemm_ffn_out",
                  "head", "select", "commit", "phase")
_LAYER_FIELDS = ("ln1_g", "ln1_b", "wq", "wk", "wv", "wo", "bq", "bk", "bv", "bo",
                 "ln2_g", "ln2_b", "w_in", "w_up", "w_out", "b_in", "b_out")
# order of the per-layer members in ppd_weights
_W_LAYER_ORDER = ("ln1_g", "ln1_b", "wq", "wk", "wv", "wo", "bq", "bk", "bv", "bo",
                  "ln2_g", "ln2_b", "w_in", "w_up", "w_out", "b_in", "b_out")


class ModelDims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "d_model", "n_heads", "head_dim", "d_ff", "vocab", "max_ctx",
                 "norm", "act", "pos", "has_bias", "wdtype")] + \
               [("norm_eps", ctypes.c_float), ("rope_theta", ctypes.c_float), ("eos_id", ctypes.c_int32)]


class Weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("tok_emb", "pos_emb", "lnf_g", "lnf_b", "lm_head", "early_head")] + \
               [(n, ctypes.POINTER(ctypes.c_void_p)) for n in _W_LAYER_ORDER]


class StepInfo(ctypes.Structure):
    _fields_ = [("token", ctypes.c_int32), ("matched", ctypes.c_int32), ("match_idx", ctypes.c_int32),
                ("cand", ctypes.c_int32 * PPD_MAX_K)]


class Stats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint64) for n in
                ("rounds", "matches", "runs", "main_layer_rows", "branch_layer_rows", "plain_steps",
                 "weight_bytes", "kv_bytes")]


EXPORTS = ("ppd_create", "ppd_reset", "ppd_prefill", "ppd_step", "plain_greedy_step", "ppd_get_logits",
           "ppd_get_early_logits", "ppd_get_stats", "ppd_set_profiling", "ppd_set_graphs", "ppd_set_sampling", "ppd_get_kernel_time",
           "ppd_time_ffn_in", "ppd_stream_read_probe", "ppd_early_topk", "ppd_early_topk_noalloc", "ppd_destroy",
           "ppd_strerror", "ppd_last_hip_error")

_lib = None


def load_library() -> ctypes.CDLL:
    """Load libppd.so (built in-tree).  Raises if it is missing and cannot be built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB_PATH):
        _build.build(True)
    # torch ships its own HIP runtime (same soname).  Import it first so that libppd binds to the
    # runtime that owns the caller's tensors and streams; loaded the other way round the process
    # would hold two HIP runtimes and device pointers of one would be unknown to the other.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_build.LIB_PATH)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    lib.ppd_create.argtypes = [ctypes.POINTER(ModelDims), ctypes.POINTER(Weights), ci, ci, vp, ctypes.POINTER(vp)]
    lib.ppd_reset.argtypes = [vp]
    lib.ppd_prefill.argtypes = [vp, vp, ci]
    lib.ppd_step.argtypes = [vp, vp, ci, ctypes.POINTER(StepInfo)]
    lib.plain_greedy_step.argtypes = [vp, vp]
    lib.ppd_get_logits.argtypes = [vp, vp]
    lib.ppd_get_early_logits.argtypes = [vp, vp]
    lib.ppd_get_stats.argtypes = [vp, ctypes.POINTER(Stats)]
    lib.ppd_set_profiling.argtypes = [vp, ci]
    lib.ppd_set_graphs.argtypes = [vp, ci]
    lib.ppd_set_sampling.argtypes = [vp, ci, ci, ctypes.c_double, ctypes.c_uint64]
    lib.ppd_get_kernel_time.argtypes = [vp, ci, ci, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_uint64)]
    lib.ppd_time_ffn_in.argtypes = [vp, ci, ci, ctypes.POINTER(ctypes.c_double)]
    lib.ppd_stream_read_probe.argtypes = [vp, ctypes.c_uint64, ci, ctypes.POINTER(ctypes.c_double)]
    lib.ppd_early_topk.argtypes = [ci, ci, ci, ctypes.c_float, ci, vp, vp, vp, vp, ci, vp, vp, vp, vp]
    lib.ppd_early_topk_noalloc.argtypes = lib.ppd_early_topk.argtypes
    lib.ppd_destroy.argtypes = [vp]
    lib.ppd_destroy.restype = None
    lib.ppd_strerror.argtypes = [ci]
    lib.ppd_strerror.restype = ctypes.c_char_p
    lib.ppd_last_hip_error.argtypes = [vp]
    _lib = lib
    return lib


class PPDError(RuntimeError):
    def __init__(self, code: int, what: str, hip: int = 0):
        msg = load_library().ppd_strerror(code).decode()
        super().__init__(f"{what}: {msg} (code {code}" + (f", hipError {hip})" if hip else ")"))
        self.code = code


def upload_model(model, device="cuda:0") -> Dict[str, object]:
    """Copy a host model (``cfg``, ``g``, ``layers`` of numpy arrays; bf16 as uint16 bits) to the GPU.
    Returns {name: tensor or list of tensors}; torch is used for device memory only."""
    import torch

    def up(a):
        if a is None:
            return None
        t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a)
        t = t.to(device)
        return t.view(torch.bfloat16) if a.dtype == np.uint16 else t

    dev = {k: up(v) for k, v in model.g.items()}
    for f in _LAYER_FIELDS:
        dev[f] = [up(a) for a in model.layers[f]]
    return dev


def ppd_stream_read_probe(dev_tensor, iters: int = 5) -> float:
    """GB/s of a plain streaming read of a device tensor (measurement aid of the library)."""
    nbytes = dev_tensor.numel() * dev_tensor.element_size()
    out = ctypes.c_double(0.0)
    rc = load_library().ppd_stream_read_probe(dev_tensor.data_ptr(), nbytes, iters, ctypes.byref(out))
    if rc != 0:
        raise PPDError(rc, "ppd_stream_read_probe", load_library().ppd_last_hip_error(None))
    return float(out.value)


def _early_topk_call(fn_name, h, norm_g, norm_b, head, k, norm, norm_eps, want_logits, stream):
    import torch
    lib = load_library()
    vocab, d_model = head.shape
    wdtype = 0 if head.dtype == torch.float32 else 1
    ids = torch.empty(k, dtype=torch.int32, device=h.device)
    vals = torch.empty(k, dtype=torch.float32, device=h.device)
    logits = torch.empty(vocab, dtype=torch.float32, device=h.device) if want_logits else None
    st = stream if stream is not None else torch.cuda.current_stream()
    rc = getattr(lib, fn_name)(d_model, vocab, int(norm), float(norm_eps), wdtype, norm_g.data_ptr(),
                               None if norm_b is None else norm_b.data_ptr(), head.data_ptr(), h.data_ptr(), int(k),
                               ids.data_ptr(), vals.data_ptr(), None if logits is None else logits.data_ptr(),
                               ctypes.c_void_p(st.cuda_stream))
    if rc != 0:
        raise PPDError(rc, fn_name, lib.ppd_last_hip_error(None))
    return ids, vals, logits


def ppd_early_topk(h, norm_g, norm_b, head, k, norm, norm_eps=1e-5, want_logits=False, stream=None):
    """Stand-alone early prediction on device tensors: (ids int32[k], logits of those float[k], all logits or None).
    h: float32 [d_model]; norm_g / norm_b / head: float32 or bfloat16 tensors of the model's weight type."""
    return _early_topk_call("ppd_early_topk", h, norm_g, norm_b, head, k, norm, norm_eps, want_logits, stream)


def ppd_early_topk_noalloc(h, norm_g, norm_b, head, k, norm, norm_eps=1e-5, want_logits=False, stream=None):
    """The same through the entry point that allocates nothing (fixed scratch array in the library; asynchronous:
    the outputs are complete once the stream's work has run).  The output tensors are the caller's, made here."""
    return _early_topk_call("ppd_early_topk_noalloc", h, norm_g, norm_b, head, k, norm, norm_eps, want_logits, stream)


class PPD:
    """One decoding context.  ``dev`` is what ``upload_model`` returned (kept alive here)."""

    def __init__(self, cfg, dev: Dict[str, object], k: Optional[int] = None, exit_layer: Optional[int] = None,
                 eos_id: int = -1, early_head=None, stream=None):
        import torch
        lib = load_library()
        self.cfg, self.dev = cfg, dev
        self.k = cfg.k if k is None else k
        self.exit_layer = cfg.exit_layer if exit_layer is None else exit_layer
        d = ModelDims(cfg.n_layers, cfg.d_model, cfg.n_heads, cfg.head_dim, cfg.d_ff, cfg.vocab, cfg.max_ctx,
                      cfg.norm, cfg.act, cfg.pos, cfg.has_bias, cfg.wdtype, cfg.norm_eps, cfg.rope_theta, eos_id)
        w = Weights()

        def ptr(t):
            return None if t is None else t.data_ptr()

        for n in ("tok_emb", "pos_emb", "lnf_g", "lnf_b", "lm_head"):
            setattr(w, n, ptr(dev.get(n)))
        self._early = early_head
        w.early_head = ptr(early_head)
        self._tabs = []
        for f in _W_LAYER_ORDER:
            tab = (ctypes.c_void_p * cfg.n_layers)(*[ptr(t) for t in dev[f]])
            self._tabs.append(tab)
            setattr(w, f, tab)
        self._stream = stream if stream is not None else torch.cuda.current_stream()
        h = ctypes.c_void_p()
        rc = lib.ppd_create(ctypes.byref(d), ctypes.byref(w), self.k, self.exit_layer,
                            ctypes.c_void_p(self._stream.cuda_stream), ctypes.byref(h))
        if rc != 0:
            raise PPDError(rc, "ppd_create", lib.ppd_last_hip_error(None))
        self._h = h
        self._tok = np.zeros(4, dtype=np.int32)
        self._logits = np.zeros(cfg.vocab, dtype=np.float32)
        # looked up once: the step calls are made thousands of times per second
        self._tok_ptr = self._tok.ctypes.data
        self._fn_step, self._fn_plain = lib.ppd_step, lib.plain_greedy_step

    def _chk(self, rc: int, what: str) -> int:
        if rc < 0:
            raise PPDError(rc, what, load_library().ppd_last_hip_error(self._h))
        return rc

    def close(self):
        if getattr(self, "_h", None):
            load_library().ppd_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def ppd_reset(self):
        self._chk(load_library().ppd_reset(self._h), "ppd_reset")

    def ppd_prefill(self, prompt):
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        self._chk(load_library().ppd_prefill(self._h, p.ctypes.data, len(p)), "ppd_prefill")

    def ppd_step(self, want_info: bool = True):
        """One round.  Returns (token or None after EOS, StepInfo or None)."""
        info = StepInfo() if want_info else None
        n = self._fn_step(self._h, self._tok_ptr, 1, ctypes.byref(info) if want_info else None)
        if n < 0:
            self._chk(n, "ppd_step")
        return (int(self._tok[0]) if n == 1 else None), info

    def plain_greedy_step(self):
        n = self._fn_plain(self._h, self._tok_ptr)
        if n < 0:
            self._chk(n, "plain_greedy_step")
        return int(self._tok[0]) if n == 1 else None

    def ppd_get_logits(self) -> np.ndarray:
        self._chk(load_library().ppd_get_logits(self._h, self._logits.ctypes.data), "ppd_get_logits")
        return self._logits.copy()

    def ppd_get_early_logits(self) -> np.ndarray:
        self._chk(load_library().ppd_get_early_logits(self._h, self._logits.ctypes.data), "ppd_get_early_logits")
        return self._logits.copy()

    def ppd_get_stats(self) -> Dict[str, int]:
        s = Stats()
        self._chk(load_library().ppd_get_stats(self._h, ctypes.byref(s)), "ppd_get_stats")
        return {n: int(getattr(s, n)) for n, _ in Stats._fields_}

    def ppd_set_profiling(self, level: int):
        self._chk(load_library().ppd_set_profiling(self._h, int(level)), "ppd_set_profiling")

    def ppd_set_graphs(self, on: bool):
        self._chk(load_library().ppd_set_graphs(self._h, int(on)), "ppd_set_graphs")

    def ppd_set_sampling(self, mode: int, top_k: int = 0, top_p: float = 1.0, seed: int = 0):
        """Final prediction by arg max (0), top-k sampling (1) or top-p sampling (2)."""
        self._chk(load_library().ppd_set_sampling(self._h, int(mode), int(top_k), float(top_p), int(seed)), "ppd_set_sampling")

    def ppd_time_ffn_in(self, reps: int = 64, groups: int = 1) -> float:
        """Average milliseconds per FFN-in GEMM launch in a back-to-back burst (invalidates the sequence);
        groups = 2: the two-group launch of a pipelined step."""
        out = ctypes.c_double(0.0)
        self._chk(load_library().ppd_time_ffn_in(self._h, reps, groups, ctypes.byref(out)), "ppd_time_ffn_in")
        return float(out.value)

    def ppd_get_kernel_time(self) -> Dict[str, Dict[str, float]]:
        out = {}
        ms, n = ctypes.c_double(), ctypes.c_uint64()
        for groups in (1, 2):
            for i, name in enumerate(KERNEL_CLASSES):
                self._chk(load_library().ppd_get_kernel_time(self._h, i, groups, ctypes.byref(ms), ctypes.byref(n)),
                          "ppd_get_kernel_time")
                if n.value:
                    out[f"{name}.g{groups}"] = {"ms": ms.value, "launches": int(n.value)}
        return out
