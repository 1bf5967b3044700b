"""Seeded synthetic models and prompts shared by the CPU oracle and the GPU library.

Nothing in here belongs to the decoding method: this module only names the
model shapes of the five benchmark configurations and fills their tensors
with reproducible random numbers (``gen.c``).  The oracle and the HIP library
both receive the very same bytes.

Recipe
------
* every matrix, embedding table and linear bias: iid N(0, 0.02)
* norm gains: 1 + N(0, 0.02); LayerNorm biases: N(0, 0.02) (so that a dropped
  gain or bias changes the result)
* controlled-match-rate variant: ``wo`` and ``w_out`` of the blocks after the
  exit layer are multiplied by ``alpha`` in fp32 before the single rounding
  to bf16
* bf16 tensors are rounded once, round-to-nearest-even, from fp32
* prompts: token ids iid uniform on [0, vocab)
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
import subprocess
from typing import Dict, List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libppd_inputs.so")
_lib = None

NORM_LAYERNORM, NORM_RMS = 0, 1
ACT_GELU, ACT_RELU, ACT_SWIGLU = 0, 1, 2
POS_LEARNED, POS_ROPE = 0, 1
WD_FP32, WD_BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile gen.c with gcc (CPU only)."""
    src = os.path.join(_HERE, "gen.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                               "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.ppd_inputs_fill_normal.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64,
                                               ctypes.c_uint64, ctypes.c_double, ctypes.c_double,
                                               ctypes.c_float, ctypes.c_int]
        lib.ppd_inputs_fill_normal.restype = None
        lib.ppd_inputs_fill_tokens.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64,
                                               ctypes.c_uint64, ctypes.c_int32]
        lib.ppd_inputs_fill_tokens.restype = None
        lib.ppd_inputs_checksum.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64]
        lib.ppd_inputs_checksum.restype = ctypes.c_uint64
        _lib = lib
    return _lib


@dataclasses.dataclass(frozen=True)
class ModelConfig:
    name: str
    n_layers: int          # d
    d_model: int
    n_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    max_ctx: int
    norm: int
    act: int
    pos: int
    has_bias: int
    wdtype: int
    norm_eps: float = 1e-5
    rope_theta: float = 10000.0
    # workload
    n_prompt: int = 16
    n_gen: int = 32        # l
    k: int = 3
    exit_layer: int = 2    # d-bar
    seed_w: int = 1000
    seed_p: int = 2000
    alpha: float = 1.0     # scale of wo / w_out in blocks exit_layer+1 .. d

    def replace(self, **kw) -> "ModelConfig":
        return dataclasses.replace(self, **kw)

    @property
    def wbytes(self) -> int:
        return 4 if self.wdtype == WD_FP32 else 2

    def layer_weight_bytes(self) -> int:
        dm, f = self.d_model, self.d_ff
        n = 4 * dm * dm + (3 if self.act == ACT_SWIGLU else 2) * dm * f
        return n * self.wbytes

    def head_weight_bytes(self) -> int:
        return self.vocab * self.d_model * self.wbytes

    def kv_bytes_per_pos_layer(self) -> int:
        return 2 * self.d_model * 4      # keys and values are cached in fp32


CONFIGS: Dict[str, ModelConfig] = {
    "tiny": ModelConfig("tiny", 4, 256, 4, 64, 1024, 1024, 128, NORM_LAYERNORM, ACT_GELU, POS_LEARNED, 1,
                        WD_FP32, n_prompt=16, n_gen=32, k=3, exit_layer=2, seed_w=1001, seed_p=2001),
    "opt125m": ModelConfig("opt125m", 12, 768, 12, 64, 3072, 50272, 2048, NORM_LAYERNORM, ACT_RELU,
                           POS_LEARNED, 1, WD_BF16, n_prompt=128, n_gen=128, k=3, exit_layer=6,
                           seed_w=1002, seed_p=2002),
    "llama7b": ModelConfig("llama7b", 32, 4096, 32, 128, 11008, 32000, 1024, NORM_RMS, ACT_SWIGLU, POS_ROPE,
                           0, WD_BF16, n_prompt=512, n_gen=256, k=3, exit_layer=16, seed_w=1003, seed_p=2003),
    "llama13b": ModelConfig("llama13b", 40, 5120, 40, 128, 13824, 32000, 4608, NORM_RMS, ACT_SWIGLU,
                            POS_ROPE, 0, WD_BF16, n_prompt=4096, n_gen=256, k=3, exit_layer=20,
                            seed_w=1004, seed_p=2004),
}
# controlled-match-rate variants of the 7B shape: same seed as llama7b, so alpha = 1.0 is that model
for _a, _n in ((1.0, "llama7b_a1"), (0.1, "llama7b_a0p1"), (0.02, "llama7b_a0p02")):
    CONFIGS[_n] = CONFIGS["llama7b"].replace(name=_n, alpha=_a, seed_p=2005)

# stream ids: kind * 4096 + layer
_GLOBAL_KINDS = {"tok_emb": 1, "pos_emb": 2, "lnf_g": 3, "lnf_b": 4, "lm_head": 5}
_LAYER_KINDS = {"ln1_g": 10, "ln1_b": 11, "wq": 12, "wk": 13, "wv": 14, "wo": 15, "bq": 16, "bk": 17,
                "bv": 18, "bo": 19, "ln2_g": 20, "ln2_b": 21, "w_in": 22, "w_up": 23, "w_out": 24,
                "b_in": 25, "b_out": 26}
LAYER_TENSORS = tuple(_LAYER_KINDS)
GLOBAL_TENSORS = tuple(_GLOBAL_KINDS)


def _normal(shape, seed, stream, mean, std, scale, wdtype) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(shape, dtype=np.float32 if wdtype == WD_FP32 else np.uint16)
    _load().ppd_inputs_fill_normal(out.ctypes.data, n, seed, stream, mean, std, scale,
                                   0 if wdtype == WD_FP32 else 1)
    return out


class SynthModel:
    """Host copy of a synthetic model.

    ``g[name]`` holds the global tensors and ``layers[name][l]`` the per-layer
    ones (0-based ``l``), each a C-contiguous numpy array: float32 when
    ``cfg.wdtype`` is fp32, uint16 holding bf16 bit patterns otherwise.
    Linear weights are row-major ``[out][in]``.  Absent tensors are ``None``.
    """

    def __init__(self, cfg: ModelConfig):
        self.cfg = cfg
        self.g: Dict[str, Optional[np.ndarray]] = {}
        self.layers: Dict[str, List[Optional[np.ndarray]]] = {k: [] for k in LAYER_TENSORS}

    def tensors(self):
        for k in GLOBAL_TENSORS:
            if self.g.get(k) is not None:
                yield k, self.g[k]
        for k in LAYER_TENSORS:
            for l, t in enumerate(self.layers[k]):
                if t is not None:
                    yield f"{k}.{l}", t

    def nbytes(self) -> int:
        return sum(t.nbytes for _, t in self.tensors())

    def checksum(self) -> int:
        """Label of the generated bytes (head of every tensor), for stored fixtures."""
        lib = _load()
        h = 0
        for _, t in self.tensors():
            h = lib.ppd_inputs_checksum(t.ctypes.data, min(t.nbytes, 4096), h)
        return int(h)


def make_model(cfg: ModelConfig) -> SynthModel:
    m = SynthModel(cfg)
    s, wd, dm, f = cfg.seed_w, cfg.wdtype, cfg.d_model, cfg.d_ff
    std = 0.02

    def gen(kind_id, layer, shape, mean=0.0, scale=1.0):
        return _normal(shape, s, kind_id * 4096 + layer, mean, std, scale, wd)

    G = _GLOBAL_KINDS
    m.g["tok_emb"] = gen(G["tok_emb"], 0, (cfg.vocab, dm))
    m.g["pos_emb"] = gen(G["pos_emb"], 0, (cfg.max_ctx, dm)) if cfg.pos == POS_LEARNED else None
    m.g["lnf_g"] = gen(G["lnf_g"], 0, (dm,), mean=1.0)
    m.g["lnf_b"] = gen(G["lnf_b"], 0, (dm,)) if cfg.norm == NORM_LAYERNORM else None
    m.g["lm_head"] = gen(G["lm_head"], 0, (cfg.vocab, dm))
    K = _LAYER_KINDS
    for l in range(cfg.n_layers):
        late = cfg.alpha if (l + 1) > cfg.exit_layer else 1.0
        L = m.layers
        L["ln1_g"].append(gen(K["ln1_g"], l, (dm,), mean=1.0))
        L["ln1_b"].append(gen(K["ln1_b"], l, (dm,)) if cfg.norm == NORM_LAYERNORM else None)
        L["wq"].append(gen(K["wq"], l, (dm, dm)))
        L["wk"].append(gen(K["wk"], l, (dm, dm)))
        L["wv"].append(gen(K["wv"], l, (dm, dm)))
        L["wo"].append(gen(K["wo"], l, (dm, dm), scale=late))
        for b in ("bq", "bk", "bv", "bo"):
            L[b].append(gen(K[b], l, (dm,)) if cfg.has_bias else None)
        L["ln2_g"].append(gen(K["ln2_g"], l, (dm,), mean=1.0))
        L["ln2_b"].append(gen(K["ln2_b"], l, (dm,)) if cfg.norm == NORM_LAYERNORM else None)
        L["w_in"].append(gen(K["w_in"], l, (f, dm)))
        L["w_up"].append(gen(K["w_up"], l, (f, dm)) if cfg.act == ACT_SWIGLU else None)
        L["w_out"].append(gen(K["w_out"], l, (dm, f), scale=late))
        L["b_in"].append(gen(K["b_in"], l, (f,)) if cfg.has_bias else None)
        L["b_out"].append(gen(K["b_out"], l, (dm,)) if cfg.has_bias else None)
    return m


def make_early_head(cfg: ModelConfig, model: Optional[SynthModel] = None, mix: float = 1.0) -> np.ndarray:
    """A second ``[vocab][d_model]`` classifier matrix for the early prediction (stands for the classifier
    trained per exit layer; here: seeded noise).  Without ``model``: iid N(0, 0.02), unrelated to the LM
    head.  With ``model``: the model's LM head plus ``mix`` times such noise, rounded once to the weight
    type, so that its predictions are close to the LM head's but its logits are not."""
    noise = _normal((cfg.vocab, cfg.d_model), cfg.seed_w, 6 * 4096, 0.0, 0.02, 1.0, WD_FP32)
    if model is None:
        base = np.zeros_like(noise)
        mix = 1.0
    else:
        base = to_float64(model.g["lm_head"]).astype(np.float32)
    v = (base + np.float32(mix) * noise).astype(np.float32)
    if cfg.wdtype == WD_FP32:
        return np.ascontiguousarray(v)
    u = v.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16            # round to nearest even (no NaNs here)
    return np.ascontiguousarray(u.astype(np.uint16))


def make_prompt(cfg: ModelConfig, n: Optional[int] = None) -> np.ndarray:
    n = cfg.n_prompt if n is None else n
    out = np.empty(n, dtype=np.int32)
    _load().ppd_inputs_fill_tokens(out.ctypes.data, n, cfg.seed_p, 0, cfg.vocab)
    return out


def to_float64(t: np.ndarray) -> np.ndarray:
    """Widen a generated tensor (fp32, or uint16 bf16 bits) to float64 exactly."""
    if t.dtype == np.uint16:
        return (t.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return t.astype(np.float64)
