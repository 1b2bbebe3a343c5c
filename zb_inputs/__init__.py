"""Seeded synthetic inputs for one zero-bubble pipeline stage.

This module only *makes data*: the stage's initial parameters, the activations
a previous stage would send, the output gradients a next stage would send, and
the scalar state other stages would contribute to the global gradient norm.
It holds none of the method's arithmetic (no layer math, no schedule rule, no
optimizer formula), so both the CPU oracle and the HIP library may be fed from
it without sharing code with each other.

Recipe (every tensor is drawn independently from a counter-based Philox stream
keyed by ``(seed, stream_id)``; ``stream_id`` packs tensor kind, layer,
iteration and microbatch):

* weight matrices  ~ N(0, 0.02^2); biases 0; LayerNorm gamma 1, beta 0
* stage input      X_k  ~ N(0, 1)         shape [seq*mb_size, hidden]
* upstream grads   dY_k ~ N(0, 1e-4)      (variance 1e-4, i.e. std 0.01)
* "other stages" squared gradient norm: a seeded positive scalar

For bf16 workloads the values are additionally rounded to the nearest bf16
(ties to even) and returned as float32 holding exactly representable values,
so that both consumers start from identical numbers.

The shapes follow the GPT-3-like models of the paper's experiment table
(hidden / heads / sequence 1024, FFN = 4*hidden, microbatch size 1).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List

import numpy as np

__all__ = [
    "Workload", "WORKLOADS", "workload", "PARAM_NAMES", "param_shape",
    "stage_params", "stage_input", "upstream_grad", "rest_state",
    "round_to_bf16", "nan_injection", "end_stage_params", "token_ids", "target_ids",
]

# tensor kinds used in stream ids
_K_PARAM, _K_X, _K_DY, _K_REST, _K_INJECT, _K_IDS, _K_TARGETS, _K_END = 1, 2, 3, 4, 5, 6, 7, 8

#: per-layer parameter names in the order used everywhere (weights are [in, out])
PARAM_NAMES = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
               "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "fp32" | "bf16"
    layers: int
    hidden: int
    heads: int
    ffn: int
    seq: int
    mb_size: int
    p: int                # pipeline stages
    stage: int            # 0-based stage index
    m: int                # microbatches per iteration
    kind: str             # "H1" | "H2"
    seed: int = 20240110
    iterations: int = 1
    optimizer: bool = False
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.95
    adam_eps: float = 1e-8
    weight_decay: float = 0.01
    clip: float = 1.0
    ln_eps: float = 1e-5
    nan_iteration: int = -1   # 0-based iteration that gets a NaN in one dY element

    @property
    def tokens(self) -> int:
        return self.seq * self.mb_size

    @property
    def head_dim(self) -> int:
        return self.hidden // self.heads

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    "c1": Workload("c1", "fp32", 2, 256, 4, 1024, 128, 1, 4, 0, 8, "H1"),
    "c2": Workload("c2", "bf16", 3, 2304, 24, 9216, 1024, 1, 8, 4, 24, "H1"),
    "c3": Workload("c3", "bf16", 4, 4096, 32, 16384, 1024, 1, 8, 4, 32, "H2"),
    "c4": Workload("c4", "bf16", 3, 5120, 40, 20480, 1024, 1, 16, 8, 48, "H1",
                   optimizer=True, lr=1e-4, beta1=0.9, beta2=0.95, clip=1.0),
    "c5": Workload("c5", "bf16", 2, 6144, 48, 24576, 1024, 1, 32, 16, 64, "H2",
                   iterations=4, optimizer=True, clip=1.0, nan_iteration=2),
}


def workload(name: str) -> Workload:
    return WORKLOADS[name]


def param_shape(w: Workload, name: str):
    h, f = w.hidden, w.ffn
    return {
        "ln1_g": (h,), "ln1_b": (h,), "wqkv": (h, 3 * h), "bqkv": (3 * h,),
        "wo": (h, h), "bo": (h,), "ln2_g": (h,), "ln2_b": (h,),
        "w1": (h, f), "b1": (f,), "w2": (f, h), "b2": (h,),
    }[name]


def _stream_id(kind: int, layer: int, it: int, mb: int, sub: int = 0) -> int:
    return (kind << 56) | (sub << 48) | (layer << 40) | (it << 20) | mb


def _normal(seed: int, sid: int, shape, std: float) -> np.ndarray:
    gen = np.random.Generator(np.random.Philox(key=np.array([seed, sid], dtype=np.uint64)))
    out = gen.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest-even rounding of float32 values to bf16, returned as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    expo = u & np.uint32(0x7F800000)
    finite = expo != np.uint32(0x7F800000)
    isnan = (~finite) & ((u & np.uint32(0x007FFFFF)) != 0)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    upper = u & np.uint32(0xFFFF0000)
    rounded = (u + bias) & np.uint32(0xFFFF0000)
    r = np.where(finite, rounded, np.where(isnan, upper | np.uint32(0x00400000), upper))
    return r.astype(np.uint32).view(np.float32).reshape(x.shape)


def _finish(w: Workload, x: np.ndarray) -> np.ndarray:
    return round_to_bf16(x) if w.dtype == "bf16" else x


def stage_params(w: Workload) -> List[Dict[str, np.ndarray]]:
    """Initial fp32 master parameters, one dict per layer (not bf16-rounded:
    the master copy is fp32; the working copy is whatever its consumer makes)."""
    out = []
    for l in range(w.layers):
        P = {}
        for i, name in enumerate(PARAM_NAMES):
            shp = param_shape(w, name)
            if name in ("wqkv", "wo", "w1", "w2"):
                P[name] = _normal(w.seed, _stream_id(_K_PARAM, l, 0, 0, i), shp, 0.02)
            elif name in ("ln1_g", "ln2_g"):
                P[name] = np.ones(shp, np.float32)
            else:
                P[name] = np.zeros(shp, np.float32)
        out.append(P)
    return out


def stage_input(w: Workload, it: int, mb: int) -> np.ndarray:
    """Activation the previous stage would send for microbatch mb: N(0,1)."""
    return _finish(w, _normal(w.seed, _stream_id(_K_X, 0, it, mb), (w.tokens, w.hidden), 1.0))


def upstream_grad(w: Workload, it: int, mb: int) -> np.ndarray:
    """Output gradient the next stage would send for microbatch mb: N(0,1e-4)."""
    g = _finish(w, _normal(w.seed, _stream_id(_K_DY, 0, it, mb), (w.tokens, w.hidden), 0.01))
    inj = nan_injection(w, it)
    if inj is not None and inj[0] == mb:
        g = g.copy()
        g.reshape(-1)[inj[1]] = np.float32("nan")
    return g


def nan_injection(w: Workload, it: int):
    """(microbatch, flat element index) that holds a NaN in iteration it, or None."""
    if it != w.nan_iteration:
        return None
    gen = np.random.Generator(np.random.Philox(key=np.array([w.seed, _stream_id(_K_INJECT, 0, it, 0)], dtype=np.uint64)))
    mb = int(gen.integers(0, w.m))
    elem = int(gen.integers(0, w.tokens * w.hidden))
    return mb, elem


def rest_state(w: Workload, it: int, scale: float = 1.0) -> float:
    """Seeded squared gradient norm contributed by the stages after this one."""
    gen = np.random.Generator(np.random.Philox(key=np.array([w.seed, _stream_id(_K_REST, 0, it, 0)], dtype=np.uint64)))
    return float(scale * (0.5 + gen.random()))


# ---------------------------------------------------------------------------------------------
# first / last stage (Sec. 5.1 of the paper: embedding lookup in the first, loss in the last)
# ---------------------------------------------------------------------------------------------
def end_stage_params(w: Workload, role: str, vocab: int) -> Dict[str, np.ndarray]:
    """Stage-level fp32 parameters: role "first" -> token and position tables N(0, 0.02^2);
    role "last" -> final LayerNorm (gamma 1, beta 0) and the head matrix [hidden, vocab] N(0, 0.02^2)."""
    h = w.hidden
    if role == "first":
        return {"emb_tok": _normal(w.seed, _stream_id(_K_END, 0, 0, 0, 0), (vocab, h), 0.02),
                "emb_pos": _normal(w.seed, _stream_id(_K_END, 0, 0, 0, 1), (w.seq, h), 0.02)}
    if role == "last":
        return {"lnf_g": np.ones((h,), np.float32), "lnf_b": np.zeros((h,), np.float32),
                "w_head": _normal(w.seed, _stream_id(_K_END, 0, 0, 0, 2), (h, vocab), 0.02)}
    raise ValueError("role must be 'first' or 'last'")


def _zipf_ids(seed: int, sid: int, n: int, vocab: int) -> np.ndarray:
    """Token ids with the rank-frequency shape of text: P(rank r) proportional to 1 / (r + 2.7), ranks mapped
    to ids by a fixed seeded permutation (so frequent ids are spread over the table).  A microbatch of 1024
    tokens then repeats its frequent ids many times, which is what the embedding gradient has to cope with."""
    gen = np.random.Generator(np.random.Philox(key=np.array([seed, sid], dtype=np.uint64)))
    weights = 1.0 / (np.arange(vocab, dtype=np.float64) + 2.7)
    cdf = np.cumsum(weights)
    ranks = np.searchsorted(cdf, gen.random(n) * cdf[-1], side="right")
    perm = np.random.Generator(np.random.Philox(key=np.array([seed, 0x5EED], dtype=np.uint64))).permutation(vocab)
    return perm[np.minimum(ranks, vocab - 1)].astype(np.int32)


def token_ids(w: Workload, it: int, mb: int, vocab: int) -> np.ndarray:
    """int32 [tokens] input ids of microbatch mb (first stage)."""
    return _zipf_ids(w.seed, _stream_id(_K_IDS, 0, it, mb), w.tokens, vocab)


def target_ids(w: Workload, it: int, mb: int, vocab: int) -> np.ndarray:
    """int32 [tokens] target ids of microbatch mb (last stage)."""
    return _zipf_ids(w.seed, _stream_id(_K_TARGETS, 0, it, mb), w.tokens, vocab)
