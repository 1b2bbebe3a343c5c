"""A whole pipeline stage on the CPU (test infrastructure): L decoder layers run
as separate F / B / W passes per microbatch, parameter gradients accumulated
over microbatches, then the post-validated AdamW step.

The only per-stage ordering constraint of the paper (Sec. 2) is enforced:
F_k before B_k before W_k, each at most once per iteration.  Memory follows
Appendix G's life cycle: F creates the B-stash, B turns it into the W-stash, W
releases it; the pending counts are exposed so tests can compare them with the
closed forms of Sec. 2.3.

Precision model for the "bf16" data type (the paper says only "mixed
precision"): fp32 master parameters, Adam moments and accumulated gradients;
the four weight matrices are used in the layer math rounded to bf16 (nearest
even); everything here is then computed in fp64, so a comparison against a
bf16 device path measures only that path's internal rounding.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np

from . import layers as L
from . import optimizer as O
from .schedule import F as PASS_F, B as PASS_B, W as PASS_W

MATRICES = ("wqkv", "wo", "w1", "w2")
PARAM_ORDER = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
               "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round fp32-representable values to the nearest bf16 (ties to even); returns fp64."""
    f = np.asarray(x, np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    keep = bits >> np.uint64(16)
    rem = bits & np.uint64(0xFFFF)
    up = (rem > 0x8000) | ((rem == 0x8000) & ((keep & np.uint64(1)) == 1))
    special = (bits & np.uint64(0x7F800000)) == np.uint64(0x7F800000)   # inf or NaN: truncate
    nan = special & ((bits & np.uint64(0x007FFFFF)) != 0)
    keep = np.where(special, np.where(nan, keep | np.uint64(0x40), keep), keep + up)
    out = (keep << np.uint64(16)).astype(np.uint32).view(np.float32)
    return out.astype(np.float64).reshape(np.shape(x))


class OrderError(RuntimeError):
    pass


class StageOracle:
    def __init__(self, *, layers: int, hidden: int, heads: int, ffn: int, seq: int,
                 mb_size: int = 1, dtype: str = "fp32", ln_eps: float = 1e-5,
                 hyper: O.Hyper = None, params: Sequence[Dict[str, np.ndarray]] = None,
                 count_flops: bool = False):
        assert dtype in ("fp32", "bf16")
        assert len(params) == layers
        self.nl, self.h, self.a, self.ffn, self.s, self.b = layers, hidden, heads, ffn, seq, mb_size
        self.dtype, self.ln_eps = dtype, ln_eps
        self.hp = hyper or O.Hyper()
        self.master = [{k: np.array(P[k], np.float64) for k in PARAM_ORDER} for P in params]
        self.adam_m = [{k: np.zeros_like(P[k]) for k in PARAM_ORDER} for P in self.master]
        self.adam_v = [{k: np.zeros_like(P[k]) for k in PARAM_ORDER} for P in self.master]
        self.t = 0
        self.tally = L.FlopTally() if count_flops else None
        self._refresh_working()
        self.begin_iteration(0)

    # -- parameters --------------------------------------------------------
    def _refresh_working(self):
        self.work = []
        for P in self.master:
            Wk = dict(P)
            if self.dtype == "bf16":
                for k in MATRICES:
                    Wk[k] = bf16_round(P[k].astype(np.float32))
            self.work.append(Wk)

    def _flat(self, dicts) -> np.ndarray:
        return np.concatenate([d[k].reshape(-1) for d in dicts for k in d])

    def _unflat(self, vec, dicts):
        o = 0
        for d in dicts:
            for k in d:
                n = d[k].size
                d[k][...] = vec[o:o + n].reshape(d[k].shape)
                o += n

    # -- iteration ---------------------------------------------------------
    def begin_iteration(self, m: int):
        self.m = m
        self.X: Dict[int, np.ndarray] = {}
        self.dY: Dict[int, np.ndarray] = {}
        self.Y: Dict[int, np.ndarray] = {}
        self.dX: Dict[int, np.ndarray] = {}
        self._bstash: Dict[int, list] = {}
        self._wstash: Dict[int, list] = {}
        self._done = {PASS_F: set(), PASS_B: set(), PASS_W: set()}
        self.grads = [{k: np.zeros_like(v) for k, v in P.items()} for P in self.master]
        self.max_pending_b = self.max_pending_w = 0

    def set_input(self, mb: int, X: np.ndarray):
        self.X[mb] = np.asarray(X, np.float64)

    def set_upstream_grad(self, mb: int, dY: np.ndarray):
        self.dY[mb] = np.asarray(dY, np.float64)

    def _check(self, c: int, mb: int):
        if not 0 <= mb < self.m:
            raise OrderError(f"microbatch {mb} out of range")
        if mb in self._done[c]:
            raise OrderError(f"pass {c} of microbatch {mb} repeated")
        if c == PASS_B and mb not in self._done[PASS_F]:
            raise OrderError(f"B({mb}) before F({mb})")
        if c == PASS_W and mb not in self._done[PASS_B]:
            raise OrderError(f"W({mb}) before B({mb})")

    def forward(self, mb: int):
        self._check(PASS_F, mb)
        x = self.X[mb]
        caches = []
        for l in range(self.nl):
            x, cache = L.layer_forward(x, self.work[l], self.a, self.s, self.ln_eps, self.tally)
            caches.append(cache)
        self.Y[mb] = x
        self._bstash[mb] = caches
        self._done[PASS_F].add(mb)
        self.max_pending_b = max(self.max_pending_b, len(self._bstash))

    def backward_input(self, mb: int):
        self._check(PASS_B, mb)
        g = self.dY[mb]
        caches = self._bstash.pop(mb)
        wst = [None] * self.nl
        for l in reversed(range(self.nl)):
            g, wst[l], lng = L.layer_backward_input(g, self.work[l], caches[l], self.tally)
            for k, val in lng.items():
                self.grads[l][k] += val
        self.dX[mb] = g
        self._wstash[mb] = wst
        self._done[PASS_B].add(mb)
        self.max_pending_w = max(self.max_pending_w, len(self._wstash))

    def backward_weight(self, mb: int):
        self._check(PASS_W, mb)
        wst = self._wstash.pop(mb)
        for l in reversed(range(self.nl)):
            for k, val in L.layer_backward_weight(wst[l], self.tally).items():
                self.grads[l][k] += val
        self._done[PASS_W].add(mb)

    def run(self, order):
        for c, mb in order:
            (self.forward, self.backward_input, self.backward_weight)[c](mb)

    # -- optimizer ---------------------------------------------------------
    def optimizer_step(self, gs: O.GlobalState, synchronous: bool = False) -> O.StepReport:
        st = O.AdamState(self._flat(self.master), self._flat(self.adam_m), self._flat(self.adam_v), self.t)
        g = self._flat(self.grads)
        fn = O.synchronous_step if synchronous else O.post_validated_step
        rep = fn(st, g, self.hp, gs)
        self._unflat(st.theta, self.master)
        self._unflat(st.m, self.adam_m)
        self._unflat(st.v, self.adam_v)
        self.t = st.t
        self._refresh_working()
        return rep
