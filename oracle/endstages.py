"""First and last pipeline stage (test infrastructure).

Sec. 5.1 of the paper: the first and the last stage hold one transformer layer
fewer than the stages between them, because the first also does the embedding
lookup and the last the loss computation.  The paper says no more about the two;
the model is "analogous to GPT-3", so the readings of this build are:

 * first stage: activation entering its layers = token embedding + learned
   position embedding, X0[t] = E_tok[ids[t]] + E_pos[t mod s] (no dropout);
   its parameter gradients dE_tok[v] = sum of dX0[t] over the tokens t with
   ids[t] = v, dE_pos[p] = sum of dX0 over the sequences' position p, belong to
   the W pass (they are parameter gradients; what W needs for them, ids and dX0,
   is what B leaves behind);
 * last stage: final LayerNorm, linear head h -> V without bias (not tied to
   the embedding: the two live on different devices), softmax cross-entropy
   against target ids, loss of a microbatch = mean over its tokens; the
   iteration's loss is the mean over its m microbatches, so the gradient that
   starts B is (softmax - onehot) / (tokens * m).  As for the layers, the
   LayerNorm's gamma/beta gradients are produced in B, the head's weight
   gradient Z^T dLogits in W.

Plain definitions in fp64 (numpy); `EndStageOracle` wraps them around the layer
stack of oracle/stage.py with the same F / B / W calls and optimizer.
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence

import numpy as np

from . import layers as L
from .stage import MATRICES, PARAM_ORDER, StageOracle, bf16_round
from .schedule import F as PASS_F, B as PASS_B, W as PASS_W

FIRST_PARAMS = ("emb_tok", "emb_pos")
LAST_PARAMS = ("lnf_g", "lnf_b", "w_head")


def embedding_forward(ids: np.ndarray, emb_tok: np.ndarray, emb_pos: np.ndarray, seq: int) -> np.ndarray:
    """X0[t] = E_tok[ids[t]] + E_pos[t mod seq] for the sample-major token rows t."""
    ids = np.asarray(ids, np.int64)
    pos = np.arange(ids.size) % seq
    return emb_tok[ids] + emb_pos[pos]


def embedding_backward_weight(ids: np.ndarray, dX0: np.ndarray, vocab: int, seq: int):
    """(dE_tok, dE_pos): every token adds its gradient row to its table rows."""
    ids = np.asarray(ids, np.int64)
    dX0 = np.asarray(dX0, np.float64)
    d_tok = np.zeros((vocab, dX0.shape[1]))
    np.add.at(d_tok, ids, dX0)
    d_pos = dX0.reshape(-1, seq, dX0.shape[1]).sum(axis=0)
    return d_tok, d_pos


def head_forward(X, lnf_g, lnf_b, w_head, targets, ln_eps, tally=None):
    """Final LayerNorm, logits, softmax cross-entropy.  Returns (mean loss, cache for B)."""
    X = np.asarray(X, np.float64)
    targets = np.asarray(targets, np.int64)
    Z, xhat, r = L.layernorm_fwd(X, lnf_g, lnf_b, ln_eps)
    logits = L._mm(Z, w_head, tally, "F")
    top = logits.max(axis=-1, keepdims=True)
    lse = top[:, 0] + np.log(np.exp(logits - top).sum(axis=-1))
    per_token = lse - logits[np.arange(targets.size), targets]
    return float(per_token.mean()), dict(Z=Z, xhat=xhat, r=r, logits=logits, lse=lse, targets=targets)


def head_backward_input(cache, lnf_g, w_head, scale: float, tally=None):
    """Gradient of scale * (mean loss) w.r.t. the head's input X.  Returns (dX, stash for W, (dgamma, dbeta))."""
    logits, lse, targets = cache["logits"], cache["lse"], cache["targets"]
    T = targets.size
    dlogits = np.exp(logits - lse[:, None])
    dlogits[np.arange(T), targets] -= 1.0
    dlogits *= scale / T
    dZ = L._mm(dlogits, w_head.T, tally, "B")
    dX, dg, db = L.layernorm_bwd_input(dZ, cache["xhat"], cache["r"], lnf_g)
    return dX, dict(Z=cache["Z"], dlogits=dlogits), (dg, db)


def head_backward_weight(stash, tally=None):
    return L._mm(stash["Z"].T, stash["dlogits"], tally, "W")


class EndStageOracle(StageOracle):
    """role = "first": ids -> embedding -> layers; role = "last": layers -> LayerNorm -> head -> loss."""

    def __init__(self, *, role: str, vocab: int, extra_params: Dict[str, np.ndarray], **kw):
        assert role in ("first", "last")
        self.role, self.vocab = role, vocab
        names = FIRST_PARAMS if role == "first" else LAST_PARAMS
        self._extra_init = {k: np.array(extra_params[k], np.float64) for k in names}
        super().__init__(**kw)

    # the stage-level parameters travel as one more dictionary behind the layers' in master / moments / grads
    def _refresh_working(self):
        if len(self.master) == self.nl:
            self.master.append(self._extra_init)
            self.adam_m.append({k: np.zeros_like(v) for k, v in self._extra_init.items()})
            self.adam_v.append({k: np.zeros_like(v) for k, v in self._extra_init.items()})
        self.work = []
        for P in self.master[:self.nl]:
            Wk = dict(P)
            if self.dtype == "bf16":
                for k in MATRICES:
                    Wk[k] = bf16_round(P[k].astype(np.float32))
            self.work.append(Wk)
        ex = dict(self.master[self.nl])
        if self.dtype == "bf16":   # the tables and the head are weight matrices: bf16 working copies
            for k in ("emb_tok", "emb_pos", "w_head"):
                if k in ex:
                    ex[k] = bf16_round(ex[k].astype(np.float32))
        self.work_extra = ex

    def begin_iteration(self, m: int):
        super().begin_iteration(m)
        self.ids: Dict[int, np.ndarray] = {}
        self.targets: Dict[int, np.ndarray] = {}
        self.loss: Dict[int, float] = {}
        self._head: Dict[int, dict] = {}
        self._head_w: Dict[int, dict] = {}

    def set_ids(self, mb: int, ids):
        self.ids[mb] = np.asarray(ids, np.int64)

    def set_targets(self, mb: int, targets):
        self.targets[mb] = np.asarray(targets, np.int64)

    def forward(self, mb: int):
        if self.role == "first":
            self.X[mb] = embedding_forward(self.ids[mb], self.work_extra["emb_tok"], self.work_extra["emb_pos"], self.s)
        super().forward(mb)
        if self.role == "last":
            ex = self.work_extra
            self.loss[mb], self._head[mb] = head_forward(self.Y[mb], ex["lnf_g"], ex["lnf_b"], ex["w_head"],
                                                         self.targets[mb], self.ln_eps, self.tally)

    def backward_input(self, mb: int):
        if self.role == "last":
            ex = self.work_extra
            dY, self._head_w[mb], (dg, db) = head_backward_input(self._head.pop(mb), ex["lnf_g"], ex["w_head"],
                                                                 1.0 / self.m, self.tally)
            self.dY[mb] = dY
            self.grads[self.nl]["lnf_g"] += dg
            self.grads[self.nl]["lnf_b"] += db
        super().backward_input(mb)

    def backward_weight(self, mb: int):
        super().backward_weight(mb)
        if self.role == "last":
            self.grads[self.nl]["w_head"] += head_backward_weight(self._head_w.pop(mb), self.tally)
        else:
            d_tok, d_pos = embedding_backward_weight(self.ids[mb], self.dX[mb], self.vocab, self.s)
            self.grads[self.nl]["emb_tok"] += d_tok
            self.grads[self.nl]["emb_pos"] += d_pos

    def iteration_loss(self) -> float:
        """Mean over the microbatches run so far of their mean token loss."""
        return float(np.mean([self.loss[k] for k in sorted(self.loss)]))
