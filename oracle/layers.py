"""F, B and W of a pre-LN GPT decoder layer, in fp64 (test infrastructure).

The paper (Sec. 1) writes a layer as y = f(x, W) and splits its backward into
  B:  grad_x f(x, W)^T dl/dy     (input gradient)
  W:  grad_W f(x, W)^T dl/dy     (parameter gradient)
with W free to run any time after the same stage's B (Sec. 2).  The layer shape
is the GPT-3-like one of Sec. 2.3: FFN inner size 4h (here `ffn`), head size
h/a.  Only matmuls are counted as FLOPs (Sec. 2.3, Table 1); every matmul goes
through `_mm`, which tallies 2*M*N*K per pass so that the tally can be checked
against Table 1.

Readings where the paper is silent (they are this build's, stated once here):
pre-LN residual blocks; causal attention; tanh-form GELU; LayerNorm with biased
variance; LayerNorm gamma/beta gradients are produced in B (its inputs are not
among what Table 1 keeps for W: 32sbh = the inputs and output-gradients of the
four linears only), bias gradients in W from the kept output-gradients.

Token layout: X is [b*s, h] row-major, sample-major (row = sample*s + position).
Weights are [in, out]; QKV columns are [Q | K | V], each head-major.
"""
from __future__ import annotations

import math
from typing import Dict, Optional, Tuple

import numpy as np

F64 = np.float64
GELU_C = math.sqrt(2.0 / math.pi)
GELU_A = 0.044715


class FlopTally:
    """Matmul FLOPs (2*M*N*K) per pass name."""

    def __init__(self):
        self.count = {"F": 0, "B": 0, "W": 0}

    def add(self, key: str, m: int, n: int, k: int, batch: int = 1):
        self.count[key] += 2 * m * n * k * batch


def _mm(a: np.ndarray, b: np.ndarray, tally: Optional[FlopTally], key: str) -> np.ndarray:
    """Matrix product (batched over leading dims) with FLOP accounting."""
    out = np.matmul(a, b)
    if tally is not None:
        batch = int(np.prod(out.shape[:-2])) if out.ndim > 2 else 1
        tally.add(key, a.shape[-2], b.shape[-1], a.shape[-1], batch)
    return out


# ----------------------------------------------------------------------------
# elementwise pieces
# ----------------------------------------------------------------------------
def layernorm_fwd(x, gamma, beta, eps):
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    r = 1.0 / np.sqrt(var + eps)
    xhat = xc * r
    return xhat * gamma + beta, xhat, r


def layernorm_bwd_input(g, xhat, r, gamma):
    """dx of LayerNorm given g = dl/d(out); also returns (dgamma, dbeta)."""
    gg = g * gamma
    m1 = gg.mean(axis=-1, keepdims=True)
    m2 = (gg * xhat).mean(axis=-1, keepdims=True)
    dx = r * (gg - m1 - xhat * m2)
    return dx, (g * xhat).sum(axis=0), g.sum(axis=0)


def gelu(x):
    return 0.5 * x * (1.0 + np.tanh(GELU_C * (x + GELU_A * x ** 3)))


def gelu_grad(x):
    t = np.tanh(GELU_C * (x + GELU_A * x ** 3))
    return 0.5 * (1.0 + t) + 0.5 * x * (1.0 - t * t) * GELU_C * (1.0 + 3.0 * GELU_A * x * x)


def _split_heads(z, b, s, a, d):
    """[b*s, a*d] -> [b, a, s, d]"""
    return z.reshape(b, s, a, d).transpose(0, 2, 1, 3)


def _merge_heads(z, b, s, a, d):
    """[b, a, s, d] -> [b*s, a*d]"""
    return z.transpose(0, 2, 1, 3).reshape(b * s, a * d)


# ----------------------------------------------------------------------------
# F
# ----------------------------------------------------------------------------
def layer_forward(X, P: Dict[str, np.ndarray], heads: int, seq: int, ln_eps: float,
                  tally: Optional[FlopTally] = None) -> Tuple[np.ndarray, dict]:
    """One decoder layer forward.  Returns (Y, cache-for-B)."""
    X = np.asarray(X, F64)
    T, h = X.shape
    b, a, d = T // seq, heads, h // heads
    A, xhat1, r1 = layernorm_fwd(X, P["ln1_g"], P["ln1_b"], ln_eps)
    QKV = _mm(A, P["wqkv"], tally, "F") + P["bqkv"]
    Q = _split_heads(QKV[:, 0:h], b, seq, a, d)
    K = _split_heads(QKV[:, h:2 * h], b, seq, a, d)
    V = _split_heads(QKV[:, 2 * h:3 * h], b, seq, a, d)
    S = _mm(Q, K.transpose(0, 1, 3, 2), tally, "F") / math.sqrt(d)
    future = np.triu(np.ones((seq, seq), dtype=bool), k=1)
    S = np.where(future, -np.inf, S)
    S = S - S.max(axis=-1, keepdims=True)
    E = np.exp(S)
    Pm = E / E.sum(axis=-1, keepdims=True)
    C = _merge_heads(_mm(Pm, V, tally, "F"), b, seq, a, d)
    Y1 = X + _mm(C, P["wo"], tally, "F") + P["bo"]
    U, xhat2, r2 = layernorm_fwd(Y1, P["ln2_g"], P["ln2_b"], ln_eps)
    Fh = _mm(U, P["w1"], tally, "F") + P["b1"]
    G = gelu(Fh)
    Y = Y1 + _mm(G, P["w2"], tally, "F") + P["b2"]
    cache = dict(xhat1=xhat1, r1=r1, A=A, Q=Q, K=K, V=V, Pm=Pm, C=C,
                 xhat2=xhat2, r2=r2, U=U, Fh=Fh, G=G, dims=(b, seq, a, d))
    return Y, cache


# ----------------------------------------------------------------------------
# B: input gradient.  Keeps, for W, the inputs and output-gradients of the four
# linears (Table 1: 32sbh bytes in the paper's 2-byte accounting) and nothing else.
# ----------------------------------------------------------------------------
def layer_backward_input(dY, P, cache, tally: Optional[FlopTally] = None):
    """Returns (dX, wstash, ln_grads).  ln_grads = LayerNorm gamma/beta gradients."""
    dY = np.asarray(dY, F64)
    b, s, a, d = cache["dims"]
    dG = _mm(dY, P["w2"].T, tally, "B")
    dFh = dG * gelu_grad(cache["Fh"])
    dU = _mm(dFh, P["w1"].T, tally, "B")
    dln2, dg2, db2 = layernorm_bwd_input(dU, cache["xhat2"], cache["r2"], P["ln2_g"])
    dY1 = dY + dln2
    dC = _mm(dY1, P["wo"].T, tally, "B")
    dO = _split_heads(dC, b, s, a, d)
    Pm, Q, K, V = cache["Pm"], cache["Q"], cache["K"], cache["V"]
    dV = _mm(Pm.transpose(0, 1, 3, 2), dO, tally, "B")
    dP = _mm(dO, V.transpose(0, 1, 3, 2), tally, "B")
    dS = Pm * (dP - (dP * Pm).sum(axis=-1, keepdims=True))
    scale = 1.0 / math.sqrt(d)
    dQ = _mm(dS, K, tally, "B") * scale
    dK = _mm(dS.transpose(0, 1, 3, 2), Q, tally, "B") * scale
    dQKV = np.concatenate([_merge_heads(dQ, b, s, a, d), _merge_heads(dK, b, s, a, d),
                           _merge_heads(dV, b, s, a, d)], axis=1)
    dA = _mm(dQKV, P["wqkv"].T, tally, "B")
    dln1, dg1, db1 = layernorm_bwd_input(dA, cache["xhat1"], cache["r1"], P["ln1_g"])
    dX = dY1 + dln1
    wstash = dict(A=cache["A"], dQKV=dQKV, C=cache["C"], dY1=dY1,
                  U=cache["U"], dFh=dFh, G=cache["G"], dY=dY)
    ln_grads = dict(ln1_g=dg1, ln1_b=db1, ln2_g=dg2, ln2_b=db2)
    return dX, wstash, ln_grads


# ----------------------------------------------------------------------------
# W: parameter gradient of the four linears from the kept (input, output-grad) pairs
# ----------------------------------------------------------------------------
def layer_backward_weight(wstash, tally: Optional[FlopTally] = None):
    g = {}
    for wname, bname, xin, dout in (("wqkv", "bqkv", "A", "dQKV"), ("wo", "bo", "C", "dY1"),
                                    ("w1", "b1", "U", "dFh"), ("w2", "b2", "G", "dY")):
        g[wname] = _mm(wstash[xin].T, wstash[dout], tally, "W")
        g[bname] = wstash[dout].sum(axis=0)
    return g


# ----------------------------------------------------------------------------
# The traditional single backward function (B and W grouped), written on its own
# with different formulations (einsum per head, Jacobian-style LayerNorm), so
# that "B then W" can be checked against it.
# ----------------------------------------------------------------------------
def layer_backward_unsplit(dY, X, P, heads: int, seq: int, ln_eps: float):
    """Recomputes the forward from X, then returns (dX, grads of all 12 parameters)."""
    X = np.asarray(X, F64)
    dY = np.asarray(dY, F64)
    T, h = X.shape
    b, a, d = T // seq, heads, h // heads

    def ln(x, g_, b_):
        mu = x.sum(-1, keepdims=True) / h
        sd = np.sqrt(((x - mu) ** 2).sum(-1, keepdims=True) / h + ln_eps)
        return (x - mu) / sd * g_ + b_, (x - mu) / sd, sd

    def ln_back(g_out, xh, sd, gam):
        # dx_j = (1/sd) * sum_i (delta_ij - 1/h - xh_i xh_j / h) * gam_i g_i
        w = g_out * gam
        return (w - w.sum(-1, keepdims=True) / h - xh * (w * xh).sum(-1, keepdims=True) / h) / sd

    grads = {}
    A, xh1, sd1 = ln(X, P["ln1_g"], P["ln1_b"])
    qkv = (A @ P["wqkv"] + P["bqkv"]).reshape(b, seq, 3, a, d)
    q, k, v = qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2]          # [b, s, a, d]
    sc = np.einsum("bian,bjan->baij", q, k) / math.sqrt(d)
    i_idx, j_idx = np.meshgrid(np.arange(seq), np.arange(seq), indexing="ij")
    sc[:, :, j_idx > i_idx] = -np.inf
    pr = np.exp(sc - sc.max(-1, keepdims=True))
    pr /= pr.sum(-1, keepdims=True)
    c = np.einsum("baij,bjan->bian", pr, v).reshape(T, h)
    y1 = X + c @ P["wo"] + P["bo"]
    U, xh2, sd2 = ln(y1, P["ln2_g"], P["ln2_b"])
    fh = U @ P["w1"] + P["b1"]
    G = gelu(fh)

    # MLP block
    grads["w2"] = G.T @ dY
    grads["b2"] = dY.sum(0)
    dfh = (dY @ P["w2"].T) * gelu_grad(fh)
    grads["w1"] = U.T @ dfh
    grads["b1"] = dfh.sum(0)
    dU = dfh @ P["w1"].T
    grads["ln2_g"] = (dU * xh2).sum(0)
    grads["ln2_b"] = dU.sum(0)
    dy1 = dY + ln_back(dU, xh2, sd2, P["ln2_g"])
    # attention block
    grads["wo"] = c.T @ dy1
    grads["bo"] = dy1.sum(0)
    dc = (dy1 @ P["wo"].T).reshape(b, seq, a, d)
    dv = np.einsum("baij,bian->bjan", pr, dc)
    dp = np.einsum("bian,bjan->baij", dc, v)
    ds = pr * (dp - (dp * pr).sum(-1, keepdims=True))
    dq = np.einsum("baij,bjan->bian", ds, k) / math.sqrt(d)
    dk = np.einsum("baij,bian->bjan", ds, q) / math.sqrt(d)
    dqkv = np.stack([dq, dk, dv], axis=2).reshape(T, 3 * h)
    grads["wqkv"] = A.T @ dqkv
    grads["bqkv"] = dqkv.sum(0)
    dA = dqkv @ P["wqkv"].T
    grads["ln1_g"] = (dA * xh1).sum(0)
    grads["ln1_b"] = dA.sum(0)
    dX = dy1 + ln_back(dA, xh1, sd1, P["ln1_g"])
    return dX, grads


# ----------------------------------------------------------------------------
# Table 1 of the paper: matmul FLOPs per transformer layer per pass
# ----------------------------------------------------------------------------
def table1_flops(s: int, b: int, h: int) -> Dict[str, int]:
    return {"F": s * b * h * (24 * h + 4 * s), "B": s * b * h * (24 * h + 8 * s), "W": s * b * h * 24 * h}
