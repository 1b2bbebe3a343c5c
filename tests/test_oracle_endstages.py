"""Pins of the first- and last-stage oracle (oracle/endstages.py; Sec. 5.1 of the paper): brute force, closed
forms, finite differences.  No GPU, no library."""
import math

import numpy as np
import pytest

import zb_inputs
from oracle import endstages as E
from oracle import optimizer as O
from oracle.schedule import stage_order
from oracle.stage import StageOracle

TINY = zb_inputs.Workload("tiny_end", "fp32", 1, 16, 2, 32, 8, 2, 4, 0, 3, "H1", seed=9)
V = 11


def test_embedding_forward_by_loops():
    rng = np.random.default_rng(0)
    tok, pos = rng.standard_normal((V, 5)), rng.standard_normal((4, 5))
    ids = np.array([3, 3, 0, 10, 7, 3, 1, 1])       # two sequences of 4
    X = E.embedding_forward(ids, tok, pos, 4)
    for t in range(8):
        for c in range(5):
            assert X[t, c] == tok[ids[t], c] + pos[t % 4, c]


def test_embedding_gradient_by_loops_and_finite_differences():
    rng = np.random.default_rng(1)
    ids = np.array([3, 3, 0, 10, 7, 3, 1, 1])
    dX0 = rng.standard_normal((8, 5))
    d_tok, d_pos = E.embedding_backward_weight(ids, dX0, V, 4)
    want_tok, want_pos = np.zeros((V, 5)), np.zeros((4, 5))
    for t in range(8):
        want_tok[ids[t]] += dX0[t]
        want_pos[t % 4] += dX0[t]
    np.testing.assert_allclose(d_tok, want_tok, rtol=0, atol=1e-15)
    np.testing.assert_allclose(d_pos, want_pos, rtol=0, atol=1e-15)
    assert np.all(d_tok[[2, 4, 5, 6, 8, 9]] == 0)                      # rows of unused ids stay zero
    tok, pos = rng.standard_normal((V, 5)), rng.standard_normal((4, 5))
    loss = lambda tk, ps: float((E.embedding_forward(ids, tk, ps, 4) * dX0).sum())
    eps = 1e-6
    for (v, c) in ((3, 2), (1, 0), (9, 4)):
        tp = tok.copy(); tp[v, c] += eps
        tm = tok.copy(); tm[v, c] -= eps
        assert (loss(tp, pos) - loss(tm, pos)) / (2 * eps) == pytest.approx(d_tok[v, c], abs=1e-8)
    pp = pos.copy(); pp[2, 1] += eps
    pm = pos.copy(); pm[2, 1] -= eps
    assert (loss(tok, pp) - loss(tok, pm)) / (2 * eps) == pytest.approx(d_pos[2, 1], abs=1e-8)


def test_loss_closed_forms():
    h, T = 6, 5
    rng = np.random.default_rng(2)
    X = rng.standard_normal((T, h))
    g, b = np.ones(h), np.zeros(h)
    targets = np.array([0, 3, 3, 10, 7])
    # a head of zeros gives uniform logits: the loss is log V whatever the targets
    loss, _ = E.head_forward(X, g, b, np.zeros((h, V)), targets, 1e-5)
    assert loss == pytest.approx(math.log(V), abs=1e-14)
    # textbook cross-entropy from explicit probabilities
    Wh = rng.standard_normal((h, V))
    loss, cache = E.head_forward(X, g, b, Wh, targets, 1e-5)
    mu = X.mean(1, keepdims=True)
    Z = (X - mu) / np.sqrt(((X - mu) ** 2).mean(1, keepdims=True) + 1e-5)
    p = np.exp(Z @ Wh)
    p /= p.sum(1, keepdims=True)
    assert loss == pytest.approx(-np.log(p[np.arange(T), targets]).mean(), rel=1e-13)
    # gradient of the logits: rows sum to zero, probabilities minus one-hot over T (and the loss scale)
    dX, stash, _ = E.head_backward_input(cache, g, Wh, 0.5)
    onehot = np.eye(V)[targets]
    np.testing.assert_allclose(stash["dlogits"], 0.5 * (p - onehot) / T, atol=1e-15)
    np.testing.assert_allclose(stash["dlogits"].sum(1), 0, atol=1e-16)
    # a huge logit on the target: loss -> 0 without overflow
    big = np.zeros((h, V)); big[:, 4] = 1e3
    loss, _ = E.head_forward(np.ones((2, h)) + np.arange(h), g, b + 1.0, big, np.array([4, 4]), 1e-5)
    assert 0.0 <= loss < 1e-12


def test_head_gradients_by_finite_differences():
    h, T = 6, 5
    rng = np.random.default_rng(3)
    X = rng.standard_normal((T, h))
    g, b = rng.standard_normal(h) + 1.0, rng.standard_normal(h)
    Wh = rng.standard_normal((h, V)) * 0.5
    targets = np.array([0, 3, 3, 10, 7])
    scale = 0.25
    f = lambda X_, g_, b_, W_: scale * E.head_forward(X_, g_, b_, W_, targets, 1e-5)[0]
    _, cache = E.head_forward(X, g, b, Wh, targets, 1e-5)
    dX, stash, (dg, db) = E.head_backward_input(cache, g, Wh, scale)
    dW = E.head_backward_weight(stash)
    eps = 1e-6

    def fd(arr, idx, fn):
        p_, m_ = arr.copy(), arr.copy()
        p_[idx] += eps
        m_[idx] -= eps
        return (fn(p_) - fn(m_)) / (2 * eps)

    for idx in ((0, 0), (2, 3), (4, 5)):
        assert fd(X, idx, lambda a: f(a, g, b, Wh)) == pytest.approx(dX[idx], abs=1e-8)
    for idx in ((0,), (4,)):
        assert fd(g, idx, lambda a: f(X, a, b, Wh)) == pytest.approx(dg[idx], abs=1e-8)
        assert fd(b, idx, lambda a: f(X, g, a, Wh)) == pytest.approx(db[idx], abs=1e-8)
    for idx in ((0, 0), (3, 3), (5, 10)):
        assert fd(Wh, idx, lambda a: f(X, g, b, a)) == pytest.approx(dW[idx], abs=1e-8)


def make(role, m=3, dtype="fp32"):
    w = TINY.scaled(dtype=dtype, m=m)
    return w, E.EndStageOracle(role=role, vocab=V, extra_params=zb_inputs.end_stage_params(w, role, V),
                               layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq,
                               mb_size=w.mb_size, dtype=dtype, params=zb_inputs.stage_params(w))


def test_first_stage_end_to_end_finite_differences_and_order_independence():
    w, orc = make("first")
    m = w.m
    def run(o, order):
        o.begin_iteration(m)
        for k in range(m):
            o.set_ids(k, zb_inputs.token_ids(w, 0, k, V))
            o.set_upstream_grad(k, zb_inputs.upstream_grad(w, 0, k))
        o.run(order)
    run(orc, stage_order(4, 0, m, "H1"))
    objective = lambda o: sum(float((o.Y[k] * o.dY[k]).sum()) for k in range(m))
    base_grads = {k: v.copy() for k, v in orc.grads[orc.nl].items()}
    assert np.abs(base_grads["emb_tok"]).max() > 0
    eps = 1e-5
    ids0 = zb_inputs.token_ids(w, 0, 0, V)
    for name, idx in (("emb_tok", (int(ids0[0]), 3)), ("emb_tok", (int(ids0[5]), 0)), ("emb_pos", (2, 7))):
        vals = []
        for sgn in (+1, -1):
            _, o2 = make("first")
            o2.master[o2.nl][name][idx] += sgn * eps
            o2._refresh_working()
            run(o2, stage_order(4, 0, m, "H1"))
            vals.append(objective(o2))
        assert (vals[0] - vals[1]) / (2 * eps) == pytest.approx(base_grads[name][idx], rel=1e-5, abs=1e-9)
    # any legal order gives the same bits (fp64 sums in microbatch order)
    _, o3 = make("first")
    run(o3, [(0, k) for k in range(m)] + [(1, k) for k in range(m)] + [(2, k) for k in range(m)])
    for k in base_grads:
        assert o3.grads[o3.nl][k].tobytes() == base_grads[k].tobytes()


def test_last_stage_end_to_end_finite_differences_and_loss_scale():
    w, orc = make("last")
    m = w.m
    def run(o):
        o.begin_iteration(m)
        for k in range(m):
            o.set_input(k, zb_inputs.stage_input(w, 0, k))
            o.set_targets(k, zb_inputs.target_ids(w, 0, k, V))
        o.run(stage_order(4, 3, m, "H1"))
        return o.iteration_loss()
    loss = run(orc)
    assert 0.5 * math.log(V) < loss < 2.0 * math.log(V)      # random head: near the uniform value
    eps = 1e-5
    checks = [(orc.nl, "w_head", (3, 4)), (orc.nl, "lnf_g", (5,)), (orc.nl, "lnf_b", (0,)), (0, "w1", (2, 9)),
              (0, "ln1_g", (1,)), (0, "bqkv", (7,))]
    for l, name, idx in checks:
        vals = []
        for sgn in (+1, -1):
            _, o2 = make("last")
            o2.master[l][name][idx] += sgn * eps
            o2._refresh_working()
            vals.append(run(o2))
        # the accumulated gradients are those of the ITERATION loss: mean over microbatches of the mean token loss
        assert (vals[0] - vals[1]) / (2 * eps) == pytest.approx(orc.grads[l][name][idx], rel=2e-5, abs=1e-9)
    # the gradient sent to the previous stage: d(iteration loss) / d(input of microbatch 1)
    X1 = zb_inputs.stage_input(w, 0, 1).astype(np.float64)
    vals = []
    for sgn in (+1, -1):
        _, o2 = make("last")
        o2.begin_iteration(m)
        for k in range(m):
            Xk = zb_inputs.stage_input(w, 0, k).astype(np.float64)
            if k == 1:
                Xk = Xk.copy(); Xk[3, 2] += sgn * eps
            o2.set_input(k, Xk)
            o2.set_targets(k, zb_inputs.target_ids(w, 0, k, V))
        o2.run(stage_order(4, 3, m, "H1"))
        vals.append(o2.iteration_loss())
    assert (vals[0] - vals[1]) / (2 * eps) == pytest.approx(orc.dX[1][3, 2], rel=2e-5, abs=1e-10)


def test_optimizer_covers_the_stage_level_parameters():
    w, orc = make("last", m=2)
    orc.begin_iteration(2)
    for k in range(2):
        orc.set_input(k, zb_inputs.stage_input(w, 0, k))
        orc.set_targets(k, zb_inputs.target_ids(w, 0, k, V))
    orc.run(stage_order(4, 3, 2, "H1"))
    before = orc.master[orc.nl]["w_head"].copy()
    g = orc.grads[orc.nl]["w_head"].copy()
    rep = orc.optimizer_step(O.GlobalState(0.0, 0.0))
    assert rep.outcome == O.COMMITTED and orc.t == 1
    # first AdamW step of an element: theta - lr*wd*theta - lr*g/(|g| + eps)
    hp = orc.hp
    want = before - hp.lr * hp.weight_decay * before - hp.lr * g / (np.abs(g) + hp.eps)
    np.testing.assert_allclose(orc.master[orc.nl]["w_head"], want, rtol=1e-12, atol=1e-18)


def test_bf16_mode_rounds_tables_and_head_only_in_the_working_copy():
    w, orc = make("first", dtype="bf16")
    tok = orc.master[orc.nl]["emb_tok"]
    assert np.array_equal(orc.work_extra["emb_tok"], zb_inputs.round_to_bf16(tok.astype(np.float32)).astype(np.float64))
    assert not np.array_equal(orc.work_extra["emb_tok"], tok)


def test_token_ids_are_skewed_and_in_range():
    w = zb_inputs.workload("c4")
    ids = zb_inputs.token_ids(w, 0, 0, 50432)
    assert ids.dtype == np.int32 and ids.shape == (1024,) and ids.min() >= 0 and ids.max() < 50432
    assert len(np.unique(ids)) < 1000            # repeated ids inside one microbatch
    assert not np.array_equal(ids, zb_inputs.token_ids(w, 0, 1, 50432))
    assert np.array_equal(ids, zb_inputs.token_ids(w, 0, 0, 50432))
