"""Pins for oracle/layers.py and oracle/stage.py: each check ties the oracle to
something other than itself (finite differences, brute-force loops, an
independently written monolithic backward, the paper's Table 1, torch's own
bf16 conversion)."""
import math

import numpy as np
import pytest

from oracle import layers as L
from oracle.stage import StageOracle, bf16_round, PARAM_ORDER, OrderError
from oracle.schedule import stage_order, F as PF, B as PB, W as PW


def make_params(rng, layers, h, ffn, scale=0.3):
    out = []
    for _ in range(layers):
        out.append({
            "ln1_g": 1 + 0.1 * rng.standard_normal(h), "ln1_b": 0.1 * rng.standard_normal(h),
            "wqkv": scale * rng.standard_normal((h, 3 * h)), "bqkv": 0.1 * rng.standard_normal(3 * h),
            "wo": scale * rng.standard_normal((h, h)), "bo": 0.1 * rng.standard_normal(h),
            "ln2_g": 1 + 0.1 * rng.standard_normal(h), "ln2_b": 0.1 * rng.standard_normal(h),
            "w1": scale * rng.standard_normal((h, ffn)), "b1": 0.1 * rng.standard_normal(ffn),
            "w2": scale * rng.standard_normal((ffn, h)), "b2": 0.1 * rng.standard_normal(h),
        })
    return out


def tiny_stage(seed=0, layers=2, s=8, h=16, a=2, b=1, **kw):
    rng = np.random.default_rng(seed)
    params = make_params(rng, layers, h, 4 * h)
    st = StageOracle(layers=layers, hidden=h, heads=a, ffn=4 * h, seq=s, mb_size=b, params=params, **kw)
    return st, rng


# --------------------------------------------------------------------------
# forward: brute-force loops for one layer, one head (textbook attention + MLP)
# --------------------------------------------------------------------------
def brute_force_layer(X, P, heads, eps):
    s, h = X.shape
    d = h // heads

    def ln_row(x, g, b):
        mu = sum(x) / h
        var = sum((xi - mu) ** 2 for xi in x) / h
        return [(xi - mu) / math.sqrt(var + eps) * gi + bi for xi, gi, bi in zip(x, g, b)]

    A = [ln_row(list(X[i]), P["ln1_g"], P["ln1_b"]) for i in range(s)]
    QKV = [[sum(A[i][k] * P["wqkv"][k][n] for k in range(h)) + P["bqkv"][n] for n in range(3 * h)] for i in range(s)]
    C = [[0.0] * h for _ in range(s)]
    for hd in range(heads):
        qo, ko, vo = hd * d, h + hd * d, 2 * h + hd * d
        for i in range(s):
            sc = [sum(QKV[i][qo + e] * QKV[j][ko + e] for e in range(d)) / math.sqrt(d) for j in range(i + 1)]
            mx = max(sc)
            ex = [math.exp(v - mx) for v in sc]
            z = sum(ex)
            for e in range(d):
                C[i][hd * d + e] = sum(ex[j] / z * QKV[j][vo + e] for j in range(i + 1))
    Y1 = [[X[i][n] + sum(C[i][k] * P["wo"][k][n] for k in range(h)) + P["bo"][n] for n in range(h)] for i in range(s)]
    U = [ln_row(Y1[i], P["ln2_g"], P["ln2_b"]) for i in range(s)]
    f = P["w1"].shape[1]
    Fh = [[sum(U[i][k] * P["w1"][k][n] for k in range(h)) + P["b1"][n] for n in range(f)] for i in range(s)]
    G = [[0.5 * v * (1 + math.tanh(math.sqrt(2 / math.pi) * (v + 0.044715 * v ** 3))) for v in row] for row in Fh]
    Y = [[Y1[i][n] + sum(G[i][k] * P["w2"][k][n] for k in range(f)) + P["b2"][n] for n in range(h)] for i in range(s)]
    return np.array(Y)


@pytest.mark.parametrize("heads", [1, 2])
def test_forward_matches_brute_force_loops(heads):
    rng = np.random.default_rng(1)
    s, h = 5, 8
    P = make_params(rng, 1, h, 4 * h)[0]
    X = rng.standard_normal((s, h))
    Y, _ = L.layer_forward(X, P, heads, s, 1e-5)
    np.testing.assert_allclose(Y, brute_force_layer(X, P, heads, 1e-5), rtol=1e-12, atol=1e-12)


def test_softmax_rows_sum_to_one_and_causal():
    rng = np.random.default_rng(2)
    s, h, a = 12, 16, 4
    P = make_params(rng, 1, h, 4 * h)[0]
    X = rng.standard_normal((s, h))
    Y, cache = L.layer_forward(X, P, a, s, 1e-5)
    np.testing.assert_allclose(cache["Pm"].sum(-1), 1.0, atol=1e-14)
    assert np.all(np.triu(cache["Pm"], k=1) == 0.0)
    # output row i must not depend on input rows > i
    X2 = X.copy()
    X2[7:] += rng.standard_normal((s - 7, h))
    Y2, _ = L.layer_forward(X2, P, a, s, 1e-5)
    np.testing.assert_array_equal(Y[:7], Y2[:7])
    assert np.abs(Y[7:] - Y2[7:]).max() > 1e-3


def test_batched_samples_do_not_attend_to_each_other():
    rng = np.random.default_rng(3)
    s, h, a, b = 6, 8, 2, 3
    P = make_params(rng, 1, h, 4 * h)[0]
    X = rng.standard_normal((b * s, h))
    Y, _ = L.layer_forward(X, P, a, s, 1e-5)
    for n in range(b):
        Yn, _ = L.layer_forward(X[n * s:(n + 1) * s], P, a, s, 1e-5)
        np.testing.assert_allclose(Y[n * s:(n + 1) * s], Yn, rtol=1e-13, atol=1e-13)


def test_layernorm_and_gelu_closed_forms():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((7, 32)) * 3 + 5
    out, xhat, r = L.layernorm_fwd(x, np.ones(32), np.zeros(32), 0.0)
    np.testing.assert_allclose(out.mean(-1), 0, atol=1e-13)
    np.testing.assert_allclose((out ** 2).mean(-1), 1, rtol=1e-12)
    out2, _, _ = L.layernorm_fwd(x + 11.0, np.ones(32), np.zeros(32), 0.0)
    np.testing.assert_allclose(out, out2, atol=1e-11)
    z = np.linspace(-6, 6, 41)
    assert L.gelu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(L.gelu(z) - L.gelu(-z), z, atol=1e-14)       # identity of the tanh form
    np.testing.assert_allclose(L.gelu(np.array([30.0])), 30.0)
    # against the erf definition x*Phi(x): the tanh form is a <1e-3 approximation of it
    erf_form = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in z])
    assert np.abs(L.gelu(z) - erf_form).max() < 1e-3
    eps = 1e-6
    np.testing.assert_allclose(L.gelu_grad(z), (L.gelu(z + eps) - L.gelu(z - eps)) / (2 * eps), atol=1e-8)


# --------------------------------------------------------------------------
# B and W: central finite differences of l = sum_k <Y_k, dY_k>
# --------------------------------------------------------------------------
def stage_loss(st, params, Xs, dYs):
    s2 = StageOracle(layers=st.nl, hidden=st.h, heads=st.a, ffn=st.ffn, seq=st.s, mb_size=st.b, params=params)
    s2.begin_iteration(len(Xs))
    tot = 0.0
    for k, X in enumerate(Xs):
        s2.set_input(k, X)
        s2.forward(k)
        tot += float((s2.Y[k] * dYs[k]).sum())
    return tot


def test_split_backward_matches_finite_differences():
    st, rng = tiny_stage(seed=5)
    m = 3
    Xs = [rng.standard_normal((st.s, st.h)) for _ in range(m)]
    dYs = [rng.standard_normal((st.s, st.h)) for _ in range(m)]
    st.begin_iteration(m)
    for k in range(m):
        st.set_input(k, Xs[k])
        st.set_upstream_grad(k, dYs[k])
    st.run(stage_order(4, 1, m, "H1"))
    eps = 1e-5
    # input gradient (B)
    for k in range(m):
        for _ in range(12):
            i, j = rng.integers(st.s), rng.integers(st.h)
            Xp = [x.copy() for x in Xs]
            Xm = [x.copy() for x in Xs]
            Xp[k][i, j] += eps
            Xm[k][i, j] -= eps
            fd = (stage_loss(st, st.master, Xp, dYs) - stage_loss(st, st.master, Xm, dYs)) / (2 * eps)
            assert abs(fd - st.dX[k][i, j]) <= 1e-6 * max(1.0, abs(fd))
    # parameter gradients (W, plus the LayerNorm ones produced in B), accumulated over microbatches
    for l in range(st.nl):
        for name in PARAM_ORDER:
            for _ in range(6):
                idx = tuple(rng.integers(n) for n in st.master[l][name].shape)
                Pp = [{k: v.copy() for k, v in P.items()} for P in st.master]
                Pm = [{k: v.copy() for k, v in P.items()} for P in st.master]
                Pp[l][name][idx] += eps
                Pm[l][name][idx] -= eps
                fd = (stage_loss(st, Pp, Xs, dYs) - stage_loss(st, Pm, Xs, dYs)) / (2 * eps)
                got = st.grads[l][name][idx]
                assert abs(fd - got) <= 2e-6 * max(1.0, abs(fd)), (l, name, idx, fd, got)


def test_B_then_W_equals_unsplit_backward():
    rng = np.random.default_rng(6)
    s, h, a, b = 10, 24, 3, 2
    P = make_params(rng, 1, h, 4 * h)[0]
    X = rng.standard_normal((b * s, h))
    dY = rng.standard_normal((b * s, h))
    _, cache = L.layer_forward(X, P, a, s, 1e-5)
    dX, wst, lng = L.layer_backward_input(dY, P, cache)
    gW = L.layer_backward_weight(wst)
    gW.update(lng)
    dX_ref, g_ref = L.layer_backward_unsplit(dY, X, P, a, s, 1e-5)
    np.testing.assert_allclose(dX, dX_ref, rtol=1e-11, atol=1e-12)
    assert set(gW) == set(PARAM_ORDER)
    for k in PARAM_ORDER:
        np.testing.assert_allclose(gW[k], g_ref[k], rtol=1e-11, atol=1e-12, err_msg=k)


def test_W_stash_is_exactly_inputs_and_output_grads_of_the_four_linears():
    # Table 1: W needs 32sbh bytes = (2+2+2+8) sbh of inputs + (6+2+8+2) sbh of output grads at 2 B/element
    rng = np.random.default_rng(7)
    s, h, a = 6, 8, 2
    P = make_params(rng, 1, h, 4 * h)[0]
    X = rng.standard_normal((s, h))
    _, cache = L.layer_forward(X, P, a, s, 1e-5)
    _, wst, _ = L.layer_backward_input(rng.standard_normal((s, h)), P, cache)
    assert sum(v.size for v in wst.values()) * 2 == 32 * s * 1 * h


def test_accumulated_gradient_equals_full_batch_gradient_any_legal_order():
    st, rng = tiny_stage(seed=8, s=6, h=16, a=4)
    m = 5
    Xs = [rng.standard_normal((st.s, st.h)) for _ in range(m)]
    dYs = [rng.standard_normal((st.s, st.h)) for _ in range(m)]

    def run(order):
        st.begin_iteration(m)
        for k in range(m):
            st.set_input(k, Xs[k])
            st.set_upstream_grad(k, dYs[k])
        st.run(order)
        return [{k: v.copy() for k, v in g.items()} for g in st.grads]

    g_h1 = run(stage_order(4, 1, m, "H1"))
    g_h2 = run(stage_order(4, 1, m, "H2"))
    g_flat = run([(PF, k) for k in range(m)] + [(PB, k) for k in range(m)] + [(PW, k) for k in range(m)])
    # any order that issues B_k and W_k in increasing k accumulates in the same order: same bits
    for a_, b_ in ((g_h1, g_h2), (g_h1, g_flat)):
        for l in range(st.nl):
            for k in PARAM_ORDER:
                np.testing.assert_array_equal(a_[l][k], b_[l][k])
    # a legal order with W's shuffled: equal up to fp64 summation order
    g_shuf = run([(PF, k) for k in range(m)] + [(PB, k) for k in reversed(range(m))] + [(PW, k) for k in (3, 0, 4, 1, 2)])
    # the m microbatches as ONE pass over a batch of m sequences (block-diagonal causal attention)
    big = StageOracle(layers=st.nl, hidden=st.h, heads=st.a, ffn=st.ffn, seq=st.s, mb_size=m, params=st.master)
    big.begin_iteration(1)
    big.set_input(0, np.concatenate(Xs, 0))
    big.set_upstream_grad(0, np.concatenate(dYs, 0))
    big.run([(PF, 0), (PB, 0), (PW, 0)])
    for l in range(st.nl):
        for k in PARAM_ORDER:
            np.testing.assert_allclose(g_h1[l][k], big.grads[l][k], rtol=1e-11, atol=1e-12)
            np.testing.assert_allclose(g_shuf[l][k], big.grads[l][k], rtol=1e-11, atol=1e-12)


def test_flop_tally_equals_table_1():
    for (s, b, h, a) in ((16, 1, 32, 4), (8, 3, 64, 8)):
        rng = np.random.default_rng(9)
        params = make_params(rng, 2, h, 4 * h)
        st = StageOracle(layers=2, hidden=h, heads=a, ffn=4 * h, seq=s, mb_size=b, params=params, count_flops=True)
        st.begin_iteration(1)
        st.set_input(0, rng.standard_normal((s * b, h)))
        st.set_upstream_grad(0, rng.standard_normal((s * b, h)))
        st.run([(PF, 0), (PB, 0), (PW, 0)])
        want = L.table1_flops(s, b, h)
        assert st.tally.count == {k: 2 * v for k, v in want.items()}    # 2 layers
        # Sec. 2.3: T_W < T_F < T_B and T_B + T_W = 2 T_F in FLOPs
        assert want["W"] < want["F"] < want["B"] and want["B"] + want["W"] == 2 * want["F"]


def test_dependency_checks():
    st, rng = tiny_stage(seed=10)
    st.begin_iteration(2)
    for k in range(2):
        st.set_input(k, rng.standard_normal((st.s, st.h)))
        st.set_upstream_grad(k, rng.standard_normal((st.s, st.h)))
    with pytest.raises(OrderError):
        st.backward_input(0)
    st.forward(0)
    with pytest.raises(OrderError):
        st.forward(0)
    with pytest.raises(OrderError):
        st.backward_weight(0)
    st.backward_input(0)
    st.backward_weight(0)
    with pytest.raises(OrderError):
        st.backward_weight(0)
    with pytest.raises(OrderError):
        st.forward(2)


def test_bf16_round_matches_torch():
    import torch
    rng = np.random.default_rng(11)
    x = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-20, 20, 20000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 3.3895314e38, np.inf, -np.inf,
                  1e-40, 65280.0, 65408.0], np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = bf16_round(x).astype(np.float32)
    np.testing.assert_array_equal(got.view(np.uint32), want.view(np.uint32))
    assert np.isnan(bf16_round(np.array([np.nan], np.float32))[0])
    # the shared input generator rounds the same way
    from zb_inputs import round_to_bf16
    np.testing.assert_array_equal(round_to_bf16(x).view(np.uint32), want.view(np.uint32))
    assert np.isnan(round_to_bf16(np.array([np.nan], np.float32))[0])
