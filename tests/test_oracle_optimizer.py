"""Pins for oracle/optimizer.py: closed forms for one element, torch's own AdamW
(a library routine written by others), exact reversibility in rational arithmetic
for Algorithm 1, and the equivalence of the post-validated protocol with the
synchronised optimizer it replaces (Sec. 4)."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import optimizer as O


def state(n, seed=0, dtype=np.float64):
    rng = np.random.default_rng(seed)
    return O.AdamState(rng.standard_normal(n).astype(dtype), np.zeros(n, dtype), np.zeros(n, dtype), 0), rng


def bits_equal(a, b):
    return a.tobytes() == b.tobytes()


def test_first_step_closed_form():
    # lambda = 0, t = 1: m' = g, v' = g^2, so theta_1 = theta_0 - lr * g / (|g| + eps)
    hp = O.Hyper(lr=1e-2, weight_decay=0.0, eps=1e-8)
    st = O.AdamState(np.array([0.5, -1.0, 2.0]), np.zeros(3), np.zeros(3), 0)
    g = np.array([3.0, -0.25, 1e-3])
    O.adamw_step(st, g, hp)
    np.testing.assert_allclose(st.theta, np.array([0.5, -1.0, 2.0]) - 1e-2 * g / (np.abs(g) + 1e-8), rtol=1e-14)
    np.testing.assert_allclose(st.m, 0.1 * g, rtol=1e-15)
    np.testing.assert_allclose(st.v, 0.05 * g * g, rtol=1e-14)
    assert st.t == 1
    # decay only: g = 0 leaves theta * (1 - lr*lambda)
    hp = O.Hyper(lr=1e-2, weight_decay=0.1)
    st = O.AdamState(np.array([2.0]), np.zeros(1), np.zeros(1), 0)
    O.adamw_step(st, np.zeros(1), hp)
    np.testing.assert_allclose(st.theta, 2.0 * (1 - 1e-3), rtol=1e-15)


def test_matches_torch_adamw_over_several_steps():
    import torch
    hp = O.Hyper(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.01)
    st, rng = state(257, seed=1)
    p = torch.nn.Parameter(torch.tensor(st.theta.copy(), dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=hp.lr, betas=(hp.beta1, hp.beta2), eps=hp.eps, weight_decay=hp.weight_decay)
    for _ in range(5):
        g = rng.standard_normal(257)
        O.adamw_step(st, g, hp)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
    np.testing.assert_allclose(st.theta, p.detach().numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(st.m, opt.state[p]["exp_avg"].numpy(), rtol=1e-13)
    np.testing.assert_allclose(st.v, opt.state[p]["exp_avg_sq"].numpy(), rtol=1e-13)


def test_algorithm_1_is_exactly_reversible_in_rational_arithmetic():
    # Appendix C's claim, checked with exact fractions on the update's rational parts:
    # rollback of m, v; and theta given the same (irrational) denominator value
    b1, b2, lr, lam = Fraction(9, 10), Fraction(19, 20), Fraction(1, 1000), Fraction(1, 100)
    m0, v0, th0, g = Fraction(3, 7), Fraction(5, 11), Fraction(-2, 3), Fraction(13, 17)
    m1 = b1 * m0 + (1 - b1) * g
    v1 = b2 * v0 + (1 - b2) * g * g
    denom = Fraction(math.sqrt(float(v1 / (1 - b2 ** 4)))) + Fraction(1, 10 ** 8)
    upd = lr * (m1 / (1 - b1 ** 4)) / denom
    th1 = th0 - lr * lam * th0 - upd
    assert (th1 + upd) / (1 - lr * lam) == th0
    assert (m1 - (1 - b1) * g) / b1 == m0
    assert (v1 - (1 - b2) * g * g) / b2 == v0


def test_rollback_inverts_step_to_rounding_in_fp64_and_restores_t():
    hp = O.Hyper(lr=1e-3, weight_decay=0.01)
    st, rng = state(1000, seed=2)
    for _ in range(3):
        O.adamw_step(st, rng.standard_normal(1000), hp)
    before = st.copy()
    g = rng.standard_normal(1000)
    O.adamw_step(st, g, hp)
    assert st.t == 4 and not bits_equal(st.theta, before.theta)
    O.adamw_rollback(st, g, hp)
    assert st.t == 3
    np.testing.assert_allclose(st.theta, before.theta, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(st.m, before.m, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(st.v, before.v, rtol=1e-12, atol=1e-15)


def test_algorithm_1_is_not_bit_reversible_in_fp32():
    # why a saved copy is needed for a bit-identical rollback
    hp = O.Hyper(lr=1e-3, weight_decay=0.01)
    st, rng = state(4096, seed=3, dtype=np.float32)
    O.adamw_step(st, rng.standard_normal(4096).astype(np.float32), hp)
    before = st.copy()
    g = (rng.standard_normal(4096) * 50).astype(np.float32)
    O.adamw_step(st, g, hp)
    O.adamw_rollback(st, g, hp)
    np.testing.assert_allclose(st.theta, before.theta, rtol=1e-5, atol=1e-6)
    assert not bits_equal(st.m, before.m)


CASES = [
    # (prev_sq, rest_sq, prev_nf, rest_nf, grad scale, nan in g, force, expected outcome)
    (0.0, 0.0, False, False, 1e-3, False, False, O.COMMITTED),
    (0.0, 4.0, False, False, 1e-3, False, False, O.ROLLED_BACK_RECLIPPED),
    (0.0, 0.0, False, True, 1e-3, False, False, O.ROLLED_BACK_NONFINITE),
    (0.0, float("inf"), False, False, 1e-3, False, False, O.ROLLED_BACK_NONFINITE),
    (9.0, 0.0, False, False, 1e-3, False, False, O.DEFERRED_CLIPPED),
    (0.0, 0.0, False, False, 1.0, False, False, O.DEFERRED_CLIPPED),
    (9.0, 0.0, False, True, 1e-3, False, False, O.DEFERRED_SKIPPED),
    (0.0, 0.0, True, False, 1e-3, False, False, O.SKIPPED_LOCAL),
    (0.0, 0.0, False, False, 1e-3, True, False, O.SKIPPED_LOCAL),
    (0.0, 0.0, False, False, 1e-3, True, True, O.ROLLED_BACK_NONFINITE),
    (9.0, 0.0, False, False, 1e-3, False, True, O.ROLLED_BACK_RECLIPPED),
    (0.0, 0.0, False, False, 1e-3, False, True, O.COMMITTED),
]


@pytest.mark.parametrize("case", CASES, ids=[f"{i}-{O.OUTCOME_NAMES[c[-1]]}" for i, c in enumerate(CASES)])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_post_validation_reaches_the_synchronous_result_bitwise(case, dtype):
    prev_sq, rest_sq, prev_nf, rest_nf, gscale, nan_in_g, force, want = case
    hp = O.Hyper(lr=1e-3, weight_decay=0.01, clip=1.0)
    a, rng = state(512, seed=4, dtype=dtype)
    for _ in range(2):
        O.adamw_step(a, rng.standard_normal(512).astype(dtype), hp)
    b = a.copy()
    start = a.copy()
    g = (rng.standard_normal(512) * gscale).astype(dtype)
    if nan_in_g:
        g[17] = np.nan
    gs = O.GlobalState(prev_sq, rest_sq, prev_nf, rest_nf, force)
    rep = O.post_validated_step(a, g, hp, gs, measure_alg1=True)
    ref = O.synchronous_step(b, g, hp, gs)
    assert rep.outcome == want
    assert bits_equal(a.theta, b.theta) and bits_equal(a.m, b.m) and bits_equal(a.v, b.v) and a.t == b.t
    skipped = want in (O.SKIPPED_LOCAL, O.ROLLED_BACK_NONFINITE, O.DEFERRED_SKIPPED)
    if skipped:   # bit-identical to never having stepped, t unchanged
        assert bits_equal(a.theta, start.theta) and bits_equal(a.m, start.m) and bits_equal(a.v, start.v)
        assert a.t == start.t
    else:
        assert a.t == start.t + 1
        assert rep.global_norm == pytest.approx(ref.global_norm) and rep.clip_coef == pytest.approx(ref.clip_coef)
        if want in (O.ROLLED_BACK_RECLIPPED, O.DEFERRED_CLIPPED):
            assert rep.clip_coef < 1.0


def test_clip_coefficient_and_norm():
    assert O.clip_coef(0.5, 1.0) == 1.0
    assert O.clip_coef(2.0, 1.0) == pytest.approx(1.0 / (2.0 + 1e-6))
    g = np.array([3.0, 4.0])
    assert O.local_state(g) == (25.0, False)
    assert O.local_state(np.array([1.0, np.inf]))[1] is True
    assert O.local_state(np.array([1.0, np.nan]))[1] is True
    # clipped step = step with the scaled gradient
    hp = O.Hyper(clip=1.0, weight_decay=0.0)
    a, _ = state(2, seed=5)
    b = a.copy()
    O.synchronous_step(a, g, hp, O.GlobalState())
    O.adamw_step(b, g * O.clip_coef(5.0, 1.0), hp)
    assert bits_equal(a.theta, b.theta)
