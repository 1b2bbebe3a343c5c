"""AdamW Step / Rollback and the post-validated optimizer step (test infrastructure).

Step is AdamW with decoupled weight decay and bias-corrected moments (Appendix C,
Algorithm 1): the time stamp advances, the two moments take their exponential
averages of g and g*g, and theta moves by lr * (m' / (sqrt(v') + eps) + lambda *
theta), with m', v' the bias-corrected moments and epsilon added outside the
square root.  Rollback is its arithmetic inverse (same algorithm): theta is
recovered first, from the moments and time stamp the step left behind, then the
moments, then the time stamp.

The protocol follows Sec. 4: the stage receives a partially reduced global
state (squared gradient norm and a non-finite flag of the stages before it),
combines it with its own, takes the optimizer step under the control of that
partial state (skips it when a non-finite value is seen or the partial norm
already exceeds the clipping threshold), later receives the fully reduced
state, validates, and if the step taken was not the legitimate one rolls it
back and redoes it with the full state.

Readings of this build (the paper does not fix them): clip coefficient
c = min(1, clip / (norm + 1e-6)); an iteration whose global state holds a
non-finite value leaves theta, m, v, t untouched; Algorithm 1's Rollback is
only arithmetically (not bitwise) reversible, so `post_validated_step` restores
the pre-step values from a saved copy (an undo journal) and `adamw_rollback`
is kept as the paper's arithmetic inverse to measure how far it drifts.

All functions work on flat numpy arrays in the arrays' own dtype (fp64 by
default in the tests; fp32 to study Algorithm 1's drift).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional

import numpy as np

# outcome codes of a validated step
COMMITTED = 0              # optimistic step taken and confirmed
SKIPPED_LOCAL = 1          # partial state already non-finite: no step, iteration skipped
ROLLED_BACK_NONFINITE = 2  # optimistic step taken, full state non-finite: rolled back, skipped
ROLLED_BACK_RECLIPPED = 3  # optimistic step taken, full norm needs clipping: rolled back, redone clipped
DEFERRED_CLIPPED = 4       # partial norm already above threshold: waited, one clipped step
DEFERRED_SKIPPED = 5       # waited for the full state, which turned out non-finite: skipped
OUTCOME_NAMES = ("COMMITTED", "SKIPPED_LOCAL", "ROLLED_BACK_NONFINITE",
                 "ROLLED_BACK_RECLIPPED", "DEFERRED_CLIPPED", "DEFERRED_SKIPPED")


@dataclass
class Hyper:
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.01
    clip: float = 1.0


@dataclass
class AdamState:
    theta: np.ndarray
    m: np.ndarray
    v: np.ndarray
    t: int = 0

    def copy(self) -> "AdamState":
        return AdamState(self.theta.copy(), self.m.copy(), self.v.copy(), self.t)


def adamw_step(st: AdamState, g: np.ndarray, hp: Hyper) -> None:
    """AdamW step with gradient g, in place (Appendix C, Algorithm 1)."""
    dt = st.theta.dtype.type
    g = g.astype(st.theta.dtype, copy=False)
    st.t = st.t + 1
    with np.errstate(all="ignore"):
        st.m[...] = dt(hp.beta1) * st.m + dt(1.0 - hp.beta1) * g
        st.v[...] = dt(hp.beta2) * st.v + dt(1.0 - hp.beta2) * (g * g)
        m_hat = st.m / dt(1.0 - hp.beta1 ** st.t)
        v_hat = st.v / dt(1.0 - hp.beta2 ** st.t)
        st.theta[...] = st.theta - dt(hp.lr * hp.weight_decay) * st.theta \
            - dt(hp.lr) * m_hat / (np.sqrt(v_hat) + dt(hp.eps))


def adamw_rollback(st: AdamState, g: np.ndarray, hp: Hyper) -> None:
    """The arithmetic inverse of adamw_step for the same g, in place (Appendix C, Algorithm 1)."""
    dt = st.theta.dtype.type
    g = g.astype(st.theta.dtype, copy=False)
    with np.errstate(all="ignore"):
        m_hat = st.m / dt(1.0 - hp.beta1 ** st.t)
        v_hat = st.v / dt(1.0 - hp.beta2 ** st.t)
        st.theta[...] = (st.theta + dt(hp.lr) * m_hat / (np.sqrt(v_hat) + dt(hp.eps))) \
            / dt(1.0 - hp.lr * hp.weight_decay)
        st.m[...] = (st.m - dt(1.0 - hp.beta1) * g) / dt(hp.beta1)
        st.v[...] = (st.v - dt(1.0 - hp.beta2) * (g * g)) / dt(hp.beta2)
    st.t = st.t - 1


def local_state(g: np.ndarray):
    """This stage's contribution to the global state: (sum of squares, non-finite flag)."""
    g64 = g.astype(np.float64, copy=False)
    nonfinite = not bool(np.isfinite(g64).all())
    with np.errstate(all="ignore"):
        sq = float(np.dot(g64, g64))
    return sq, nonfinite


def clip_coef(norm: float, clip: float) -> float:
    return min(1.0, clip / (norm + 1e-6))


@dataclass
class GlobalState:
    prev_sq: float = 0.0          # squared norm reduced over the stages before this one
    rest_sq: float = 0.0          # squared norm of the stages after this one
    prev_nonfinite: bool = False
    rest_nonfinite: bool = False
    force_optimistic: bool = False  # take the optimistic step whatever the partial state says


@dataclass
class StepReport:
    outcome: int
    local_sq: float
    global_norm: float
    clip_coef: float
    t: int
    stepped_optimistically: bool
    alg1_mismatch_elems: int = 0


def synchronous_step(st: AdamState, g: np.ndarray, hp: Hyper, gs: GlobalState) -> StepReport:
    """What a synchronised optimizer does (Sec. 4, 'existing implementations'):
    reduce the global state first, then one step conditioned on it."""
    sq, nf = local_state(g)
    nonfinite = nf or gs.prev_nonfinite or gs.rest_nonfinite
    total = gs.prev_sq + sq + gs.rest_sq
    if nonfinite or not math.isfinite(total):
        return StepReport(SKIPPED_LOCAL, sq, float("nan"), 0.0, st.t, False)
    norm = math.sqrt(total)
    c = clip_coef(norm, hp.clip)
    adamw_step(st, g * st.theta.dtype.type(c) if c < 1.0 else g, hp)
    return StepReport(COMMITTED, sq, norm, c, st.t, False)


def post_validated_step(st: AdamState, g: np.ndarray, hp: Hyper, gs: GlobalState,
                        measure_alg1: bool = False) -> StepReport:
    """Sec. 4: optimistic step on the partial state, validation on the full state,
    rollback and redo when they disagree.  Ends in the same state as synchronous_step."""
    sq, nf = local_state(g)
    # partially reduced state: stages before this one combined with this stage
    part_nf = nf or gs.prev_nonfinite
    part_sq = gs.prev_sq + sq
    part_bad = part_nf or not math.isfinite(part_sq)
    part_clips = (not part_bad) and clip_coef(math.sqrt(part_sq), hp.clip) < 1.0

    stepped = False
    journal: Optional[AdamState] = None
    if gs.force_optimistic or not (part_bad or part_clips):
        journal = st.copy()
        adamw_step(st, g, hp)
        stepped = True

    # fully reduced state arrives (during the next iteration's warm-up in the paper)
    full_nf = part_nf or gs.rest_nonfinite
    full_sq = part_sq + gs.rest_sq
    full_bad = full_nf or not math.isfinite(full_sq)
    mismatch = 0

    def undo():
        nonlocal mismatch
        if measure_alg1:
            trial = st.copy()
            adamw_rollback(trial, g, hp)
            same = (trial.theta.view(np.uint8).reshape(-1, trial.theta.itemsize) ==
                    journal.theta.view(np.uint8).reshape(-1, trial.theta.itemsize)).all(axis=1)
            same &= (trial.m.view(np.uint8).reshape(-1, trial.m.itemsize) ==
                     journal.m.view(np.uint8).reshape(-1, trial.m.itemsize)).all(axis=1)
            same &= (trial.v.view(np.uint8).reshape(-1, trial.v.itemsize) ==
                     journal.v.view(np.uint8).reshape(-1, trial.v.itemsize)).all(axis=1)
            mismatch = int((~same).sum())
        st.theta[...] = journal.theta
        st.m[...] = journal.m
        st.v[...] = journal.v
        st.t = journal.t

    if full_bad:
        if stepped:
            undo()
            out = ROLLED_BACK_NONFINITE
        else:
            out = SKIPPED_LOCAL if part_bad else DEFERRED_SKIPPED
        return StepReport(out, sq, float("nan"), 0.0, st.t, stepped, mismatch)

    norm = math.sqrt(full_sq)
    c = clip_coef(norm, hp.clip)
    if c < 1.0:
        if stepped:
            undo()
            out = ROLLED_BACK_RECLIPPED
        else:
            out = DEFERRED_CLIPPED
        adamw_step(st, g * st.theta.dtype.type(c), hp)
    else:
        assert stepped, "no clipping and finite: the optimistic step must have been taken"
        out = COMMITTED
    return StepReport(out, sq, norm, c, st.t, stepped, mismatch)
