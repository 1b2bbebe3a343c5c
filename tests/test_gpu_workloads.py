"""GPU parity at the full shapes of workloads c2..c5, in the launch configuration bench.py
times (full m, the workload's schedule kind, p and stage).

The fp64 oracle needs ~10 s of host time per microbatch at these sizes, so it is run on SAMPLED
microbatches: Y_k and dX_k depend only on (X_k, dY_k) and the weights, so any k can be checked alone.
Accumulated gradients are checked on a second device iteration that holds exactly the sampled
microbatches (same kernels, same shapes), and the full-m gradients by a property that holds at any
size: they are bitwise identical when the same microbatches run in a different legal order."""
import numpy as np
import pytest

import zb_inputs
from oracle import optimizer as O
from oracle.schedule import stage_order
from zb_testlib import TOL, compare_grads, make_device_stage, make_oracle, rel_fro

pytestmark = pytest.mark.gpu


def sampled_parity(w, sample, with_optimizer=False):
    import paper_2401_10241_amd as zb
    tol = TOL[w.dtype]
    m = w.m
    params = zb_inputs.stage_params(w)
    dev = make_device_stage(w, m)
    dev.set_params(params)
    # --- full-m iteration in the workload's own order -------------------------------------------------
    dev.begin_iteration(0, m)
    for k in range(m):
        dev.set_tensor(zb.T_INPUT_X, 0, k, zb_inputs.stage_input(w, 0, k))
        dev.set_tensor(zb.T_INPUT_DY, 0, k, zb_inputs.upstream_grad(w, 0, k))
    assert zb.schedule_order(w.p, w.stage, m, w.kind) == stage_order(w.p, w.stage, m, w.kind)
    dev.run_schedule(w.p, w.stage, m, w.kind)
    dev.synchronize()
    full_grads = dev.get_tensor(zb.T_FLAT_GRADS).copy()
    assert np.isfinite(full_grads).all() and np.abs(full_grads).max() > 0
    orc = make_oracle(w, params)
    orc.begin_iteration(m)
    worst = 0.0
    for k in sample:
        orc.set_input(k, zb_inputs.stage_input(w, 0, k))
        orc.set_upstream_grad(k, zb_inputs.upstream_grad(w, 0, k))
        orc.forward(k)
        orc.backward_input(k)
        orc.backward_weight(k)
        e1 = rel_fro(dev.get_tensor(zb.T_OUTPUT_Y, 0, k), orc.Y[k])
        e2 = rel_fro(dev.get_tensor(zb.T_OUTPUT_DX, 0, k), orc.dX[k])
        assert e1 <= tol and e2 <= tol, (k, e1, e2)
        worst = max(worst, e1, e2)
        print(f"[{w.name}] microbatch {k}: Y {e1:.2e} dX {e2:.2e}", flush=True)
    # --- the same microbatches in another legal order: gradients must not change in any bit --------------
    order = zb.schedule_order(w.p, w.stage, m, "1F1B")   # W glued to B: fits the same stash pools
    dev.begin_iteration(1, m)
    for c, k in order:
        (dev.forward, dev.backward_input, dev.backward_weight)[c](k)
    dev.synchronize()
    assert dev.get_tensor(zb.T_FLAT_GRADS).tobytes() == full_grads.tobytes()
    # --- an iteration holding only the sampled microbatches: accumulated gradients vs the oracle --------
    ms = len(sample)
    dev.begin_iteration(2, ms)
    for slot, k in enumerate(sample):
        dev.set_tensor(zb.T_INPUT_X, 0, slot, zb_inputs.stage_input(w, 0, k))
        dev.set_tensor(zb.T_INPUT_DY, 0, slot, zb_inputs.upstream_grad(w, 0, k))
    dev.run_schedule(w.p, w.stage, ms, w.kind)
    dev.synchronize()
    eg = compare_grads(dev, orc, tol)
    print(f"[{w.name}] accumulated gradients over {ms} sampled microbatches: {eg:.2e}", flush=True)
    if with_optimizer:
        # The oracle's whole-stage optimizer would shuffle several 7 GB fp64 vectors; its pieces are used
        # instead: local state over all gradients, clip coefficient, and Algorithm 1's Step on a few tensors.
        import math
        from zb_testlib import hyper
        rest = zb_inputs.rest_state(w, 0)
        sq = sum(O.local_state(orc.grads[l][n].reshape(-1))[0] for l in range(w.layers) for n in orc.grads[l])
        part_clips = O.clip_coef(math.sqrt(sq), w.clip) < 1.0
        norm = math.sqrt(sq + rest)
        c = O.clip_coef(norm, w.clip)
        want = O.DEFERRED_CLIPPED if part_clips else (O.ROLLED_BACK_RECLIPPED if c < 1.0 else O.COMMITTED)
        rep = dev.optimizer_step_validated(0.0, rest)
        assert rep.outcome == want and rep.t == 1
        assert rep.local_sq == pytest.approx(sq, rel=4e-2)
        assert rep.global_norm == pytest.approx(norm, rel=4e-2)
        assert rep.clip_coef == pytest.approx(c, rel=4e-2)
        for l, name in ((0, "wo"), (w.layers - 1, "wqkv"), (1, "ln2_g"), (0, "w2")):
            st = O.AdamState(orc.master[l][name].reshape(-1).copy(), np.zeros(orc.master[l][name].size),
                             np.zeros(orc.master[l][name].size), 0)
            O.adamw_step(st, orc.grads[l][name].reshape(-1) * c, hyper(w))
            idx = zb.PARAM_INDEX[name]
            assert rel_fro(dev.get_tensor(zb.T_PARAM + idx, l).reshape(-1), st.theta) <= tol
            assert rel_fro(dev.get_tensor(zb.T_ADAM_M + idx, l).reshape(-1), st.m) <= tol
            assert rel_fro(dev.get_tensor(zb.T_ADAM_V + idx, l).reshape(-1), st.v) <= 2 * tol
        print(f"[{w.name}] optimizer outcome {rep.outcome_name}, clip {rep.clip_coef:.3e}", flush=True)
    dev.close()
    return worst


def test_c2_full_shapes():
    w = zb_inputs.workload("c2")
    sampled_parity(w, [0, w.m // 2, w.m - 1])


def test_c3_full_shapes():
    w = zb_inputs.workload("c3")
    sampled_parity(w, [0, w.m - 1])


def test_c4_full_shapes_with_validated_adamw():
    w = zb_inputs.workload("c4")
    sampled_parity(w, [1, w.m - 1], with_optimizer=True)


def test_c5_full_shapes():
    w = zb_inputs.workload("c5")
    sampled_parity(w, [w.m - 1])


def run_c5_scenario(w, force):
    """Four iterations with the post-validated optimizer; the NaN iteration must leave the state
    bit-identical to skipping it, whether the poisoned step is skipped up front or taken and rolled back."""
    import paper_2401_10241_amd as zb
    params = zb_inputs.stage_params(w)
    dev = make_device_stage(w, w.m)
    orc = make_oracle(w, params)
    dev.set_params(params)
    tol = TOL[w.dtype]
    outcomes = []
    for it in range(w.iterations):
        dev.begin_iteration(it, w.m)
        orc.begin_iteration(w.m)
        for k in range(w.m):
            X, dY = zb_inputs.stage_input(w, it, k), zb_inputs.upstream_grad(w, it, k)
            dev.set_tensor(zb.T_INPUT_X, 0, k, X)
            dev.set_tensor(zb.T_INPUT_DY, 0, k, dY)
            orc.set_input(k, X)
            orc.set_upstream_grad(k, dY)
        dev.run_schedule(w.p, w.stage, w.m, w.kind)
        orc.run(stage_order(w.p, w.stage, w.m, w.kind))
        before = [dev.get_tensor(x).copy() for x in (zb.T_FLAT_PARAMS, zb.T_FLAT_ADAM_M, zb.T_FLAT_ADAM_V)]
        rest = zb_inputs.rest_state(w, it, scale=1e-6)
        rep = dev.optimizer_step_validated(0.0, rest, force_optimistic=force)
        ref = orc.optimizer_step(O.GlobalState(0.0, rest, force_optimistic=force))
        outcomes.append(rep.outcome)
        assert rep.outcome == ref.outcome and rep.t == ref.t, (it, rep.outcome_name)
        after = [dev.get_tensor(x) for x in (zb.T_FLAT_PARAMS, zb.T_FLAT_ADAM_M, zb.T_FLAT_ADAM_V)]
        if it == w.nan_iteration:
            assert rep.outcome == (O.ROLLED_BACK_NONFINITE if force else O.SKIPPED_LOCAL)
            assert rep.stepped_optimistically == force
            for a, b in zip(after, before):
                assert a.tobytes() == b.tobytes()
        else:
            assert rep.outcome in (O.COMMITTED, O.DEFERRED_CLIPPED, O.ROLLED_BACK_RECLIPPED)
            assert after[0].tobytes() != before[0].tobytes()
        got = dev.get_group(zb.T_PARAM)
        for l in range(w.layers):
            for name in ("wqkv", "wo", "w1", "w2"):
                assert rel_fro(got[l][name], orc.master[l][name]) <= tol
    assert rep.t == w.iterations - 1
    dev.close()
    return outcomes


@pytest.mark.parametrize("force", [False, True])
def test_c5_scenario_scaled_down_full_m(force):
    # c5's schedule (p=32, stage 16, ZB-H2, m=64, 4 iterations, NaN in the third) at hidden 256
    w = zb_inputs.workload("c5").scaled(name="c5_small", hidden=256, heads=2, ffn=1024, seq=128)
    run_c5_scenario(w, force)


def test_c5_full_shapes_rollback_identity():
    """At c5's full shapes (the oracle's optimizer over 9e8 parameters would take minutes) the property that
    holds at any size is checked on the device alone: an iteration whose gradients hold a NaN leaves theta,
    m, v bit-identical, both when the step is skipped up front and when it is taken and rolled back."""
    import paper_2401_10241_amd as zb
    w = zb_inputs.workload("c5").scaled(name="c5_m1", m=1)
    dev = make_device_stage(w, 1)
    dev.set_params(zb_inputs.stage_params(w))
    flats = (zb.T_FLAT_PARAMS, zb.T_FLAT_ADAM_M, zb.T_FLAT_ADAM_V)
    for it, (nan, force, want) in enumerate([(False, False, None), (True, False, O.SKIPPED_LOCAL),
                                             (True, True, O.ROLLED_BACK_NONFINITE), (False, True, None)]):
        dev.begin_iteration(it, 1)
        dY = zb_inputs.upstream_grad(w, 0, 0).copy()
        if nan:
            dY.reshape(-1)[zb_inputs.nan_injection(zb_inputs.workload("c5"), 2)[1]] = np.nan
        dev.set_tensor(zb.T_INPUT_X, 0, 0, zb_inputs.stage_input(w, 0, 0))
        dev.set_tensor(zb.T_INPUT_DY, 0, 0, dY)
        dev.run_schedule(w.p, w.stage, 1, w.kind)
        before = [dev.get_tensor(x).copy() for x in flats]
        rep = dev.optimizer_step_validated(0.0, 1e-9, force_optimistic=force)
        after = [dev.get_tensor(x) for x in flats]
        print(f"[c5 full] iteration {it}: {rep.outcome_name}, t={rep.t}, "
              f"alg1 mismatches {rep.alg1_mismatch_elems}", flush=True)
        if nan:
            assert rep.outcome == want and rep.stepped_optimistically == force
            for a, b in zip(after, before):
                assert a.tobytes() == b.tobytes()
        else:
            assert rep.outcome in (O.COMMITTED, O.DEFERRED_CLIPPED, O.ROLLED_BACK_RECLIPPED)
            assert after[0].tobytes() != before[0].tobytes()
    assert rep.t == 2
    dev.close()


@pytest.mark.parametrize("name,h,a,ffn,b", [("1.5B-b6", 2304, 24, 9216, 6), ("6.2B-b3", 4096, 32, 16384, 3)])
def test_papers_microbatch_sizes(name, h, a, ffn, b):
    # Sec. 5.1's table runs the 1.5B model with 6 and the 6.2B model with 3 sequences per microbatch
    # (workloads c2 / c3 use 1): one layer, two microbatches of that size, every tensor against the oracle
    from zb_testlib import compare_outputs, load_iteration
    w = zb_inputs.Workload(name, "bf16", 1, h, a, ffn, 1024, b, 8, 4, 2, "H1", seed=41)
    params = zb_inputs.stage_params(w)
    dev = make_device_stage(w, w.m)
    orc = make_oracle(w, params)
    dev.set_params(params)
    dev.begin_iteration(0, w.m)
    orc.begin_iteration(w.m)
    load_iteration(w, 0, w.m, dev, orc)
    dev.run_schedule(w.p, w.stage, w.m, w.kind)
    dev.synchronize()
    orc.run(stage_order(w.p, w.stage, w.m, w.kind))
    e1 = compare_outputs(dev, orc, w.m, TOL["bf16"])
    e2 = compare_grads(dev, orc, TOL["bf16"])
    print(f"[{name}] outputs {e1:.2e} grads {e2:.2e}", flush=True)
    dev.close()
