"""GPU parity at the full shapes of workloads c2..c5, in the launch configuration bench.py
times (full m, the workload's schedule kind, p and stage).

c2 is compared end to end: all 24 microbatches and the 24-microbatch accumulated gradients against the
oracle.  At c3..c5 the fp64 oracle needs ~10 s of host time per microbatch, so it runs on SAMPLED
microbatches: Y_k and dX_k depend only on (X_k, dY_k) and the weights, so any k can be checked alone;
accumulated gradients are checked on a second device iteration that holds exactly the sampled microbatches
(same kernels, same shapes).  The gradients accumulated over ALL m microbatches are checked on 4096 sampled
entries per weight matrix (and 64 per bias) by fp64 dot products over what the device itself kept for W
(the inputs and output gradients of the linears, read between B_k and W_k), whose producers the sampled
microbatches check; and they must be bitwise identical when the passes run in another legal order."""
import math

import numpy as np
import pytest

import zb_inputs
from oracle import optimizer as O
from oracle.schedule import stage_order
from zb_testlib import (TOL, WORST_ELEM, check_delta_theta, check_second_moment, check_tensor, compare_grads, hyper,
                        make_device_stage, make_oracle, rel_fro)

pytestmark = pytest.mark.gpu

# linear -> (stash selector of its input, of its output gradient, weight, bias)
LINEARS = (("wqkv", 0, 4, "bqkv"), ("wo", 1, 5, "bo"), ("w1", 2, 6, "b1"), ("w2", 3, 7, "b2"))
N_PICK = 64   # 64 rows x 64 columns = 4096 entries per weight matrix


def full_m_gradients_from_the_stash(dev, w, order, seed):
    """Runs `order` pass by pass; before every W reads the sampled columns of what B kept for it and adds the
    fp64 products.  Returns {(layer, weight name): (rows, cols, 64x64 fp64 sums)} and the bias column sums."""
    import paper_2401_10241_amd as zb
    rng = np.random.default_rng(seed)
    picks = {}
    for l in range(w.layers):
        for name, _, _, _ in LINEARS:
            kin, nout = zb_inputs.param_shape(w, name)
            picks[(l, name)] = (np.sort(rng.choice(kin, N_PICK, replace=False)),
                                np.sort(rng.choice(nout, N_PICK, replace=False)))
    sums = {key: np.zeros((N_PICK, N_PICK)) for key in picks}
    bias = {key: np.zeros(N_PICK) for key in picks}
    for c, k in order:
        if c == 2:
            for l in range(w.layers):
                for name, s_in, s_dout, _ in LINEARS:
                    rows, cols = picks[(l, name)]
                    a = dev.get_stash_columns(s_in, l, k, rows).astype(np.float64)
                    d = dev.get_stash_columns(s_dout, l, k, cols).astype(np.float64)
                    sums[(l, name)] += a.T @ d
                    bias[(l, name)] += d.sum(axis=0)
        (dev.forward, dev.backward_input, dev.backward_weight)[c](k)
    return picks, sums, bias


PIECE_LIMIT = 1 << 22   # entries of a picked tensor that go through the oracle's Step (the first ones)


class PieceOptimizer:
    """The oracle's AdamW Step on a few tensors of the stage (the first PIECE_LIMIT entries of each).  The step
    is element-wise once the clip coefficient is known, so these entries get exactly what the whole-stage
    oracle would give them (which would shuffle several 7 GB fp64 vectors at these sizes)."""

    def __init__(self, w, params, picks):
        self.w, self.picks = w, picks
        self.state = {}
        for l, name in picks:
            th = np.array(params[l][name].reshape(-1)[:PIECE_LIMIT], np.float64)
            self.state[(l, name)] = O.AdamState(th, np.zeros_like(th), np.zeros_like(th), 0)

    def set_theta(self, groups):
        for (l, name), st in self.state.items():
            st.theta[...] = np.asarray(groups[l][name].reshape(-1)[:PIECE_LIMIT], np.float64)

    def step_and_compare(self, dev, label, grads, coef, theta_before, tol):
        """grads: the oracle's gradients by layer and name; coef: clip coefficient of the step taken."""
        import paper_2401_10241_amd as zb
        worst = 0.0
        for (l, name), st in self.state.items():
            g = np.asarray(grads[l][name].reshape(-1)[:PIECE_LIMIT], np.float64)
            ref_before = st.theta.copy()
            O.adamw_step(st, g * coef if coef < 1.0 else g, hyper(self.w))
            idx = zb.PARAM_INDEX[name]
            th = dev.get_tensor(zb.T_PARAM + idx, l).reshape(-1)[:PIECE_LIMIT]
            if name in ("wqkv", "wo", "w1", "w2", "ln1_g", "ln2_g"):
                check_tensor(f"{label} theta {l} {name}", th, st.theta, tol, "fp32")
            check_tensor(f"{label} m {l} {name}", dev.get_tensor(zb.T_ADAM_M + idx, l).reshape(-1)[:PIECE_LIMIT],
                         st.m, tol, "fp32")
            check_second_moment(f"{label} v {l} {name}", dev.get_tensor(zb.T_ADAM_V + idx, l).reshape(-1)[:PIECE_LIMIT],
                                st.v, tol)
            e = check_delta_theta(f"{label} update {l} {name}",
                                  np.asarray(theta_before[l][name]).reshape(-1)[:PIECE_LIMIT], th,
                                  ref_before, st.theta, st.v, tol)
            worst = max(worst, e)
        return worst


def optimizer_picks(w):
    return ((0, "wo"), (w.layers - 1, "wqkv"), (w.layers // 2, "ln2_g"), (0, "w2"), (w.layers - 1, "b1"))


def sampled_parity(w, sample, with_optimizer=False):
    import paper_2401_10241_amd as zb
    tol = TOL[w.dtype]
    m = w.m
    params = zb_inputs.stage_params(w)
    # the workload's order with its steady-state W passes two at a time needs one more W stash slot
    grouped = zb.order_group_w(zb.schedule_order(w.p, w.stage, m, w.kind), 2)
    pools = tuple(max(a, b) for a, b in zip(zb.schedule_stash_need(w.p, w.stage, m, w.kind), zb.order_stash_need(grouped)))
    dev = make_device_stage(w, m, pools=pools)
    dev.set_params(params)
    # --- full-m iteration in the workload's own order, as bench.py runs it ------------------------------
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
        e1, x1 = check_tensor(f"Y[{k}]", dev.get_tensor(zb.T_OUTPUT_Y, 0, k), orc.Y[k], tol, w.dtype)
        e2, x2 = check_tensor(f"dX[{k}]", dev.get_tensor(zb.T_OUTPUT_DX, 0, k), orc.dX[k], tol, w.dtype)
        worst = max(worst, e1, e2)
        WORST_ELEM[0] = max(WORST_ELEM[0], x1, x2)
        del orc.Y[k], orc.dX[k]
        print(f"[{w.name}] microbatch {k}: Y {e1:.2e} dX {e2:.2e} (entries {max(x1, x2):.2f} x bound)", flush=True)
    if len(sample) == m:
        # every microbatch went through the oracle: the full-m accumulated gradients against it, end to end
        eg = compare_grads(dev, orc, tol)
        print(f"[{w.name}] gradients accumulated over all {m} microbatches: {eg:.2e}", flush=True)
    # --- the same microbatches in another legal order (1F1B: W glued to B, fits the same pools), pass by pass:
    #     gradients must not change in any bit; on the way, the full-m sums are rebuilt from the W stash
    order = zb.schedule_order(w.p, w.stage, m, "1F1B")
    dev.begin_iteration(1, m)
    picks, sums, bias = full_m_gradients_from_the_stash(dev, w, order, seed=w.seed + 17)
    dev.synchronize()
    assert dev.get_tensor(zb.T_FLAT_GRADS).tobytes() == full_grads.tobytes()
    grads = dev.get_group(zb.T_GRAD)
    worst_pick = 0.0
    for (l, name), (rows, cols) in picks.items():
        got = grads[l][name][np.ix_(rows, cols)]
        e = rel_fro(got, sums[(l, name)])
        # fp32 MFMA accumulation over tokens x microbatches against fp64 sums of the same bf16 operands
        assert e <= 1e-3, f"full-m gradient entries of layer {l} {name}: {e:.3e}"
        bname = [b for n, _, _, b in LINEARS if n == name][0]
        eb = rel_fro(grads[l][bname][cols], bias[(l, name)])
        assert eb <= 1e-3, f"full-m bias gradient entries of layer {l} {bname}: {eb:.3e}"
        worst_pick = max(worst_pick, e, eb)
    print(f"[{w.name}] full-m gradients, 4096 entries per matrix from the device's own W stash: {worst_pick:.2e}",
          flush=True)
    # --- and with the W passes of the steady state two per launch (zb_order_group_w): every bit again --------
    if grouped != zb.schedule_order(w.p, w.stage, m, w.kind):
        dev.begin_iteration(3, m)
        dev.run_order(grouped)
        dev.synchronize()
        assert dev.get_tensor(zb.T_FLAT_GRADS).tobytes() == full_grads.tobytes()
        print(f"[{w.name}] W in aligned groups of two: gradients bitwise equal", flush=True)
    if len(sample) == m:
        dev.close()
        return worst
    # --- an iteration holding only the sampled microbatches: accumulated gradients vs the oracle --------
    # The upstream gradients are scaled by a power of two (exact in bf16 and in every rounding on the way, so
    # the oracle's gradients scale by exactly that factor) such that this stage's gradient norm falls below the
    # clipping threshold: the workload's own seeds give a local norm above it, which only ever reaches the
    # outcome DEFERRED_CLIPPED.
    ms = len(sample)
    sq = sum(O.local_state(orc.grads[l][n].reshape(-1))[0] for l in range(w.layers) for n in orc.grads[l])
    scale = 1.0
    if with_optimizer:
        scale = 2.0 ** math.floor(math.log2(0.5 / math.sqrt(sq)))
        assert scale < 1.0
        for l in range(w.layers):
            for n in orc.grads[l]:
                orc.grads[l][n] *= scale
        sq *= scale * scale
    dev.begin_iteration(2, ms)
    for slot, k in enumerate(sample):
        dev.set_tensor(zb.T_INPUT_X, 0, slot, zb_inputs.stage_input(w, 0, k))
        dev.set_tensor(zb.T_INPUT_DY, 0, slot, zb_inputs.upstream_grad(w, 0, k) * np.float32(scale))
    dev.run_schedule(w.p, w.stage, ms, w.kind)
    dev.synchronize()
    eg = compare_grads(dev, orc, tol)
    print(f"[{w.name}] accumulated gradients over {ms} sampled microbatches (x {scale}): {eg:.2e}", flush=True)
    if with_optimizer:
        # Three optimizer calls on these gradients (a call leaves them in place), one per outcome that takes a
        # step, at the workload's full parameter count: the optimistic step confirmed; taken, rolled back and
        # redone clipped; deferred and clipped.
        piece = PieceOptimizer(w, params, optimizer_picks(w))
        for label, prev, rest, want in (("commit", 0.0, 0.1, O.COMMITTED),
                                        ("rollback-reclip", 0.0, 4.0, O.ROLLED_BACK_RECLIPPED),
                                        ("deferred", 9.0, 0.0, O.DEFERRED_CLIPPED)):
            theta_before = dev.get_group(zb.T_PARAM)
            norm = math.sqrt(prev + sq + rest)
            c = O.clip_coef(norm, w.clip)
            rep = dev.optimizer_step_validated(prev, rest)
            assert rep.outcome == want, (label, rep.outcome_name)
            assert rep.stepped_optimistically == (want != O.DEFERRED_CLIPPED)
            assert rep.local_sq == pytest.approx(sq, rel=1e-3)
            assert rep.global_norm == pytest.approx(norm, rel=1e-3)
            assert rep.clip_coef == pytest.approx(c, rel=1e-3)
            eu = piece.step_and_compare(dev, f"[{w.name}] {label}", orc.grads, c, theta_before, tol)
            print(f"[{w.name}] optimizer {rep.outcome_name}: clip {rep.clip_coef:.3e}, update error {eu:.2e}, "
                  f"Algorithm-1 mismatches on rollback {rep.alg1_mismatch_elems}", flush=True)
        assert rep.t == 3
    dev.close()
    return worst


def test_c2_end_to_end_all_microbatches():
    w = zb_inputs.workload("c2")
    sampled_parity(w, list(range(w.m)))


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
        theta_before = dev.get_group(zb.T_PARAM)
        ref_before = [{k: v.copy() for k, v in P.items()} for P in orc.master]
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
            for name in ("wqkv", "wo", "w1", "w2", "ln1_g", "ln2_g"):
                check_tensor(f"iteration {it} theta {l} {name}", got[l][name], orc.master[l][name], tol, "fp32")
            if it != w.nan_iteration:   # the update itself (theta moves by lr, far less than tol * theta)
                for name in orc.master[l]:
                    check_delta_theta(f"iteration {it} update {l} {name}", theta_before[l][name], got[l][name],
                                      ref_before[l][name], orc.master[l][name], orc.adam_v[l][name], tol)
    assert rep.t == w.iterations - 1
    dev.close()
    return outcomes


@pytest.mark.parametrize("force", [False, True])
def test_c5_scenario_scaled_down_full_m(force):
    # c5's schedule (p=32, stage 16, ZB-H2, m=64, 4 iterations, NaN in the third) at hidden 256
    w = zb_inputs.workload("c5").scaled(name="c5_small", hidden=256, heads=2, ffn=1024, seq=128)
    run_c5_scenario(w, force)


def test_c5_scenario_full_shapes_one_microbatch():
    """c5's four iterations (NaN in the third, post-validated AdamW after each) at its full layer shapes and
    parameter count, with m reduced from 64 to 1 so that the oracle's F/B/W (about 10 s per microbatch) and
    its AdamW on five tensors stay within a test's time.  Before every iteration the oracle takes the
    device's current fp32 parameters (its own whole-stage AdamW over 9e8 fp64 parameters would take minutes);
    the update that produced them is checked on the picked tensors of every iteration, update by update."""
    import paper_2401_10241_amd as zb
    w0 = zb_inputs.workload("c5")
    w = w0.scaled(name="c5_m1", m=1)
    params = zb_inputs.stage_params(w)
    dev = make_device_stage(w, 1)
    dev.set_params(params)
    piece = PieceOptimizer(w, params, optimizer_picks(w))
    tol = TOL[w.dtype]
    flats = (zb.T_FLAT_PARAMS, zb.T_FLAT_ADAM_M, zb.T_FLAT_ADAM_V)
    t_want = 0
    for it in range(w.iterations):
        current = dev.get_group(zb.T_PARAM)
        X = zb_inputs.stage_input(w, it, 0)
        dY = zb_inputs.upstream_grad(w, it, 0).copy()
        if it == w.nan_iteration:   # the workload's seeded element (its microbatch index does not exist at m = 1)
            dY.reshape(-1)[zb_inputs.nan_injection(w0, it)[1]] = np.nan
        dev.begin_iteration(it, 1)
        dev.set_tensor(zb.T_INPUT_X, 0, 0, X)
        dev.set_tensor(zb.T_INPUT_DY, 0, 0, dY)
        dev.run_schedule(w.p, w.stage, 1, w.kind)
        before = [dev.get_tensor(x).copy() for x in flats]
        rest = zb_inputs.rest_state(w, it, scale=1e-6)
        rep = dev.optimizer_step_validated(0.0, rest)
        if it == w.nan_iteration:
            assert rep.outcome == O.SKIPPED_LOCAL and rep.t == t_want
            for x, b in zip(flats, before):
                assert dev.get_tensor(x).tobytes() == b.tobytes()
            print(f"[c5 full, m=1] iteration {it}: {rep.outcome_name}, state bit-identical", flush=True)
            continue
        orc = make_oracle(w, current)
        orc.begin_iteration(1)
        orc.set_input(0, X)
        orc.set_upstream_grad(0, dY)
        orc.run(stage_order(w.p, w.stage, 1, w.kind))
        e = compare_grads(dev, orc, tol)
        sq = sum(O.local_state(orc.grads[l][n].reshape(-1))[0] for l in range(w.layers) for n in orc.grads[l])
        norm = math.sqrt(sq + rest)
        c = O.clip_coef(norm, w.clip)
        part_clips = O.clip_coef(math.sqrt(sq), w.clip) < 1.0
        want = O.DEFERRED_CLIPPED if part_clips else (O.ROLLED_BACK_RECLIPPED if c < 1.0 else O.COMMITTED)
        t_want += 1
        assert rep.outcome == want and rep.t == t_want, (it, rep.outcome_name)
        assert rep.local_sq == pytest.approx(sq, rel=1e-3)
        piece.set_theta(current)
        eu = piece.step_and_compare(dev, f"[c5 full, m=1] iteration {it}", orc.grads, c, current, tol)
        print(f"[c5 full, m=1] iteration {it}: {rep.outcome_name}, gradients {e:.2e}, update {eu:.2e}", flush=True)
    assert t_want == w.iterations - 1
    dev.close()


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
