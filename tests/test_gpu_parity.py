"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.
Tolerances: max relative Frobenius error 1e-4 (fp32), 2e-2 (bf16);
schedule order, rollback and accumulation determinism are bit-exact."""
import numpy as np
import pytest

import zb_inputs
from oracle import optimizer as O
from oracle.schedule import stage_order
from zb_testlib import (TOL, WORST_ELEM, check_delta_theta, check_second_moment, check_tensor, compare_grads, compare_outputs,
                        load_iteration, make_device_stage, make_oracle, rel_fro)
from oracle.stage import PARAM_ORDER

pytestmark = pytest.mark.gpu

W = zb_inputs.Workload


def run_and_compare(w, m=None, mbs_full=None):
    import paper_2401_10241_amd as zb
    m = m or w.m
    params = zb_inputs.stage_params(w)
    dev = make_device_stage(w, m)
    orc = make_oracle(w, params)
    dev.set_params(params)
    dev.begin_iteration(0, m)
    orc.begin_iteration(m)
    load_iteration(w, 0, m, dev, orc)
    dev.run_schedule(w.p, w.stage, m, w.kind)
    dev.synchronize()
    orc.run(stage_order(w.p, w.stage, m, w.kind))
    tol = TOL[w.dtype]
    e1 = compare_outputs(dev, orc, m, tol, mbs_full)
    e2 = compare_grads(dev, orc, tol)
    print(f"[{w.name}] worst rel-fro: outputs {e1:.2e}, grads {e2:.2e} (tol {tol}); largest entry error so far "
          f"{WORST_ELEM[0]:.2f} x the element-wise bound", flush=True)
    dev.close()
    return e1, e2


def test_c1_tiny_fp32_full():
    # workload c1: stage 0 of p=4, ZB-H1, m=8, fp32
    run_and_compare(zb_inputs.workload("c1"))


def test_small_bf16_mfma_shapes():
    # bf16, shapes that are multiples of the MFMA tiles, ZB-H2 order
    w = W("small_bf16", "bf16", 2, 256, 4, 1024, 128, 1, 4, 1, 6, "H2", seed=11)
    run_and_compare(w)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_ragged_shapes_generic_kernels(dtype):
    # nothing is a multiple of a tile: seq 80, hidden 72 (3 heads of 24), ffn 200, two sequences per microbatch
    w = W("ragged", dtype, 2, 72, 3, 200, 80, 2, 3, 1, 4, "H1", seed=5)
    run_and_compare(w)


def test_head_dim_96_and_single_microbatch():
    w = W("d96", "bf16", 1, 192, 2, 768, 64, 1, 2, 0, 1, "H2", seed=6)
    run_and_compare(w)


@pytest.mark.parametrize("d,heads,seq,b", [(128, 2, 256, 1), (96, 2, 256, 1), (64, 4, 384, 2), (128, 1, 512, 1),
                                           (128, 8, 384, 2), (128, 1, 128, 3), (128, 1, 640, 1), (96, 1, 1152, 1),
                                           (128, 2, 2048, 1)])
def test_mfma_attention_shapes(d, heads, seq, b):
    # several query/key tiles per head, diagonal tiles, every supported head size, two sequences per microbatch;
    # (128, 8, 384, 2) has a multiple of 8 heads (backward workgroups ordered per XCD) and an odd number of blocks;
    # then a single row block (each of the forward's two wave groups gets one key tile), 5 and 9 blocks, and 16
    # blocks of 2048 tokens (twice the workloads' sequence: 32 key tiles for the last row block)
    h = d * heads
    w = W(f"attn_d{d}_s{seq}", "bf16", 1, h, heads, 4 * h, seq, b, 2, 0, 2, "H1", seed=40 + d)
    run_and_compare(w)


def test_split_k_gemm_shapes():
    # few output tiles and a long contraction (hidden 2048, ffn 8192, 256 tokens): the N = hidden GEMMs
    # run as K slices plus a fix-up kernel
    w = W("splitk", "bf16", 1, 2048, 16, 8192, 256, 1, 2, 1, 2, "H1", seed=77)
    run_and_compare(w)


def test_tail_split_gemm_shapes():
    # 1024 tokens x ffn 16896: 4 x 66 tiles of 256 x 256, two tile columns more than one round over the 256
    # CUs; those columns run as K slices plus a fix-up kernel writing a column range of the output
    w = W("tailsplit", "bf16", 1, 2048, 16, 16896, 1024, 1, 2, 1, 1, "H1", seed=78)
    run_and_compare(w)


def test_accumulation_is_bitwise_identical_across_orders():
    import paper_2401_10241_amd as zb
    w = W("det", "bf16", 2, 256, 4, 1024, 128, 1, 4, 1, 8, "H1", seed=21)
    params = zb_inputs.stage_params(w)
    dev = make_device_stage(w, 8, pools=(8, 8, 8))
    dev.set_params(params)
    load_iteration(w, 0, 8, dev)
    results = []
    flat = [(0, k) for k in range(8)] + [(1, k) for k in range(8)] + [(2, k) for k in range(8)]
    for order in (zb.schedule_order(4, 1, 8, "H1"), zb.schedule_order(4, 3, 8, "H2"),
                  zb.schedule_order(8, 0, 8, "H2"), zb.schedule_order(4, 2, 8, "1F1B"), flat):
        dev.begin_iteration(0, 8)
        for c, k in order:
            (dev.forward, dev.backward_input, dev.backward_weight)[c](k)
        dev.synchronize()
        results.append((dev.get_tensor(zb.T_FLAT_GRADS).copy(),
                        [dev.get_tensor(zb.T_OUTPUT_DX, 0, k).copy() for k in range(8)]))
    for g, dxs in results[1:]:
        assert g.tobytes() == results[0][0].tobytes()
        for a, b in zip(dxs, results[0][1]):
            assert a.tobytes() == b.tobytes()
    assert np.abs(results[0][0]).max() > 0
    # What the library guarantees bit for bit is the sum taken in increasing microbatch order, which is the
    # order of W in every schedule of the paper (and of B, which carries the LayerNorm gradients).  An order
    # that runs the W passes in another microbatch sequence (legal: W_k only needs B_k) adds the same fp32
    # terms in another order: equal to rounding, not to the bit.
    shuffled = [(0, k) for k in range(8)] + [(1, k) for k in range(8)] + [(2, k) for k in (5, 2, 7, 0, 3, 6, 1, 4)]
    dev.begin_iteration(0, 8)
    dev.run_order(shuffled)
    dev.synchronize()
    g = dev.get_tensor(zb.T_FLAT_GRADS)
    assert rel_fro(g, results[0][0]) < 1e-6
    dev.close()


@pytest.mark.parametrize("shape", [(256, 4, 1024, 128), (72, 3, 200, 80)], ids=["mfma", "generic"])
def test_grouped_w_has_the_bits_of_one_by_one_w(shape):
    # consecutive W passes of an order run as one grouped W: every gradient must keep every bit, whether the
    # grouped MFMA kernel takes the shape (hidden 256) or the group falls back to single launches (hidden 72)
    import paper_2401_10241_amd as zb
    hidden, heads, ffn, seq = shape
    m = 6
    w = W("grp", "bf16", 2, hidden, heads, ffn, seq, 1, 4, 3, m, "H1", seed=23)
    params = zb_inputs.stage_params(w)
    order = zb.schedule_order(4, 3, m, "H1")          # ends in three consecutive W
    assert [c for c, _ in order[-3:]] == [2, 2, 2]
    results = []
    for mode in ("one by one", "run_schedule grouped", "explicit group", "run_schedule, grouping off"):
        dev = make_device_stage(w, m, pools=(m, m, m), **({"group_w": False} if mode.endswith("off") else {}))
        dev.set_params(params)
        dev.begin_iteration(0, m)
        load_iteration(w, 0, m, dev)
        if mode == "one by one":
            for c, k in order:
                (dev.forward, dev.backward_input, dev.backward_weight)[c](k)
        elif mode == "explicit group":
            for k in range(m):
                dev.forward(k)
                dev.backward_input(k)
            dev.backward_weight_group([0, 1])
            dev.backward_weight(2)
            dev.backward_weight_group([3, 4, 5])
            with pytest.raises(zb.ZbError) as e:
                dev.backward_weight_group([1, 2])      # already done
            assert e.value.status == zb.EORDER
        else:
            dev.run_schedule(4, 3, m, "H1")
        dev.synchronize()
        results.append(dev.get_tensor(zb.T_FLAT_GRADS).copy())
        dev.close()
    assert np.abs(results[0]).max() > 0
    for g in results[1:]:
        assert g.tobytes() == results[0].tobytes()


@pytest.mark.parametrize("group", [2, 3])
def test_w_grouped_order_has_the_bits_of_the_plain_order(group):
    # the order with its steady-state W passes `group` at a time (zb_order_group_w) through zb_run_order: the W of
    # a parameter run in the same microbatch sequence, so every gradient and input gradient keeps every bit
    import paper_2401_10241_amd as zb
    m = 12
    w = W("pairw", "bf16", 2, 256, 4, 1024, 128, 1, 4, 1, m, "H1", seed=27)
    params = zb_inputs.stage_params(w)
    plain = zb.schedule_order(w.p, w.stage, m, "H1")
    paired = zb.order_group_w(plain, group)
    assert paired != plain and sorted(paired) == sorted(plain)
    assert sum(1 for i in range(len(paired) - 1) if paired[i][0] == 2 and paired[i + 1][0] == 2) >= 3
    results = []
    for ops in (plain, paired):
        pools = zb.order_stash_need(ops)
        dev = make_device_stage(w, m, pools=pools)
        dev.set_params(params)
        dev.begin_iteration(0, m)
        load_iteration(w, 0, m, dev)
        dev.run_order(ops)
        dev.synchronize()
        results.append((dev.get_tensor(zb.T_FLAT_GRADS).copy(),
                        [dev.get_tensor(zb.T_OUTPUT_DX, 0, k).copy() for k in range(m)]))
        dev.close()
    assert np.abs(results[0][0]).max() > 0
    assert results[0][0].tobytes() == results[1][0].tobytes()
    for a, b in zip(results[0][1], results[1][1]):
        assert a.tobytes() == b.tobytes()
    assert zb.order_stash_need(paired)[1] == zb.order_stash_need(plain)[1] + group - 1


def test_fused_backward_has_the_bits_of_b_then_w():
    # the traditional single backward (layer by layer: input gradient, then that layer's parameter
    # gradients) against B then W of the split, bit for bit, and against the oracle
    import paper_2401_10241_amd as zb
    m = 4
    w = W("fused", "bf16", 3, 256, 4, 1024, 128, 1, 4, 2, m, "H1", seed=29)
    params = zb_inputs.stage_params(w)
    order = zb.schedule_order(4, 2, m, "1F1B")
    results = []
    for mode in ("split", "fused calls", "run_schedule with fuse_bw"):
        dev = make_device_stage(w, m, pools=(m, m, m), **({"fuse_bw": True} if mode.startswith("run") else {}))
        dev.set_params(params)
        dev.begin_iteration(0, m)
        load_iteration(w, 0, m, dev)
        if mode == "split":
            for c, k in order:
                (dev.forward, dev.backward_input, dev.backward_weight)[c](k)
        elif mode == "fused calls":
            for c, k in order:
                if c == 0:
                    dev.forward(k)
                elif c == 1:
                    dev.backward_fused(k)
            with pytest.raises(zb.ZbError) as e:
                dev.backward_weight(0)                  # the fused call did W too
            assert e.value.status == zb.EORDER
        else:
            dev.run_schedule(4, 2, m, "1F1B")
        dev.synchronize()
        results.append((dev.get_tensor(zb.T_FLAT_GRADS).copy(),
                        [dev.get_tensor(zb.T_OUTPUT_DX, 0, k).copy() for k in range(m)]))
        if mode == "fused calls":
            orc = make_oracle(w, params)
            orc.begin_iteration(m)
            load_iteration(w, 0, m, orc=orc)
            orc.run(order)
            compare_outputs(dev, orc, m, TOL["bf16"])
            compare_grads(dev, orc, TOL["bf16"])
        dev.close()
    for g, dxs in results[1:]:
        assert g.tobytes() == results[0][0].tobytes()
        for a, b in zip(dxs, results[0][1]):
            assert a.tobytes() == b.tobytes()


def test_pass_order_is_enforced():
    import paper_2401_10241_amd as zb
    w = W("ord", "fp32", 1, 64, 2, 256, 32, 1, 2, 0, 2, "H1", seed=3)
    dev = make_device_stage(w, 2, pools=(1, 1, 1))
    dev.set_params(zb_inputs.stage_params(w))
    with pytest.raises(zb.ZbError) as e:
        dev.forward(0)
    assert e.value.status == zb.ESTATE          # no iteration begun
    dev.begin_iteration(0, 2)
    load_iteration(w, 0, 2, dev)
    for fn in (dev.backward_input, dev.backward_weight):
        with pytest.raises(zb.ZbError) as e:
            fn(0)
        assert e.value.status == zb.EORDER
    dev.forward(0)
    with pytest.raises(zb.ZbError) as e:
        dev.forward(0)
    assert e.value.status == zb.EORDER
    with pytest.raises(zb.ZbError) as e:
        dev.forward(1)
    assert e.value.status == zb.ENOMEM          # only one pending-B slot
    with pytest.raises(zb.ZbError) as e:
        dev.backward_weight(0)
    assert e.value.status == zb.EORDER
    dev.backward_input(0)
    dev.backward_weight(0)
    with pytest.raises(zb.ZbError) as e:
        dev.forward(2)
    assert e.value.status == zb.EINVAL
    dev.forward(1)
    dev.backward_input(1)
    dev.backward_weight(1)
    dev.synchronize()
    dev.close()


# ---------------------------------------------------------------------------------------------
# optimizer: post-validation outcomes, against the oracle's protocol and its synchronous result
# ---------------------------------------------------------------------------------------------
OPT_CASES = [
    # prev_sq, rest_sq, prev_nf, rest_nf, dY scale, nan, force, outcome
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
]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_post_validated_optimizer_outcomes(dtype):
    import paper_2401_10241_amd as zb
    w = W("opt", dtype, 2, 128, 4, 512, 64, 1, 4, 1, 3, "H1", seed=31, lr=1e-3, clip=1.0)
    m = 3
    params = zb_inputs.stage_params(w)
    dev = make_device_stage(w, m)
    orc = make_oracle(w, params)
    dev.set_params(params)
    tol = TOL[dtype]
    for it, (prev_sq, rest_sq, prev_nf, rest_nf, scale, nan, force, want) in enumerate(OPT_CASES):
        dev.begin_iteration(it, m)
        orc.begin_iteration(m)
        for k in range(m):
            X = zb_inputs.stage_input(w, it, k)
            dY = zb_inputs.upstream_grad(w, it, k) * np.float32(scale)
            if dtype == "bf16":
                dY = zb_inputs.round_to_bf16(dY)
            if nan and k == 1:
                dY = dY.copy()
                dY[5, 7] = np.nan
            dev.set_tensor(zb.T_INPUT_X, 0, k, X)
            dev.set_tensor(zb.T_INPUT_DY, 0, k, dY)
            orc.set_input(k, X)
            orc.set_upstream_grad(k, dY)
        dev.run_schedule(w.p, w.stage, m, w.kind)
        orc.run(stage_order(w.p, w.stage, m, w.kind))
        before = [dev.get_tensor(x).copy() for x in (zb.T_FLAT_PARAMS, zb.T_FLAT_ADAM_M, zb.T_FLAT_ADAM_V)]
        theta_before = dev.get_group(zb.T_PARAM)
        ref_before = [{k: v.copy() for k, v in P.items()} for P in orc.master]
        rep = dev.optimizer_step_validated(prev_sq, rest_sq, prev_nf, rest_nf, force)
        ref = orc.optimizer_step(O.GlobalState(prev_sq, rest_sq, prev_nf, rest_nf, force))
        assert rep.outcome == want == ref.outcome, (it, rep.outcome_name)
        assert rep.t == ref.t and rep.stepped_optimistically == ref.stepped_optimistically
        after = [dev.get_tensor(x) for x in (zb.T_FLAT_PARAMS, zb.T_FLAT_ADAM_M, zb.T_FLAT_ADAM_V)]
        skipped = want in (O.SKIPPED_LOCAL, O.ROLLED_BACK_NONFINITE, O.DEFERRED_SKIPPED)
        if skipped:   # bit-identical to never having stepped
            for a, b in zip(after, before):
                assert a.tobytes() == b.tobytes(), f"case {it}: state changed although the iteration is skipped"
        else:
            assert after[0].tobytes() != before[0].tobytes()
            assert rel_fro(rep.local_sq, ref.local_sq) < (1e-6 if dtype == "fp32" else 5e-2)
            assert rep.global_norm == pytest.approx(ref.global_norm, rel=1e-5 if dtype == "fp32" else 3e-2)
            assert rep.clip_coef == pytest.approx(ref.clip_coef, rel=1e-5 if dtype == "fp32" else 3e-2)
        # state against the oracle's, tensor by tensor: the moments of all 12 tensors, the parameters of those
        # that do not start at zero, and (when a step was taken) the UPDATE of all 12
        groups = {base: dev.get_group(base) for base in (zb.T_PARAM, zb.T_ADAM_M, zb.T_ADAM_V)}
        for l in range(w.layers):
            for name in PARAM_ORDER:
                check_tensor(f"case {it} m {l} {name}", groups[zb.T_ADAM_M][l][name], orc.adam_m[l][name], tol, "fp32")
                check_second_moment(f"case {it} v {l} {name}", groups[zb.T_ADAM_V][l][name], orc.adam_v[l][name], tol)
                # Parameters that start at zero (biases, LayerNorm beta) are left out of the check of theta
                # itself: Adam's first update of such an element is lr times the SIGN of its gradient, so an
                # element whose gradient is smaller than the bf16 rounding noise flips by 2*lr whatever the
                # kernel does.  Their update is checked below on the entries whose gradient is not that small.
                if name in ("wqkv", "wo", "w1", "w2", "ln1_g", "ln2_g"):
                    check_tensor(f"case {it} theta {l} {name}", groups[zb.T_PARAM][l][name], orc.master[l][name], tol,
                                 "fp32")
                if not skipped:
                    check_delta_theta(f"case {it} update {l} {name}", theta_before[l][name],
                                      groups[zb.T_PARAM][l][name], ref_before[l][name], orc.master[l][name],
                                      orc.adam_v[l][name], max(tol, 1e-3))
    dev.close()


def test_rollback_then_redo_equals_direct_clipped_step_bitwise():
    """ROLLED_BACK_RECLIPPED must land on the same bits as DEFERRED_CLIPPED-style single clipped step."""
    import paper_2401_10241_amd as zb
    w = W("opt2", "bf16", 1, 128, 4, 512, 64, 1, 2, 0, 2, "H1", seed=32, lr=1e-3)
    params = zb_inputs.stage_params(w)
    finals = []
    for force in (True, False):
        dev = make_device_stage(w, 2)
        dev.set_params(params)
        dev.begin_iteration(0, 2)
        load_iteration(w, 0, 2, dev)
        dev.run_schedule(w.p, w.stage, 2, w.kind)
        # prev_sq = 9 makes the partial norm exceed the threshold: forced -> step, rollback, redo clipped;
        # not forced -> wait, one clipped step
        rep = dev.optimizer_step_validated(9.0, 0.0, False, False, force)
        assert rep.outcome == (O.ROLLED_BACK_RECLIPPED if force else O.DEFERRED_CLIPPED)
        finals.append([dev.get_tensor(x).copy() for x in (zb.T_FLAT_PARAMS, zb.T_FLAT_ADAM_M, zb.T_FLAT_ADAM_V)])
        if force:
            assert rep.alg1_mismatch_elems >= 0
        dev.close()
    for a, b in zip(*finals):
        assert a.tobytes() == b.tobytes()


def test_algorithm_1_rollback_without_journal_is_close_but_not_exact():
    import paper_2401_10241_amd as zb
    w = W("opt3", "fp32", 1, 128, 4, 512, 64, 1, 2, 0, 2, "H1", seed=33, lr=1e-3, clip=100.0)
    params = zb_inputs.stage_params(w)
    dev = make_device_stage(w, 2, journal=False)
    dev.set_params(params)
    for it in range(2):   # the first iteration commits so that m, v are non-zero
        dev.begin_iteration(it, 2)
        load_iteration(w, it, 2, dev)
        dev.run_schedule(w.p, w.stage, 2, w.kind)
        if it == 0:
            assert dev.optimizer_step_validated().outcome == O.COMMITTED
    before = [dev.get_tensor(x).copy() for x in (zb.T_FLAT_PARAMS, zb.T_FLAT_ADAM_M, zb.T_FLAT_ADAM_V)]
    rep = dev.optimizer_step_validated(0.0, 0.0, False, True, False)   # full state non-finite -> rollback
    assert rep.outcome == O.ROLLED_BACK_NONFINITE and rep.t == 1
    after = [dev.get_tensor(x) for x in (zb.T_FLAT_PARAMS, zb.T_FLAT_ADAM_M, zb.T_FLAT_ADAM_V)]
    assert rel_fro(after[0], before[0]) < 1e-6
    assert rel_fro(after[1], before[1]) < 1e-4
    assert rel_fro(after[2], before[2]) < 1e-4
    dev.close()


SWEEP = [
    # hidden, heads, ffn, seq, b, layers, dtype      which kernels the shape reaches
    (128, 2, 512, 64, 2, 2, "bf16"),      # head size 64, N = 384 / 128 not multiples of 256: generic GEMMs
    (512, 4, 2048, 256, 1, 2, "bf16"),    # head size 128, every GEMM on the MFMA kernel, 256-token tiles
    (768, 12, 3072, 128, 3, 1, "bf16"),   # head size 64, 384 tokens: 128-row tiles only
    (320, 4, 1280, 96, 1, 2, "bf16"),     # head size 80 and 96 tokens: generic attention, mixed GEMMs
    (1024, 8, 4096, 200, 1, 1, "bf16"),   # head size 128 but a ragged sequence: generic attention, 200-token GEMMs
    (384, 4, 1536, 192, 2, 1, "bf16"),    # head size 96
    (256, 2, 1024, 320, 1, 1, "fp32"),    # fp32 arithmetic everywhere
    (2048, 16, 8192, 512, 1, 1, "bf16"),  # split-K shapes with 512 tokens
    (1536, 12, 6144, 256, 1, 1, "bf16"),  # wgrad on 128-row tiles, two workgroups per CU (288 tiles for FC1 / FC2)
]


@pytest.mark.parametrize("cfg", SWEEP, ids=lambda c: "h%d_a%d_f%d_s%d_b%d_L%d_%s" % c)
def test_shape_sweep(cfg):
    hidden, heads, ffn, seq, b, layers, dtype = cfg
    w = W("sweep", dtype, layers, hidden, heads, ffn, seq, b, 4, 1, 3, "H2", seed=101 + hidden + seq)
    run_and_compare(w)
