"""CPU-side checks of the boundary: the C-ABI library loads, exports every symbol the header
declares, and its host-only entry points (schedule order, stash need, configuration checks)
agree with the oracle.  No GPU compute is called."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "zb_stage.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zb_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2401_10241_amd as zb
    names = header_symbols()
    assert len(names) >= 20
    for n in names:
        assert hasattr(zb.lib, n), f"{n} declared in zb_stage.h but not exported"
    assert set(zb.binding.EXPORTED) == set(names)


def test_schedule_order_is_bit_exact_with_oracle():
    import paper_2401_10241_amd as zb
    from oracle.schedule import stage_order, stash_profile
    for kind in ("1F1B", "H1", "H2"):
        for p in (1, 2, 3, 4, 8, 16, 32):
            for m in (1, 2, p, 2 * p - 1, 3 * p, 64):
                for sigma in sorted({0, p // 2, p - 1}):
                    want = stage_order(p, sigma, m, kind)
                    assert zb.schedule_order(p, sigma, m, kind) == want
                    _, _, _, max_b, max_w = stash_profile(want)
                    pb, pw, fl = zb.schedule_stash_need(p, sigma, m, kind)
                    assert (pb, pw) == (max_b, max_w) and max(pb, pw) <= fl <= pb + pw


def test_the_five_workload_orders():
    import paper_2401_10241_amd as zb
    import zb_inputs
    from oracle.schedule import stage_order
    for w in zb_inputs.WORKLOADS.values():
        ops = zb.schedule_order(w.p, w.stage, w.m, w.kind)
        assert ops == stage_order(w.p, w.stage, w.m, w.kind) and len(ops) == 3 * w.m


def test_bad_arguments_are_rejected_on_the_host():
    import paper_2401_10241_amd as zb
    n = C.c_int32(0)
    buf = (zb.binding.zb_op * 8)()
    assert zb.lib.zb_schedule_order(4, 4, 2, 1, buf, 8, C.byref(n)) == zb.EINVAL     # stage >= p
    assert zb.lib.zb_schedule_order(4, 0, 2, 7, buf, 8, C.byref(n)) == zb.EINVAL     # unknown kind
    assert zb.lib.zb_schedule_order(4, 0, 4, 1, buf, 8, C.byref(n)) == zb.EINVAL     # capacity too small
    assert n.value == 12
    cfg = zb.binding.zb_config()
    zb.lib.zb_config_defaults(C.byref(cfg))
    need = C.c_size_t(0)
    assert zb.lib.zb_stage_arena_bytes(C.byref(cfg), C.byref(need)) == zb.EINVAL     # shapes unset
    cfg.layers, cfg.hidden, cfg.heads, cfg.ffn, cfg.seq = 3, 5120, 40, 20480, 1024
    cfg.max_microbatches, cfg.max_pending_b, cfg.max_pending_w, cfg.max_inflight = 48, 8, 9, 16
    assert zb.lib.zb_stage_arena_bytes(C.byref(cfg), C.byref(need)) == zb.OK
    assert 30e9 < need.value < 120e9
    cfg.heads = 7
    assert zb.lib.zb_stage_arena_bytes(C.byref(cfg), C.byref(need)) == zb.EINVAL     # hidden % heads
    h = C.c_void_p(None)
    cfg.heads = 40
    assert zb.lib.zb_stage_init(C.byref(cfg), C.byref(h)) == zb.EINVAL and not h.value  # no arena


def test_stage_refuses_to_run_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    import paper_2401_10241_amd as zb
    with pytest.raises(RuntimeError):
        zb.Stage(layers=1, hidden=64, heads=1, ffn=256, seq=16, max_microbatches=1, max_pending_b=1,
                 max_pending_w=1, max_inflight=1)


def test_order_group_w_and_the_w_run_timing_model_match_the_oracle():
    import ctypes
    import random
    import paper_2401_10241_amd as zb
    from oracle.schedule import check_order, group_w, simulate, stage_order, stash_profile
    rng = random.Random(12)
    for kind in ("1F1B", "H1", "H2"):
        for p, m in ((4, 8), (16, 48), (8, 5), (3, 2), (32, 64)):
            base = [zb.schedule_order(p, i, m, kind) for i in range(p)]
            assert [zb.order_group_w(o, 1) for o in base] == base
            for group in (2, 3, 4, 64):
                grouped = [zb.order_group_w(o, group) for o in base]
                assert grouped == [group_w(stage_order(p, i, m, kind), group) for i in range(p)]   # the oracle's rule, bit for bit
                for o, b in zip(grouped, base):
                    check_order(o, m)                                              # F_k before B_k before W_k, each once
                    assert [op for op in o if op[0] != 2] == [op for op in b if op[0] != 2]   # F and B keep their sequence
                    assert [k for c, k in o if c == 2] == [k for c, k in b if c == 2]         # W in their sequence
                    assert stash_profile(o)[4] <= stash_profile(b)[4] + group - 1
                if kind == "1F1B" or group > 4:
                    continue
                tf, tb, tw = (rng.uniform(0.5, 2.0) for _ in range(3))
                tc = 0.05
                for tw_next in (tw, 0.6 * tw, 0.0):
                    cost, spans = zb.simulate_pipeline_w_runs(grouped, tf, tb, tw, tc, tw_next)
                    start, end = simulate(grouped, tf, tb, tw, tc, T_W_next=tw_next)
                    want = [max(end[i].values()) - min(start[i].values()) for i in range(p)]
                    assert max(abs(a - b) for a, b in zip(spans, want)) < 1e-9 and abs(cost - max(want)) < 1e-9
                # with t_w_next = t_w it is zb_simulate_pipeline's model
                c0, _, _ = zb.simulate_pipeline(grouped, tf, tb, tw, tc)
                assert abs(c0 - zb.simulate_pipeline_w_runs(grouped, tf, tb, tw, tc, tw)[0]) < 1e-12
    # the c4 stage: its steady state gives 16 runs of two W, the tail one longer run
    o = zb.order_group_w(zb.schedule_order(16, 8, 48, "H1"), 2)
    assert sum(1 for i in range(len(o) - 1) if o[i][0] == 2 and o[i + 1][0] == 2 and (i == 0 or o[i - 1][0] != 2)) == 17
    buf = (zb.binding.zb_op * 4)()
    assert zb.lib.zb_order_group_w(buf, 3, 0, buf) == zb.EINVAL
    assert zb.lib.zb_order_group_w(None, 3, 2, buf) == zb.EINVAL
    t = zb.binding.zb_pass_times(1.0, 1.0, 1.0, 0.0)
    assert zb.lib.zb_simulate_pipeline_w_runs(1, 1, buf, ctypes.byref(t), -1.0, None, None) == zb.EINVAL


def test_bench_refuses_more_than_one_gpu():
    """One GPU is all this build covers: bench.py --gpus 2 must say so and exit without touching a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
