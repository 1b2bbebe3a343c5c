"""An automatically searched schedule (Sec. 3.1) run on the device: one stage's row of the library's
search result goes through zb_run_order and is compared with the oracle running the oracle's own search
result; the accumulated gradients are bitwise those of the handcrafted order."""
import numpy as np
import pytest

import zb_inputs
from oracle import autosched as A
from zb_testlib import TOL, compare_grads, compare_outputs, load_iteration, make_device_stage, make_oracle

pytestmark = pytest.mark.gpu
W = zb_inputs.Workload


def test_auto_scheduled_order_runs_and_matches_oracle():
    import paper_2401_10241_amd as zb
    p, sigma, m = 4, 1, 8
    w = W("auto", "bf16", 2, 256, 4, 1024, 128, 1, p, sigma, m, "H1", seed=31)
    times = (1.9, 2.4, 1.3, 0.05)
    orders, cost, rate, flags = zb.auto_schedule_search(p, m, *times, 2.0 * p, 1.0, 0.45)
    o_orders, o_cost, o_flags = A.search(p, m, *times, 2.0 * p, 1.0, 0.45)
    assert orders == o_orders and cost == o_cost and flags == o_flags
    ops = orders[sigma]
    pools = zb.order_stash_need(ops)

    params = zb_inputs.stage_params(w)
    dev = make_device_stage(w, m, pools=pools)
    orc = make_oracle(w, params)
    dev.set_params(params)
    dev.begin_iteration(0, m)
    orc.begin_iteration(m)
    load_iteration(w, 0, m, dev, orc)
    dev.run_order(ops)
    dev.synchronize()
    orc.run(o_orders[sigma])
    compare_outputs(dev, orc, m, TOL["bf16"])
    compare_grads(dev, orc, TOL["bf16"])
    auto_grads = dev.get_tensor(zb.T_FLAT_GRADS).copy()
    dev.close()

    # same inputs in ZB-H1 order: the accumulation order over microbatches is the same, so are the bits
    dev = make_device_stage(w, m)
    dev.set_params(params)
    dev.begin_iteration(0, m)
    load_iteration(w, 0, m, dev)
    dev.run_schedule(p, sigma, m, "H1")
    dev.synchronize()
    assert dev.get_tensor(zb.T_FLAT_GRADS).tobytes() == auto_grads.tobytes()
    dev.close()


def test_run_order_checks_its_argument_and_the_pools():
    import paper_2401_10241_amd as zb
    w = W("autoerr", "fp32", 1, 64, 2, 256, 32, 1, 2, 0, 4, "H1", seed=3)
    dev = make_device_stage(w, 4, pools=(1, 1, 2))
    dev.set_params(zb_inputs.stage_params(w))
    dev.begin_iteration(0, 4)
    load_iteration(w, 0, 4, dev)
    with pytest.raises(zb.ZbError) as e:
        dev.run_order([(0, 0), (1, 0)])                         # not 3m passes
    assert e.value.status == zb.ESTATE
    bad = [(1, 0), (0, 0), (2, 0)] + [(c, k) for k in (1, 2, 3) for c in (0, 1, 2)]
    with pytest.raises(zb.ZbError) as e:
        dev.run_order(bad)                                      # B before F
    assert e.value.status == zb.EORDER
    two_in_flight = [(0, 0), (0, 1)] + [(1, 0), (2, 0), (1, 1), (2, 1)] + [(c, k) for k in (2, 3) for c in (0, 1, 2)]
    with pytest.raises(zb.ZbError) as e:
        dev.run_order(two_in_flight)                            # second F finds no free slot
    assert e.value.status == zb.ENOMEM
    dev.close()
