"""The library's host-side timing model and automatic scheduler against the oracle: identical stage orders
and bit-equal costs (both are plain double arithmetic in the same order).  Needs the built library, no GPU."""
import os
import random

import pytest

import paper_2401_10241_amd as zb
from oracle import autosched as A
from oracle.schedule import check_order, simulate, stage_order

from test_oracle_autosched import ROWS


def oracle_cost(orders, T_F, T_B, T_W, T_comm, fused=False):
    start, end = simulate(orders, T_F, T_B, T_W, T_comm, fused_backward=fused)
    spans = [max(end[i].values()) - min(start[i].values()) for i in range(len(orders))]
    return max(spans), spans


@pytest.mark.parametrize("kind", ["1F1B", "H1", "H2"])
def test_timing_model_matches_oracle_on_handcrafted_orders(kind):
    for r in ROWS[:9]:
        p, m = r["p"], r["m"]
        orders = [stage_order(p, i, m, kind) for i in range(p)]
        cost, rate, spans = zb.simulate_pipeline(orders, r["T_F"], r["T_B"], r["T_W"], r["T_comm"],
                                                 fused_backward=(kind == "1F1B"))
        c, s = oracle_cost(orders, r["T_F"], r["T_B"], r["T_W"], r["T_comm"], fused=(kind == "1F1B"))
        assert cost == c and spans == s
        assert rate == (c - m * (r["T_F"] + r["T_B"] + r["T_W"])) / c


def test_timing_model_rejects_bad_orders():
    good = [stage_order(2, i, 2, "H1") for i in range(2)]
    bad = [list(good[0]), list(good[1])]
    bad[1][0], bad[1][1] = bad[1][1], bad[1][0]          # B before its F
    with pytest.raises(zb.ZbError) as e:
        zb.simulate_pipeline(bad, 1.0, 1.0, 1.0)
    assert e.value.status == zb.EORDER
    # stage 0 wants B0 before F1, stage 1 emits B0 only after B1, which needs F1 of stage 0: a cycle
    dead = [[(0, 0), (1, 0), (0, 1), (1, 1), (2, 0), (2, 1)],
            [(0, 0), (0, 1), (1, 1), (1, 0), (2, 0), (2, 1)]]
    with pytest.raises(zb.ZbError) as e:
        zb.simulate_pipeline(dead, 1.0, 1.0, 1.0)
    assert e.value.status == zb.EORDER
    with pytest.raises(zb.ZbError):
        zb.simulate_pipeline(good, 0.0, 1.0, 1.0)


@pytest.mark.parametrize("r", ROWS, ids=lambda r: f"{r['model']}-p{r['p']}-m{r['m']}")
@pytest.mark.parametrize("mult", [1, 2])
def test_search_matches_oracle_on_the_papers_settings(r, mult):
    p, m = r["p"], r["m"]
    args = (p, m, r["T_F"], r["T_B"], r["T_W"], r["T_comm"], float(mult * p), 1.0, r["ratio"])
    orders, cost, rate, flags = zb.auto_schedule_search(*args)
    o_orders, o_cost, o_flags = A.search(*args)
    assert flags == o_flags
    assert orders == o_orders
    assert cost == o_cost
    assert rate == (o_cost - m * (r["T_F"] + r["T_B"] + r["T_W"])) / o_cost


@pytest.mark.parametrize("r", ROWS, ids=lambda r: f"{r['model']}-p{r['p']}-m{r['m']}")
def test_library_search_against_the_printed_columns_and_zb_h1(r):
    # the library's own search against what the paper prints (Sec. 5.3 table), without the oracle in between:
    # ZB-1p on all twelve rows, ZB-2p on the eleven rows the reading reproduces; and under p M_B it is never
    # worse than the handcrafted ZB-H1 order run through the library's timing model
    p, m = r["p"], r["m"]
    t = (r["T_F"], r["T_B"], r["T_W"], r["T_comm"])
    _, cost1, rate1, _ = zb.auto_schedule_search(p, m, *t, float(p), 1.0, r["ratio"])
    assert round(rate1, 4) == r["zb1p"]
    h1, _, _ = zb.simulate_pipeline([zb.schedule_order(p, i, m, "H1") for i in range(p)], *t)
    assert cost1 <= h1 * (1 + 1e-12)
    _, _, rate2, _ = zb.auto_schedule_search(p, m, *t, float(2 * p), 1.0, r["ratio"])
    if not (r["model"] == "28.3B" and m == 256):
        assert round(rate2, 4) == r["zb2p"]


def test_every_option_matches_oracle_on_random_settings():
    rng = random.Random(11)
    for _ in range(60):
        p, m = rng.randint(1, 10), rng.randint(1, 24)
        T_F, T_B, T_W = (rng.uniform(0.5, 3.0) for _ in range(3))
        T_comm = rng.choice([0.0, rng.uniform(0.0, 0.6)])
        ratio = rng.choice([0.0, 1.0, rng.uniform(0.0, 1.0)])
        limit = rng.uniform(1.0, 2.5 * p)
        for ew, sk in A.OPTION_GRID:
            got = zb.auto_schedule(p, m, T_F, T_B, T_W, T_comm, limit, 1.0, ratio, ew, sk)
            want = A.auto_schedule(p, m, T_F, T_B, T_W, T_comm, limit, 1.0, ratio, ew, sk)
            assert got == want, (p, m, T_F, T_B, T_W, T_comm, ratio, limit, ew, sk)
            for i in range(p):
                assert zb.order_memory_peak(got[i], 1.0, ratio) == A.memory_peak(want[i], 1.0, ratio)


def test_stash_need_of_an_explicit_order():
    for kind in ("1F1B", "H1", "H2"):
        for p, sigma, m in ((4, 1, 8), (8, 4, 24), (16, 8, 48)):
            ops = zb.schedule_order(p, sigma, m, kind)
            assert zb.order_stash_need(ops) == zb.schedule_stash_need(p, sigma, m, kind)
    with pytest.raises(zb.ZbError) as e:
        zb.order_stash_need([(1, 0), (0, 0), (2, 0)])
    assert e.value.status == zb.EORDER


def test_argument_checks():
    with pytest.raises(zb.ZbError) as e:
        zb.auto_schedule(2, 2, 1.0, 1.0, 1.0, 0.0, 0.5, 1.0, 0.5)      # limit below one microbatch
    assert e.value.status == zb.EINVAL
    with pytest.raises(zb.ZbError):
        zb.auto_schedule(2, 2, 1.0, 1.0, 1.0, 0.0, 2.0, 1.0, 1.5)      # M_W above M_B
    with pytest.raises(zb.ZbError):
        zb.auto_schedule(0, 2, 1.0, 1.0, 1.0, 0.0, 2.0, 1.0, 0.5)


@pytest.mark.parametrize("p,m", [(1, 3), (2, 3), (3, 7), (4, 8), (8, 24), (16, 48), (5, 6), (32, 96)])
def test_zbv_orders_and_timing_match_oracle(p, m):
    from oracle import zbv as V
    got = zb.schedule_order_v(p, m)
    o = V.orders_v(p, m)
    assert got == [[(c, ch * m + k) for c, ch, k in ops] for ops in o]
    for times in ((1.0, 1.0, 1.0, 0.0), (1.0, 1.1, 0.8, 0.05)):
        cost, rate, spans = zb.simulate_pipeline_v(got, m, *times)
        start, end = V.simulate_v(o, *times)
        want = [max(end[i].values()) - min(start[i].values()) for i in range(p)]
        assert spans == want and cost == max(want)
        assert rate == (cost - 2 * m * (times[0] + times[1] + times[2])) / cost
    if m >= 2 * p - 1:
        assert zb.simulate_pipeline_v(got, m, 1.0, 1.0, 1.0)[1] == 0.0      # Sec. 6: zero bubble
    for ops in got:                                                        # 2p chunk activations = p M_B
        assert zb.order_memory_peak(ops, 0.5, 0.5) <= p
        assert zb.order_stash_need(ops)[2] <= 2 * p
