"""Pins of the oracle's ZB-V schedule (oracle/zbv.py) against what Sec. 6 states: the V-shaped chain of
dependencies, the warm-up counts, the steady pattern, zero bubble for equal pass times and the peak
activation memory p M_B on every worker."""
import pytest

from oracle import zbv as V
from oracle.schedule import B, F, W, stage_order, stash_profile


@pytest.mark.parametrize("p,m", [(1, 3), (2, 3), (3, 7), (4, 8), (4, 12), (8, 24), (16, 48), (5, 6)])
def test_orders_are_valid_and_complete(p, m):
    orders = V.orders_v(p, m)
    assert len(orders) == p
    for ops in orders:
        V.check_order_v(ops, m)
        for ch in (0, 1):      # all passes of one chunk in microbatch order
            for c in (F, B, W):
                assert [k for cc, hh, k in ops if cc == c and hh == ch] == list(range(m))
    V.simulate_v(orders, 1.0, 1.0, 1.0)     # no deadlock


def test_first_microbatch_walks_the_v():
    # Sec. 6: chunks are laid out worker 1..p and back p..1; forward and backward both start on worker 1
    p, m = 4, 8
    start, end = V.simulate_v(V.orders_v(p, m), 1.0, 1.0, 1.0)
    chain = [(i, (F, 0, 0)) for i in range(p)] + [(i, (F, 1, 0)) for i in reversed(range(p))] \
        + [(i, (B, 1, 0)) for i in range(p)] + [(i, (B, 0, 0)) for i in reversed(range(p))]
    times = [start[i][op] for i, op in chain]
    assert times == sorted(times) and len(set(times)) == len(times)
    assert chain[0][0] == 0 and chain[2 * p][0] == 0          # forward and backward originate on worker 1
    assert times[2 * p] == end[0][(F, 1, 0)]                  # the loss follows chunk 1 of worker 1 directly


@pytest.mark.parametrize("p,m", [(4, 8), (8, 24), (6, 11)])
def test_warm_up_counts_and_steady_pattern(p, m):
    # warm-up: 2p-1 forwards, 2p-i of chunk 0 and i-1 of chunk 1; then p-i groups F-B-W of chunk 1, then
    # groups of chunk 1 and chunk 0 in turn
    orders = V.orders_v(p, m)
    for sigma, ops in enumerate(orders):
        i = sigma + 1
        first_b = next(q for q, op in enumerate(ops) if op[0] == B)
        head = ops[:first_b - 1]           # the forward just before the first B opens the first group
        assert all(op[0] == F for op in ops[:first_b])
        assert len(head) == 2 * p - 1
        assert sum(1 for op in head if op[1] == 0) == 2 * p - i
        assert sum(1 for op in head if op[1] == 1) == i - 1
        groups = []
        q = first_b - 1
        while q + 2 < len(ops) and ops[q][0] == F and ops[q + 1][0] == B and ops[q + 2][0] == W:
            assert ops[q][1] == ops[q + 1][1] == ops[q + 2][1]
            groups.append(ops[q][1])
            q += 3
        want = [1] * (p - i) + [1, 0] * m
        assert len(groups) >= min(p - i + 2, 2)
        # the pattern holds while both chunks still have forwards left
        both_left = 0
        nf = [2 * p - i, i - 1]
        for ch in groups:
            if nf[0] >= m or nf[1] >= m:
                break
            nf[ch] += 1
            both_left += 1
        assert groups[:both_left] == want[:both_left]


@pytest.mark.parametrize("p,m", [(2, 3), (3, 5), (4, 8), (4, 12), (8, 24), (8, 15), (16, 48), (16, 31)])
def test_zero_bubble_for_equal_pass_times(p, m):
    # Sec. 6: with T_F = T_B = T_W (and enough microbatches, m >= 2p-1) ZB-V has no bubble
    orders = V.orders_v(p, m)
    start, end = V.simulate_v(orders, 1.0, 1.0, 1.0, 0.0)
    for i in range(p):
        assert max(end[i].values()) - min(start[i].values()) == 6.0 * m
    assert V.cost_v(orders, 2.5, 2.5, 2.5) == 6 * m * 2.5


@pytest.mark.parametrize("p,m", [(4, 8), (8, 24), (16, 48)])
def test_peak_memory_is_p_mb_on_every_worker(p, m):
    # Sec. 6: peak activation memory p M_B, the same on all workers (a chunk holds M_B / 2), against
    # (2p-1) M_B on the first worker of ZB-H2 and p M_B on the first worker of 1F1B
    orders = V.orders_v(p, m)
    for ops in orders:
        assert V.memory_peak_v(ops, 0.5, 0.5) == p * 1.0       # even if W kept as much as B (M_W = M_B)
        assert V.memory_peak_v(ops, 0.5, 0.0) <= p * 1.0
    assert stash_profile(stage_order(p, 0, m, "H2"), 1.0, 1.0)[0] == 2 * p - 1
    assert stash_profile(stage_order(p, 0, m, "1F1B"), 1.0, 1.0)[0] == p


def test_too_few_microbatches_still_valid():
    # below 2p-1 microbatches the schedule has bubbles but stays a legal schedule
    p, m = 5, 6
    orders = V.orders_v(p, m)
    assert V.cost_v(orders, 1.0, 1.0, 1.0) > 6 * m


def test_unequal_times_and_communication_only_stretch_it():
    p, m = 4, 12
    orders = V.orders_v(p, m)
    base = V.cost_v(orders, 1.0, 1.0, 1.0)
    assert V.cost_v(orders, 1.0, 1.0, 1.0, 0.1) > base
    c = V.cost_v(orders, 1.0, 1.1, 0.8)
    assert c >= m * 2 * (1.0 + 1.1 + 0.8) - 1e-9
