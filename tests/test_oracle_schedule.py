"""Pins for oracle/schedule.py: the paper's memory formulas (Sec. 2.3), the bubble
sizes of its Table 2, the m <= p iteration times of Appendix F and the 36 printed
bubble rates of its Table 5 (tests/golden/bubble_rates.txt)."""
import os
import random

import pytest

from oracle.schedule import (stage_order, check_order, stash_profile, pipeline_cost, bubble_rate,
                             simulate, group_w, F, B, W)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "bubble_rates.txt")


@pytest.mark.parametrize("kind", ["1F1B", "H1", "H2"])
def test_every_pass_once_and_in_dependency_order(kind):
    for p in (1, 2, 4, 7, 16):
        for m in (1, 2, 3, p, 2 * p - 1, 3 * p + 2):
            for sigma in range(p):
                ops = stage_order(p, sigma, m, kind)
                check_order(ops, m)
                # B_k and W_k are issued in increasing k on every stage
                assert [k for c, k in ops if c == B] == list(range(m))
                assert [k for c, k in ops if c == W] == list(range(m))
                assert [k for c, k in ops if c == F] == list(range(m))


def test_1f1b_shape():
    # Sec. 2: each stage does one more warm-up forward than the next; W glued to B
    p, m = 4, 8
    for sigma in range(p):
        ops = stage_order(p, sigma, m, "1F1B")
        first_b = next(n for n, (c, _) in enumerate(ops) if c == B)
        assert first_b == p - sigma
        for n, (c, k) in enumerate(ops):
            if c == B:
                assert ops[n + 1] == (W, k)


def test_peak_activation_memory_formulas():
    # Sec. 2.3: worker i (= sigma+1) peaks at (p-i+1) M_B + (i-1) M_W for ZB-H1 and
    # (2p-2i+1) M_B + (2i-2) M_W for ZB-H2; 1F1B at (p-i+1) M_B
    M_B, M_W = 34.0 + 5 * 1.5, 32.0      # Table 1 with any a*s/h > 0: M_W < M_B
    for p in (2, 4, 8, 16):
        m = 3 * p
        for sigma in range(p):
            i = sigma + 1
            peak, nb, nw, max_b, max_w = stash_profile(stage_order(p, sigma, m, "H1"), M_B, M_W)
            assert peak == (p - i + 1) * M_B + (i - 1) * M_W and (nb, nw) == (p - sigma, sigma)
            # right after a B, before the W that follows it, one more W-stash is alive
            assert (max_b, max_w) == (p - sigma, sigma + 1)
            peak, nb, nw, max_b, max_w = stash_profile(stage_order(p, sigma, m, "H2"), M_B, M_W)
            assert peak == (2 * p - 2 * i + 1) * M_B + (2 * i - 2) * M_W
            assert (nb, nw) == (2 * (p - sigma) - 1, 2 * sigma)
            assert (max_b, max_w) == (2 * (p - sigma) - 1, 2 * sigma + 1)
            peak, *_ = stash_profile(stage_order(p, sigma, m, "1F1B"), M_B, M_W)
            assert peak == (p - i + 1) * M_B
        # Table 2: maximum over workers is p*M_B (H1) and (2p-1)*M_B (H2), at the first worker
        assert max(stash_profile(stage_order(p, s_, m, "H1"), M_B, M_W)[0] for s_ in range(p)) == p * M_B
        assert max(stash_profile(stage_order(p, s_, m, "H2"), M_B, M_W)[0] for s_ in range(p)) == (2 * p - 1) * M_B


def test_bubble_sizes_of_table_2():
    rnd = random.Random(7)
    for _ in range(20):
        p = rnd.choice([2, 4, 6, 8])
        m = rnd.choice([3 * p, 4 * p + 1])
        tf, tb = rnd.uniform(5, 12), rnd.uniform(5, 12)
        tw = rnd.uniform(2, min(tf, tb))
        ideal = m * (tf + tb + tw)
        assert pipeline_cost(p, m, "1F1B", tf, tb, tw) - ideal == pytest.approx((p - 1) * (tf + tb + tw), rel=1e-9)
        assert pipeline_cost(p, m, "H1", tf, tb, tw) - ideal == pytest.approx((p - 1) * (tf + tb - tw), rel=1e-9)
        assert pipeline_cost(p, m, "H2", tf, tb, tw) - ideal == pytest.approx((p - 1) * (tf + tb - 2 * tw), rel=1e-9)
    # identical pass times: ZB-H1's bubble is a third of 1F1B's, ZB-H2's is zero (Sec. 2.1, 2.2)
    assert pipeline_cost(8, 24, "H1", 1, 1, 1) - 72 == pytest.approx((pipeline_cost(8, 24, "1F1B", 1, 1, 1) - 72) / 3)
    assert pipeline_cost(8, 24, "H2", 1, 1, 1) == pytest.approx(72)


def test_small_number_of_microbatches():
    # Appendix F: with m <= p and T_W < T_B, ignoring communication, 1F1B takes
    # (m+p-1)(T_F+T_B+T_W) and a ZB iteration (m+p-1)(T_F+T_B)+T_W
    tf, tb, tw = 10.0, 10.5, 7.0
    for p, m in ((8, 2), (8, 4), (8, 8), (16, 4), (16, 16)):
        assert pipeline_cost(p, m, "1F1B", tf, tb, tw) == pytest.approx((m + p - 1) * (tf + tb + tw))
        assert pipeline_cost(p, m, "H1", tf, tb, tw) == pytest.approx((m + p - 1) * (tf + tb) + tw)
        assert pipeline_cost(p, m, "H2", tf, tb, tw) == pytest.approx((m + p - 1) * (tf + tb) + tw)


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                t = line.split()
                rows.append((t[0], int(t[1]), int(t[2])) + tuple(float(x) for x in t[3:]))
    return rows


def test_golden_file_is_complete():
    assert len(_golden_rows()) == 12


@pytest.mark.parametrize("row", _golden_rows(), ids=lambda r: f"{r[0]}-p{r[1]}-m{r[2]}")
def test_printed_bubble_rates(row):
    _, p, m, tf, tb, tw, tc, r_1f1b, r_h1, r_h2 = row
    for kind, want in (("1F1B", r_1f1b), ("H1", r_h1), ("H2", r_h2)):
        got = bubble_rate(p, m, kind, tf, tb, tw, tc)
        assert f"{got:.4f}" == f"{want:.4f}", (kind, got, want)


def test_cross_stage_dependencies_hold_in_simulation():
    p, m = 4, 9
    orders = [stage_order(p, i, m, "H2") for i in range(p)]
    start, end = simulate(orders, 3.0, 3.5, 2.0, 0.25)
    for i in range(p):
        for k in range(m):
            if i > 0:
                assert start[i][(F, k)] >= end[i - 1][(F, k)] + 0.25 - 1e-12
            if i < p - 1:
                assert start[i][(B, k)] >= end[i + 1][(B, k)] + 0.25 - 1e-12
            assert start[i][(B, k)] >= end[i][(F, k)] and start[i][(W, k)] >= end[i][(B, k)]


# ---- W passes g at a time (Sec. 2: W anywhere after its B; Appendix A regroups W) ------------------------

def _span_cost(orders, tf, tb, tw, tc, tw_next=None):
    start, end = simulate(orders, tf, tb, tw, tc, T_W_next=tw_next)
    return max(max(end[i].values()) - min(start[i].values()) for i in range(len(orders)))


@pytest.mark.parametrize("kind", ["1F1B", "H1", "H2"])
def test_grouped_w_keeps_every_sequence_and_needs_g_minus_1_more_pending_w(kind):
    rng = random.Random(5)
    for _ in range(60):
        p = rng.randint(1, 12)
        m = rng.randint(1, 40)
        sigma = rng.randrange(p)
        g = rng.randint(1, 5)
        ops = stage_order(p, sigma, m, kind)
        out = group_w(ops, g)
        check_order(out, m)
        for c in (F, B, W):   # each kind of pass keeps its own sequence: the gradient sums keep every bit
            assert [k for cc, k in out if cc == c] == [k for cc, k in ops if cc == c]
        # F and B keep their order among themselves as well: what a neighbour receives, it receives in the same order
        assert [(cc, k) for cc, k in out if cc != W] == [(cc, k) for cc, k in ops if cc != W]
        _, _, _, _, max_w0 = stash_profile(ops)
        _, _, _, _, max_w1 = stash_profile(out)
        assert max_w0 <= max_w1 <= max_w0 + g - 1
        if g == 1:
            assert out == ops


def test_grouped_w_by_hand():
    # p = 2, stage 1 (the last), m = 4, ZB-H1: F0 B0 F1 B1 W0 F2 B2 W1 F3 B3 W2 W3
    ops = stage_order(2, 1, 4, "H1")
    assert ops == [(F, 0), (B, 0), (F, 1), (B, 1), (W, 0), (F, 2), (B, 2), (W, 1), (F, 3), (B, 3), (W, 2), (W, 3)]
    # the only  B W F_j B W  with j even is  B1 W0 F2 B2 W1
    assert group_w(ops, 2) == [(F, 0), (B, 0), (F, 1), (B, 1), (F, 2), (B, 2), (W, 0), (W, 1), (F, 3), (B, 3), (W, 2), (W, 3)]
    # groups of three: B W F_j B W F B W needs j % 3 == 0:  B2 W1 F3 B3 W2 is too short, nothing moves
    assert group_w(ops, 3) == ops
    # the middle of a long ZB-H1 order in groups of three
    mid = group_w(stage_order(4, 2, 12, "H1"), 3)
    text = " ".join("FBW"[c] + str(k) for c, k in mid)
    assert text == ("F0 F1 B0 F2 B1 F3 B2 W0 F4 B3 W1 F5 B4 F6 B5 F7 B6 W2 W3 W4 F8 B7 F9 B8 F10 B9 W5 W6 W7 "
                    "F11 B10 W8 B11 W9 W10 W11")


def test_grouped_w_costs_nothing_without_transfer_time():
    """Grouping is keyed on the forward's microbatch, so all stages shift the same forwards and backwards: with
    T_comm = 0 the pipeline is never slower than with the W one by one, whatever the pass times."""
    rng = random.Random(9)
    for _ in range(25):
        p = rng.choice([2, 3, 4, 8, 16])
        m = rng.randint(p, 4 * p + 3)
        g = rng.randint(2, 4)
        tf, tb, tw = (rng.uniform(0.5, 2.0) for _ in range(3))
        for kind in ("H1", "H2"):
            base = [stage_order(p, i, m, kind) for i in range(p)]
            grouped = [group_w(o, g) for o in base]
            assert _span_cost(grouped, tf, tb, tw, 0.0) <= _span_cost(base, tf, tb, tw, 0.0) + 1e-9


def test_shorter_following_w_shortens_the_pipeline():
    p, m = 16, 48
    tf, tb, tw, tc = 2.10, 2.41, 2.44, 0.07
    base = [stage_order(p, i, m, "H1") for i in range(p)]
    c0 = _span_cost(base, tf, tb, tw, tc)
    assert abs(c0 - pipeline_cost(p, m, "H1", tf, tb, tw, tc)) < 1e-9
    for g in (2, 4):
        grouped = [group_w(o, g) for o in base]
        c1 = _span_cost(grouped, tf, tb, tw, tc)
        assert c0 <= c1 <= c0 + m * tc          # with transfer time: at most one T_comm per group
        c2 = _span_cost(grouped, tf, tb, tw, tc, tw_next=0.7 * tw)
        assert c2 < c0                           # following W at 70 % of the time: a shorter iteration
        # T_W_next = T_W is the plain model
        assert abs(_span_cost(grouped, tf, tb, tw, tc, tw_next=tw) - c1) < 1e-12
