"""Per-stage pass orders and the timing model behind the bubble-rate metric
(test infrastructure).

Orders.  The paper defines 1F1B (Sec. 2: warm-up forwards, each stage one more
than the next; then one-forward-one-backward; then the outstanding backwards),
ZB-H1 (Sec. 2.1: 1F1B's shape, but W starts later on later stages so that every
worker holds the same number of in-flight microbatches; peak activation memory
of worker i is (p-i+1) M_B + (i-1) M_W, Sec. 2.3) and ZB-H2 (Sec. 2.2: more
warm-up forwards, W deferred further, parallelogram tail; worker i peaks at
(2p-2i+1) M_B + (2i-2) M_W).  The figures that draw them are not available, so
the order below is the reading that reproduces those memory formulas, the bubble
sizes of Table 2 and the printed bubble rates of Table 5 (see the tests).

For 0-based stage index sigma (the paper's worker i = sigma + 1):
    warm-up forwards  w     = min(p-1-sigma, m)       (1F1B, ZB-H1)
                            = min(2(p-1-sigma), m)    (ZB-H2)
    W deferral        delta = 0 (1F1B), min(sigma, m) (H1), min(2 sigma, m) (H2)
    emit F_0 .. F_{w-1};
    for k = 0 .. m-1:  F_{w+k} if it exists;  B_k;  W_{k-delta} if k >= delta
    emit the remaining W_{m-delta} .. W_{m-1}

Timing (Sec. 5.3 and Appendix G): a pass starts when the previous pass of its
stage has ended and its cross-stage input has arrived: F(i,j) needs F(i-1,j) +
T_comm, B(i,j) needs B(i+1,j) + T_comm.  A stage's span is the end of its last
pass minus the start of its first; cost is the largest span; bubble rate =
(cost - m (T_F + T_B + T_W)) / cost.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

F, B, W = 0, 1, 2
PASS_NAMES = "FBW"
Op = Tuple[int, int]


def _shape(p: int, sigma: int, m: int, kind: str) -> Tuple[int, int]:
    if not (p >= 1 and 0 <= sigma < p and m >= 1):
        raise ValueError("need p >= 1, 0 <= stage < p, m >= 1")
    if kind == "1F1B":
        return min(p - 1 - sigma, m), 0
    if kind == "H1":
        return min(p - 1 - sigma, m), min(sigma, m)
    if kind == "H2":
        return min(2 * (p - 1 - sigma), m), min(2 * sigma, m)
    raise ValueError("kind must be 1F1B, H1 or H2")


def stage_order(p: int, sigma: int, m: int, kind: str) -> List[Op]:
    """Ordered list of (pass, microbatch) executed by stage sigma."""
    w, delta = _shape(p, sigma, m, kind)
    ops: List[Op] = [(F, k) for k in range(w)]
    for k in range(m):
        if w + k < m:
            ops.append((F, w + k))
        ops.append((B, k))
        if k >= delta:
            ops.append((W, k - delta))
    ops.extend((W, k) for k in range(m - delta, m))
    return ops


def format_order(ops: Sequence[Op]) -> str:
    return " ".join(f"{PASS_NAMES[c]}{k}" for c, k in ops)


def check_order(ops: Sequence[Op], m: int) -> None:
    """Every (pass, mb) exactly once and F_k before B_k before W_k (Sec. 2)."""
    pos: Dict[Op, int] = {}
    for n, op in enumerate(ops):
        if op in pos:
            raise AssertionError(f"{op} scheduled twice")
        pos[op] = n
    for k in range(m):
        if not ((F, k) in pos and (B, k) in pos and (W, k) in pos):
            raise AssertionError(f"microbatch {k} incomplete")
        if not (pos[(F, k)] < pos[(B, k)] < pos[(W, k)]):
            raise AssertionError(f"microbatch {k} violates F -> B -> W")
    if len(ops) != 3 * m:
        raise AssertionError("wrong number of passes")


def stash_profile(ops: Sequence[Op], M_B: float = 1.0, M_W: float = 0.0):
    """Walks the memory deltas of Appendix G (F: +M_B, B: M_W - M_B, W: -M_W).

    Returns (peak_bytes, pending_B at that peak, pending_W at that peak,
    max pending_B, max pending_W)."""
    nb = nw = 0
    peak, at = -1.0, (0, 0)
    max_b = max_w = 0
    for c, _ in ops:
        if c == F:
            nb += 1
        elif c == B:
            nb -= 1
            nw += 1
        else:
            nw -= 1
        max_b, max_w = max(max_b, nb), max(max_w, nw)
        mem = nb * M_B + nw * M_W
        if mem > peak:
            peak, at = mem, (nb, nw)
    return peak, at[0], at[1], max_b, max_w


def group_w(ops: Sequence[Op], g: int) -> List[Op]:
    """W passes of the 1F1B-shaped steady state run g at a time (Sec. 2: a W may run anywhere after its B;
    Appendix A regroups W the same way).  Wherever a stage order reads  B W F_j B W F B W ... B W  (g times
    B W, forwards between) with j a multiple of g, the W wait for the last of them:  B F_j B F ... B W W ... W.
    Keyed on the forward's microbatch, every stage groups around the same forwards, so no stage asks a
    neighbour for a tensor earlier than that neighbour, grouping the same way, produces it; at zero transfer
    time the timing model's cost does not grow.  F, B and W each keep their own sequence; at most g - 1 more
    W are pending at any time."""
    if g < 1:
        raise ValueError("group size must be at least 1")
    src, out = list(ops), []
    span = 3 * g - 1
    shape = [(B, W, F)[q % 3] for q in range(span)]
    at = 0
    while at < len(src):
        window = src[at:at + span]
        if g > 1 and [c for c, _ in window] == shape and window[2][1] % g == 0:
            out.extend(op for op in window if op[0] != W)
            out.extend(op for op in window if op[0] == W)
            at += span
        else:
            out.append(src[at])
            at += 1
    return out


def simulate(orders: Sequence[Sequence[Op]], T_F: float, T_B: float, T_W: float,
             T_comm: float = 0.0, fused_backward: bool = False, T_W_next: float = None):
    """Start/end times of every pass of a p-stage pipeline.

    fused_backward=True models the traditional single backward function of 1F1B
    (Sec. 1: B at layer i-1 depends on W at layer i): the input gradient leaves
    the stage only when the W glued to that B has finished.

    T_W_next: duration of a W that directly follows another W on its stage (W passes run side by side share
    the gradient's read and write); None: T_W."""
    p = len(orders)
    dur = {F: T_F, B: T_B, W: T_W}
    end: List[Dict[Op, float]] = [dict() for _ in range(p)]
    start: List[Dict[Op, float]] = [dict() for _ in range(p)]
    ptr = [0] * p
    clock = [0.0] * p
    remaining = sum(len(o) for o in orders)
    while remaining:
        progressed = False
        for i in range(p):
            while ptr[i] < len(orders[i]):
                c, k = orders[i][ptr[i]]
                ready = clock[i]
                if c == F and i > 0:
                    if (F, k) not in end[i - 1]:
                        break
                    ready = max(ready, end[i - 1][(F, k)] + T_comm)
                elif c == B:
                    if i < p - 1:
                        src = (W, k) if fused_backward else (B, k)
                        if src not in end[i + 1]:
                            break
                        ready = max(ready, end[i + 1][src] + T_comm)
                    if (F, k) not in end[i]:
                        raise AssertionError("B before F on one stage")
                elif c == W and (B, k) not in end[i]:
                    raise AssertionError("W before B on one stage")
                start[i][(c, k)] = ready
                follows_w = c == W and T_W_next is not None and ptr[i] > 0 and orders[i][ptr[i] - 1][0] == W
                clock[i] = ready + (T_W_next if follows_w else dur[c])
                end[i][(c, k)] = clock[i]
                ptr[i] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise AssertionError("schedule deadlocks")
    return start, end


def pipeline_cost(p: int, m: int, kind: str, T_F: float, T_B: float, T_W: float,
                  T_comm: float = 0.0) -> float:
    orders = [stage_order(p, i, m, kind) for i in range(p)]
    start, end = simulate(orders, T_F, T_B, T_W, T_comm, fused_backward=(kind == "1F1B"))
    return max(max(end[i].values()) - min(start[i].values()) for i in range(p))


def bubble_rate(p: int, m: int, kind: str, T_F: float, T_B: float, T_W: float,
                T_comm: float = 0.0) -> float:
    cost = pipeline_cost(p, m, kind, T_F, T_B, T_W, T_comm)
    return (cost - m * (T_F + T_B + T_W)) / cost
