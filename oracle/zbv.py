"""ZB-V, the two-chunk schedule of Sec. 6 (test infrastructure).

Every worker holds two model chunks; chunk 0 of worker 1..p followed by chunk 1 of worker
p..1 makes the model (the "V").  For a microbatch the forward runs F(0) on workers 1..p, then
F(1) on workers p..1; the backward runs B(1) on workers 1..p, then B(0) on workers p..1; W(c)
may run anywhere after B(c) on the same worker.  An op is (pass, chunk, microbatch).

Order (Sec. 6, third paragraph; the figure that draws it is not available).  Worker i
(1-based), all passes of one chunk in microbatch order:
  1. warm-up: 2p-1 forwards, 2p-i of chunk 0 and i-1 of chunk 1: first 2(p-i)+1 of chunk 0
     (chunk 1 of the first microbatch cannot arrive earlier), then chunk 1 and chunk 0 in turn;
  2. steady phase: groups F-B-W of one chunk: p-i groups of chunk 1, then one group of chunk 1
     and one of chunk 0 in turn, until every forward has run;
  3. final phase: the remaining B and W, "B prioritised, W filling the bubbles".  The order
     of this phase is the one a pipeline with T_F = T_B = T_W and no communication time
     produces when every worker, whenever it is free, runs a B that is ready (chunk 0's first
     if both are: it is the one the earlier workers are waiting for), else its oldest pending
     W.  With that reading every worker is busy from its first to its last pass when
     m >= 2p-1 (zero bubble) and holds at most 2p chunk activations = p M_B (tests).
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

from .schedule import F, B, W

OpV = Tuple[int, int, int]   # (pass, chunk, microbatch)


def producer(p: int, i: int, op: OpV) -> Optional[Tuple[int, OpV, bool]]:
    """(worker, op, crosses a link) whose end the 0-based worker i must wait for before op."""
    c, ch, k = op
    if c == F:
        if ch == 0:
            return None if i == 0 else (i - 1, (F, 0, k), True)
        return (i + 1, (F, 1, k), True) if i < p - 1 else (i, (F, 0, k), False)
    if c == B:
        if ch == 1:
            return (i - 1, (B, 1, k), True) if i > 0 else (i, (F, 1, k), False)
        return (i + 1, (B, 0, k), True) if i < p - 1 else (i, (B, 1, k), False)
    return (i, (B, ch, k), False)


def _static_part(p: int, sigma: int, m: int) -> List[OpV]:
    """Phases 1 and 2 of worker sigma + 1."""
    i = sigma + 1
    nf, nb, nw = [0, 0], [0, 0], [0, 0]
    ops: List[OpV] = []

    def f(c):
        if nf[c] < m:
            ops.append((F, c, nf[c]))
            nf[c] += 1

    def b(c):
        if nb[c] < nf[c]:
            ops.append((B, c, nb[c]))
            nb[c] += 1

    def w(c):
        if nw[c] < nb[c]:
            ops.append((W, c, nw[c]))
            nw[c] += 1

    for _ in range(2 * (p - i) + 1):
        f(0)
    for _ in range(i - 1):
        f(1)
        f(0)
    chunks = [1] * (p - i)
    while not (nf[0] == m and nf[1] == m):
        if not chunks:
            chunks = [1, 0]
        c = chunks.pop(0)
        f(c)
        b(c)
        w(c)
    return ops


def orders_v(p: int, m: int) -> List[List[OpV]]:
    """The ZB-V orders of all p workers (6m ops each)."""
    if not (p >= 1 and m >= 1):
        raise ValueError("need p >= 1 and m >= 1")
    static = [_static_part(p, s, m) for s in range(p)]
    orders: List[List[OpV]] = [[] for _ in range(p)]
    end: List[Dict[OpV, int]] = [dict() for _ in range(p)]
    nb = [[0, 0] for _ in range(p)]
    nw = [[0, 0] for _ in range(p)]
    t, done = 0, 0

    def ready(i: int, op: OpV) -> bool:
        dep = producer(p, i, op)
        return dep is None or (dep[1] in end[dep[0]] and end[dep[0]][dep[1]] <= t)

    while done < 6 * m * p:
        chosen: List[Optional[OpV]] = [None] * p
        for i in range(p):
            pos = len(orders[i])
            if pos < len(static[i]):
                if ready(i, static[i][pos]):
                    chosen[i] = static[i][pos]
                continue
            for ch in (0, 1):
                k = nb[i][ch]
                if k < m and ready(i, (B, ch, k)):
                    chosen[i] = (B, ch, k)
                    break
            if chosen[i] is None:
                pend = [(nw[i][ch], -ch) for ch in (0, 1) if nw[i][ch] < nb[i][ch]]
                if pend:
                    k, negch = min(pend)     # oldest first; chunk 1 before chunk 0 among equals
                    chosen[i] = (W, -negch, k)
        for i, op in enumerate(chosen):
            if op is None:
                continue
            orders[i].append(op)
            end[i][op] = t + 1
            done += 1
            if op[0] == B:
                nb[i][op[1]] = op[2] + 1
            elif op[0] == W:
                nw[i][op[1]] = op[2] + 1
        t += 1
        if t > 100 * (m + p) * 6:
            raise AssertionError("construction does not terminate")
    return orders


def check_order_v(ops: Sequence[OpV], m: int) -> None:
    seen = set()
    for op in ops:
        c, ch, k = op
        assert c in (F, B, W) and ch in (0, 1) and 0 <= k < m, op
        assert op not in seen, ("twice", op)
        if c != F:
            assert (c - 1, ch, k) in seen, ("before its predecessor", op)
        seen.add(op)
    assert len(seen) == 6 * m


def simulate_v(orders: Sequence[Sequence[OpV]], T_F: float, T_B: float, T_W: float, T_comm: float = 0.0):
    """Start / end of every pass; T_F, T_B, T_W are the times of ONE chunk's pass."""
    p = len(orders)
    dur = {F: T_F, B: T_B, W: T_W}
    start: List[Dict[OpV, float]] = [dict() for _ in range(p)]
    end: List[Dict[OpV, float]] = [dict() for _ in range(p)]
    ptr = [0] * p
    clock = [0.0] * p
    remaining = sum(len(o) for o in orders)
    while remaining:
        progressed = False
        for i in range(p):
            while ptr[i] < len(orders[i]):
                op = orders[i][ptr[i]]
                ready = clock[i]
                dep = producer(p, i, op)
                if dep is not None:
                    j, key, link = dep
                    if key not in end[j]:
                        break
                    ready = max(ready, end[j][key] + (T_comm if link else 0.0))
                start[i][op] = ready
                clock[i] = ready + dur[op[0]]
                end[i][op] = clock[i]
                ptr[i] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise AssertionError("schedule deadlocks")
    return start, end


def cost_v(orders, T_F, T_B, T_W, T_comm=0.0) -> float:
    start, end = simulate_v(orders, T_F, T_B, T_W, T_comm)
    return max(max(end[i].values()) - min(start[i].values()) for i in range(len(orders)))


def memory_peak_v(ops: Sequence[OpV], M_B: float, M_W: float) -> float:
    """Appendix G's walk with chunk-sized increments (M_B, M_W are those of ONE chunk)."""
    delta = (M_B, M_W - M_B, -M_W)
    cur = peak = 0.0
    for c, _, _ in ops:
        cur += delta[c]
        peak = max(peak, cur)
    return peak
