"""Heuristic automatic scheduler of Sec. 3.1 (test infrastructure).

Given p stages, m microbatches, the pass times T_F, T_B, T_W, T_comm and an
activation-memory limit M_limit, it builds every stage's pass order by walking
the pipeline forward in time and deciding, each time a stage falls idle, which
pass it runs next.  The decision follows the section's four steps:

 1. warm-up: forwards, as many as the memory limit allows, until the first
    backward can start.  A forward that would still be running when that
    backward becomes ready is taken only under the first binary option
    (`extra_warmup_f`);
 2. then one forward and one backward in turn.  While the pass that is due
    cannot start, a pending W is run if the gap is at least T_W, or if the gap
    is shorter but idling through it would make this stage's cumulative bubble
    the largest of all stages; a W is also run to release memory when a forward
    has arrived but does not fit under M_limit;
 3. a stage may run ahead with forwards while it waits for a backward, as long
    as they end before that backward is ready; the second binary option
    (`skip_f`) forbids it once the stage already leads its successor by one
    forward;
 4. when a stage has no F and no B left it runs its remaining W one by one.

Memory follows Appendix G: F adds M_B, B adds M_W - M_B, W releases M_W.
`search` tries the four combinations of the two options and keeps the cheapest
(Sec. 3.1, last sentence of step 3); cost and bubble rate are those of Sec. 5.3.

The paper gives the steps in prose only.  Everything below the level of that
prose (which stage decides first, what counts as "ready now", ties) is this
module's reading; it is kept because it reproduces the printed bubble rates of
the automatically searched schedules (Sec. 5.3 table, columns ZB-1p and ZB-2p;
see tests/test_oracle_autosched.py).

Reading, in full.  All stages share one clock.  Repeatedly, every unfinished
stage proposes (pass, start time) from what is known so far, the proposal with
the smallest start time is carried out (lowest stage index on ties) and all
proposals are made again.  For stage i with free time c:
  s_F = max(c, end of F of the same microbatch on stage i-1 + T_comm) if that F
        has been carried out (stage 0: c); s_B likewise from stage i+1's B
        (last stage: c, once its own F is done).  A time t is "now" if
        t <= c + tol, tol = 1e-9 (T_F + T_B + T_W).
  fits(s) = the next B is not known yet, or s + T_F <= s_B + tol.
  fill(s) = with a W pending: W now if (earliest of s_B, s) - c >= T_W - tol or
        if idle_i + that gap > max_j idle_j + tol; otherwise wait for the
        earlier of the backward and the allowed forward s (backward on ties).
  warm-up (no B done yet): B if now; else fill(s_F if memory allows and
        (fits(s_F) or (extra_warmup_f and s_F < s_B - tol))).
  no F and no B left: W.
  a forward is due (last of F/B was B, F left): F if arrived and memory allows;
        W if arrived and memory does not allow; else B if now; else fill(s_F
        if memory allows).
  a backward is due: B if now; else fill(s_F if memory allows and fits(s_F) and
        not (skip_f and lead >= 1)), lead = forwards done here minus forwards
        done on the next stage (last stage: minus its own backwards).
idle_i is the time stage i has spent waiting since its first pass started.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

from .schedule import F, B, W, Op, simulate

INF = float("inf")


def auto_schedule(p: int, m: int, T_F: float, T_B: float, T_W: float, T_comm: float,
                  M_limit: float, M_B: float, M_W: float,
                  extra_warmup_f: bool = False, skip_f: bool = False) -> List[List[Op]]:
    """Per-stage orders of the heuristic for one setting of the two options."""
    if not (p >= 1 and m >= 1):
        raise ValueError("need p >= 1 and m >= 1")
    if not (M_B > 0 and 0 <= M_W <= M_B and M_limit >= M_B):
        raise ValueError("need 0 <= M_W <= M_B and M_limit >= M_B > 0")
    dur = (T_F, T_B, T_W)
    dmem = (M_B, M_W - M_B, -M_W)
    tol = 1e-9 * (T_F + T_B + T_W)
    mem_cap = M_limit * (1 + 1e-12)
    clock = [0.0] * p
    nf, nb, nw = [0] * p, [0] * p, [0] * p
    mem = [0.0] * p
    idle = [0.0] * p
    started = [False] * p
    last_fb = [F] * p          # the later of the F/B passes carried out on the stage
    end_f = [[0.0] * m for _ in range(p)]
    end_b = [[0.0] * m for _ in range(p)]
    orders: List[List[Op]] = [[] for _ in range(p)]

    def propose(i: int, max_idle: float) -> Optional[Tuple[int, float]]:
        c = clock[i]
        s_f = None
        if nf[i] < m and (i == 0 or nf[i - 1] > nf[i]):
            s_f = c if i == 0 else max(c, end_f[i - 1][nf[i]] + T_comm)
        s_b = None
        if nb[i] < nf[i] and (i == p - 1 or nb[i + 1] > nb[i]):
            s_b = c if i == p - 1 else max(c, end_b[i + 1][nb[i]] + T_comm)
        has_w = nw[i] < nb[i]
        mem_ok = mem[i] + M_B <= mem_cap
        f_arrived = s_f is not None and s_f <= c + tol
        b_now = s_b is not None and s_b <= c + tol

        def fits(s: float) -> bool:
            return s_b is None or s + T_F <= s_b + tol

        def fill(s: Optional[float]) -> Optional[Tuple[int, float]]:
            nxt = INF if s_b is None else s_b
            take_f = s is not None and s < nxt
            if take_f:
                nxt = s
            if has_w:
                gap = nxt - c
                if gap >= T_W - tol or idle[i] + gap > max_idle + tol:
                    return (W, c)
            if nxt < INF:
                return (F if take_f else B, nxt)
            return None

        if nb[i] == 0:
            if b_now:
                return (B, c)
            ok = s_f is not None and mem_ok and (
                fits(s_f) or (extra_warmup_f and (s_b is None or s_f < s_b - tol)))
            return fill(s_f if ok else None)
        if nf[i] == m and nb[i] == m:
            return (W, c) if has_w else None
        if last_fb[i] == B and nf[i] < m:
            if f_arrived:
                if mem_ok:
                    return (F, c)
                if has_w:
                    return (W, c)
                if b_now:
                    return (B, c)
                return fill(None)
            if b_now:
                return (B, c)
            return fill(s_f if mem_ok else None)
        if b_now:
            return (B, c)
        lead = nf[i] - (nf[i + 1] if i < p - 1 else nb[i])
        ok = s_f is not None and mem_ok and fits(s_f) and not (skip_f and lead >= 1)
        return fill(s_f if ok else None)

    for _ in range(3 * p * m):
        max_idle = max(idle)
        best = None
        for i in range(p):
            if len(orders[i]) == 3 * m:
                continue
            d = propose(i, max_idle)
            if d is not None and (best is None or d[1] < best[1][1]):
                best = (i, d)
        if best is None:
            raise RuntimeError("no stage can run a pass: the memory limit is too small for this pipeline")
        i, (c, s) = best
        k = (nf, nb, nw)[c][i]
        if started[i]:
            idle[i] += s - clock[i]
        started[i] = True
        e = s + dur[c]
        clock[i] = e
        if c == F:
            end_f[i][k] = e
            nf[i] += 1
            last_fb[i] = F
        elif c == B:
            end_b[i][k] = e
            nb[i] += 1
            last_fb[i] = B
        else:
            nw[i] += 1
        mem[i] += dmem[c]
        orders[i].append((c, k))
    return orders


def cost(orders: Sequence[Sequence[Op]], T_F: float, T_B: float, T_W: float, T_comm: float) -> float:
    """Largest stage span (Sec. 5.3): end of a stage's last pass minus start of its first."""
    start, end = simulate(orders, T_F, T_B, T_W, T_comm)
    return max(max(end[i].values()) - min(start[i].values()) for i in range(len(orders)))


OPTION_GRID = ((False, False), (False, True), (True, False), (True, True))


def search(p: int, m: int, T_F: float, T_B: float, T_W: float, T_comm: float,
           M_limit: float, M_B: float, M_W: float):
    """Grid search over the two binary options; returns (orders, cost, (extra_warmup_f, skip_f)).
    The first combination of OPTION_GRID wins ties."""
    best = None
    for ew, sk in OPTION_GRID:
        o = auto_schedule(p, m, T_F, T_B, T_W, T_comm, M_limit, M_B, M_W, ew, sk)
        c = cost(o, T_F, T_B, T_W, T_comm)
        if best is None or c < best[1]:
            best = (o, c, (ew, sk))
    return best


def memory_peak(ops: Sequence[Op], M_B: float, M_W: float) -> float:
    """Peak of the Appendix-G memory walk of one stage's order."""
    delta = (M_B, M_W - M_B, -M_W)
    cur = peak = 0.0
    for c, _ in ops:
        cur += delta[c]
        peak = max(peak, cur)
    return peak
