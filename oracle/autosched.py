"""Heuristic automatic scheduler of Sec. 3.1 (test infrastructure).

Given p stages, m microbatches, the pass times T_F, T_B, T_W, T_comm and an
activation-memory limit M_limit, the section's four steps are carried out in
the order the section gives them, building every stage's pass list at once:

 1. warm-up: every stage runs forwards, as many as fit under the memory limit,
    until its first backward can start; a forward that would still be running
    when that backward arrives is added only under the first binary option
    (`extra_warmup_f`), and it then delays the backward;
 2. then rounds of one backward and one forward per stage.  Before a pass that
    cannot start yet, pending W passes are put into the gap while a whole W
    fits; if a gap shorter than T_W remains, one more W is put there (delaying
    the pass) only if idling through the gap would raise the largest cumulative
    bubble of all stages; W passes are also run to release memory when the next
    forward does not fit under M_limit;
 3. stage i never lets stage i+1 catch up to fewer than one forward behind it
    while it has forwards left.  When it is more than one ahead, the second
    binary option (`skip_f`) leaves its forward out of the round, provided the
    stage has a W pending to work on instead (no new bubble);
 4. a stage whose F and B have run out runs its remaining W one by one.

Memory follows Appendix G: F adds M_B, B adds M_W - M_B, W releases M_W.
`search` tries the four combinations of the two options and keeps the cheapest
(last sentence of step 3); cost and bubble rate are those of Sec. 5.3.

The paper gives the steps in prose only; what lies below that prose is this
module's reading, kept because it reproduces the printed bubble rates of the
searched schedules (Sec. 5.3 table: all twelve ZB-1p values and eleven of the
twelve ZB-2p values to every printed digit; see tests/test_oracle_autosched.py).

Reading, in full.
  Warm-up counts.  Stage 0 may hold floor(M_limit / M_B) forwards (at most m),
  every later stage one fewer than the stage before it (step 3), at least one.
  The counts are fixed from the last stage to the first, because the moment the
  first backward reaches a stage depends on the stages after it.  Forward k of
  stage i ends at i (T_F + T_comm) + (k + 1) T_F (the stages before it hold more
  forwards and deliver without gaps).  The last stage runs F_0, then B_0.  Stage
  i takes forwards while they end no later than B_0 can start there (end of B_0
  on stage i+1 plus T_comm); with `extra_warmup_f`, if the stage would still
  idle before B_0 and its bound allows, one more.  B_0 then starts when both the
  last warm-up forward has ended and the gradient has arrived.
  Rounds j = 0 .. m-1.  Backward phase, last stage to first: fill (see below)
  up to the moment B_j can start, then B_j.  Forward phase, first stage to last:
  a stage takes its next forward if it has one left and the stage before it
  (unless that one has used up its forwards) stays at least one forward ahead
  afterwards; `skip_f` leaves it out when the stage leads its successor by more
  than one and has a W pending; neither rule applies to the forward the next
  round's backward needs, which is always taken (so tiny memory limits, where
  several stages hold a single forward, still give a valid schedule);
  pending W run while the forward does not fit under M_limit; then fill up to
  the forward's arrival, then the forward.
  fill(stage, t): while a W is pending and ends by t, run it; then, if a W is
  pending and the stage would still idle until t, run one more if
  bubble(stage) + (t - now) > max over stages of bubble.  bubble(stage) is the
  idle time the stage has accumulated since its first pass began.
  "By t" and "idle" are judged with a tolerance of 1e-9 (T_F + T_B + T_W).
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

from .schedule import F, B, W, Op, simulate


class _Pipeline:
    """Pass lists under construction, with every stage's clock, memory and cumulative bubble."""

    def __init__(self, p, m, T_F, T_B, T_W, T_comm, M_limit, M_B, M_W):
        self.p, self.m = p, m
        self.dur = (T_F, T_B, T_W)
        self.comm = T_comm
        self.delta = (M_B, M_W - M_B, -M_W)
        self.M_B = M_B
        self.cap = M_limit * (1 + 1e-12)
        self.tol = 1e-9 * (T_F + T_B + T_W)
        self.now = [0.0] * p
        self.mem = [0.0] * p
        self.bubble = [0.0] * p
        self.count = [[0, 0, 0] for _ in range(p)]
        self.end: List[Dict[Op, float]] = [dict() for _ in range(p)]
        self.orders: List[List[Op]] = [[] for _ in range(p)]

    def earliest(self, i: int, c: int) -> float:
        """When the stage's next pass of kind c can start."""
        k = self.count[i][c]
        t = self.now[i]
        if c == F and i > 0:
            t = max(t, self.end[i - 1][(F, k)] + self.comm)
        elif c == B and i < self.p - 1:
            t = max(t, self.end[i + 1][(B, k)] + self.comm)
        return t

    def run(self, i: int, c: int) -> None:
        k = self.count[i][c]
        t = self.earliest(i, c)
        if self.orders[i]:
            self.bubble[i] += t - self.now[i]
        self.now[i] = t + self.dur[c]
        self.end[i][(c, k)] = self.now[i]
        self.count[i][c] += 1
        self.mem[i] += self.delta[c]
        self.orders[i].append((c, k))

    def w_pending(self, i: int) -> bool:
        return self.count[i][W] < self.count[i][B]

    def fill(self, i: int, t: float) -> None:
        """Step 2: W passes into the gap before a pass that can start at t."""
        T_W = self.dur[W]
        while self.w_pending(i) and self.now[i] + T_W <= t + self.tol:
            self.run(i, W)
        gap = t - self.now[i]
        if self.w_pending(i) and gap > self.tol and self.bubble[i] + gap > max(self.bubble) + self.tol:
            self.run(i, W)

    def fits(self, i: int) -> bool:
        return self.mem[i] + self.M_B <= self.cap


def warmup_counts(p: int, m: int, T_F: float, T_B: float, T_comm: float, M_limit: float, M_B: float,
                  extra_warmup_f: bool) -> List[int]:
    """Step 1: forwards every stage runs before its first backward."""
    tol = 1e-9 * (T_F + T_B)
    bound = [0] * p
    bound[0] = max(1, min(m, int(M_limit * (1 + 1e-12) / M_B)))
    for i in range(1, p):
        bound[i] = max(1, bound[i - 1] - 1)
    counts = [0] * p
    b0_end = 0.0
    for i in range(p - 1, -1, -1):
        def f_end(k: int) -> float:
            return i * (T_F + T_comm) + (k + 1) * T_F
        b0_ready = f_end(0) if i == p - 1 else b0_end + T_comm
        n = 1
        while n < bound[i] and f_end(n) <= b0_ready + tol:
            n += 1
        if extra_warmup_f and n < bound[i] and f_end(n - 1) < b0_ready - tol:
            n += 1
        counts[i] = n
        b0_end = max(b0_ready, f_end(n - 1)) + T_B
    return counts


def auto_schedule(p: int, m: int, T_F: float, T_B: float, T_W: float, T_comm: float,
                  M_limit: float, M_B: float, M_W: float,
                  extra_warmup_f: bool = False, skip_f: bool = False) -> List[List[Op]]:
    """Per-stage orders of the heuristic for one setting of the two options."""
    if not (p >= 1 and m >= 1):
        raise ValueError("need p >= 1 and m >= 1")
    if not (M_B > 0 and 0 <= M_W <= M_B and M_limit >= M_B):
        raise ValueError("need 0 <= M_W <= M_B and M_limit >= M_B > 0")
    pl = _Pipeline(p, m, T_F, T_B, T_W, T_comm, M_limit, M_B, M_W)
    nf = lambda i: pl.count[i][F]
    for i, n in enumerate(warmup_counts(p, m, T_F, T_B, T_comm, M_limit, M_B, extra_warmup_f)):
        for _ in range(n):
            pl.run(i, F)
    for j in range(m):
        for i in range(p - 1, -1, -1):
            pl.fill(i, pl.earliest(i, B))
            pl.run(i, B)
        for i in range(p):
            if nf(i) == m:
                continue
            if nf(i) > j + 1:   # otherwise the next round's backward needs this forward: it is taken
                if i > 0 and nf(i - 1) < m and nf(i) + 1 >= nf(i - 1):
                    continue
                if skip_f and i < p - 1 and nf(i) - nf(i + 1) > 1 and pl.w_pending(i):
                    continue
            while not pl.fits(i):
                if not pl.w_pending(i):
                    raise RuntimeError("the memory limit is too small for this pipeline")
                pl.run(i, W)
            pl.fill(i, pl.earliest(i, F))
            pl.run(i, F)
    for i in range(p):
        while pl.w_pending(i):
            pl.run(i, W)
    return pl.orders


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
