"""Plain reference of the ready-set arbiter and of a discrete-event pipeline simulator.

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the cpu_baseline
leg of bench.py; the product (the native arbiter and simulator in the shared library) shares no code
with this file.

What is implemented, in the paper's order and notation:

* the event-driven execution loop of one stage with the backward-forward (BF) hint (App. A,
  Algorithm 1): ready buffers L^f_r and L^b_r, arbitration rounds that give a ready backward
  microbatch the first opportunity and then a ready forward one, never waiting for unready work;
  within a direction forward prefers the smaller model-chunk index, backward the larger one, ties
  go to the smaller microbatch index (App. A, "within-direction priority", "tie breaking");
* the alternative hint orders of Sec. 7.7: FB (forward first in each round), B-priority (backward
  whenever any is ready), F-priority (forward whenever any is ready);
* the BFW variant of Sec. 7.1: the task set also holds a weight task W per (microbatch, chunk),
  ready once the local B of the same pair has completed; a W is dispatched only when neither a
  backward nor a forward task is ready, then the next round starts;
* the buffer backpressure policy of App. C.2: D_i = n_f^i - n_b^i is computed before every
  arbitration; at D_i >= limit a non-interleaved stage (one chunk) disables forward dispatch and
  only drains backward work, waiting if none is ready; an interleaved stage (C > 1 chunks) focuses
  on microbatches one by one in index order, following F_0..F_{C-1}, B_{C-1}..B_0 and waiting for
  the next required task of the first unfinished microbatch;
* the release policy of App. C.1 for buffer occupancy: a forward input is retained from arrival
  until the local backward of the same (microbatch, chunk) completes, a backward input likewise;
  at the last stage the output of the last chunk's forward moves into the backward-ready buffer
  locally;
* a fixed-order 1F1B stage (the baseline the paper compares with, Sec. 7.1): the same runtime, but
  the planned sequence is binding - the stage waits for the head of its sequence.

Readings where the paper is silent:
* W under backpressure: a ready W may be dispatched while the stage waits for backward work (it
  neither produces forward output nor changes D_i).
* W priority among ready W tasks: as backward (larger chunk first, then smaller microbatch).
* "before each arbitration" with a task in flight never happens here: a stage arbitrates only
  when idle, so counting a task at dispatch or at completion gives the same D_i at that moment.

The simulator follows the simplified setting of Sec. 6 (computation time only, inter-stage
dependencies respected) plus an optional constant message latency.  Time is fp64; every time is
formed as start + duration or completion + latency, nothing else, so that an independent
implementation that forms them the same way gets bit-identical times.
"""
from __future__ import annotations

from dataclasses import dataclass, field

F, B, W = 0, 1, 2
DIR_NAME = {F: "F", B: "B", W: "W"}

HINT_BF, HINT_FB, HINT_B_PRIO, HINT_F_PRIO, HINT_BFW, HINT_FIXED_1F1B = 0, 1, 2, 3, 4, 5


def next_by_priority(ready: set, direction: int):
    """NextByPriority of Algorithm 1: forward - smallest chunk, backward (and W) - largest chunk;
    remaining ties - smallest microbatch.  `ready` holds (microbatch, chunk) pairs."""
    if direction == F:
        return min(ready, key=lambda jc: (jc[1], jc[0]))
    return min(ready, key=lambda jc: (-jc[1], jc[0]))


def one_f_one_b_sequence(stage: int, n_stages: int, M: int):
    """The fixed 1F1B order of a non-interleaved stage: N-1-stage warm-up forwards, then one
    forward one backward, then the remaining backwards."""
    warm = min(n_stages - 1 - stage, M)
    seq = [(F, j, 0) for j in range(warm)]
    nf, nb = warm, 0
    while nb < M:
        if nf < M:
            seq.append((F, nf, 0))
            nf += 1
        seq.append((B, nb, 0))
        nb += 1
    return seq


@dataclass
class StageArbiter:
    """State of one stage (Algorithm 1 'State') and the arbitration step."""
    M: int
    C: int = 1
    hint: int = HINT_BF
    limit: int = 0                      # 0 = no backpressure
    fixed: list | None = None           # binding sequence for HINT_FIXED_1F1B
    Lf: set = field(default_factory=set)
    Lb: set = field(default_factory=set)
    Lw: set = field(default_factory=set)
    n_f: int = 0
    n_b: int = 0
    n_w: int = 0
    phase: int = 0                      # position inside the current round (0 = first direction)
    done_f: set = field(default_factory=set)
    done_b: set = field(default_factory=set)
    fixed_pos: int = 0

    def n_target(self) -> int:
        return (3 if self.hint == HINT_BFW else 2) * self.M * self.C

    def n_done(self) -> int:
        return self.n_f + self.n_b + self.n_w

    def in_backpressure(self) -> bool:
        return self.limit > 0 and (self.n_f - self.n_b) >= self.limit

    def _take(self, direction: int):
        buf = {F: self.Lf, B: self.Lb, W: self.Lw}[direction]
        j, c = next_by_priority(buf, direction)
        buf.discard((j, c))
        return (direction, j, c)

    def next(self):
        """One arbitration: the chosen (dir, microbatch, chunk) removed from its ready buffer, or
        None when the stage must wait for the next readiness event."""
        if self.n_done() >= self.n_target():
            return None
        if self.hint == HINT_FIXED_1F1B:
            d, j, c = self.fixed[self.fixed_pos]
            buf = self.Lf if d == F else self.Lb
            if (j, c) in buf:
                buf.discard((j, c))
                self.fixed_pos += 1
                return (d, j, c)
            return None
        if self.in_backpressure():
            if self.C == 1:
                if self.Lb:
                    return self._take(B)
                if self.hint == HINT_BFW and self.Lw:
                    return self._take(W)
                return None
            # interleaved: first unfinished microbatch, its next required task, or wait
            for j in range(self.M):
                want = None
                for c in range(self.C):
                    if (j, c) not in self.done_f:
                        want = (F, j, c)
                        break
                if want is None:
                    for c in range(self.C - 1, -1, -1):
                        if (j, c) not in self.done_b:
                            want = (B, j, c)
                            break
                if want is None:
                    continue
                buf = self.Lf if want[0] == F else self.Lb
                if (want[1], want[2]) in buf:
                    buf.discard((want[1], want[2]))
                    return want
                if self.hint == HINT_BFW and self.Lw:
                    return self._take(W)
                return None
            if self.hint == HINT_BFW and self.Lw:
                return self._take(W)
            return None
        if self.hint in (HINT_B_PRIO, HINT_F_PRIO):
            first = B if self.hint == HINT_B_PRIO else F
            second = F if first == B else B
            if (self.Lb if first == B else self.Lf):
                return self._take(first)
            if (self.Lb if second == B else self.Lf):
                return self._take(second)
            return None
        # round-based hints: BF, FB, BFW
        order = (F, B) if self.hint == HINT_FB else (B, F)
        for _ in range(2):
            d = order[self.phase]
            self.phase ^= 1
            if (self.Lb if d == B else self.Lf):
                return self._take(d)
        # neither direction is ready: the next round starts from its first direction
        self.phase = 0
        if self.hint == HINT_BFW and self.Lw:
            return self._take(W)
        return None

    def complete(self, task):
        d, j, c = task
        if d == F:
            self.n_f += 1
            self.done_f.add((j, c))
        elif d == B:
            self.n_b += 1
            self.done_b.add((j, c))
            if self.hint == HINT_BFW:
                self.Lw.add((j, c))
        else:
            self.n_w += 1


@dataclass
class SimResult:
    makespan: float
    trace: list            # per stage: list of (dir, microbatch, chunk, start, end) in dispatch order
    busy: list             # per stage: summed task time
    max_fwd_buffer: list   # per stage: peak number of retained forward inputs
    max_bwd_buffer: list   # per stage: peak number of backward inputs present
    max_D: list            # per stage: peak of n_f - n_b seen at an arbitration
    deadlock: bool


_MASK = (1 << 64) - 1


def splitmix64(x: int) -> int:
    """The splitmix64 output function (Steele, Lea, Flood 2014) on x + golden-ratio increment."""
    z = (x + 0x9E3779B97F4A7C15) & _MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


def task_uniforms(seed: int, stage: int, d: int, j: int, c: int, M: int, C: int):
    """Two uniforms in [0, 1) that depend only on (seed, task identity): paired jitter patterns for
    runs that execute the same tasks in different orders (Sec. 7.6 protocol)."""
    k = ((stage * 3 + d) * C + c) * M + j
    h1 = splitmix64(seed ^ splitmix64(2 * k))
    h2 = splitmix64(seed ^ splitmix64(2 * k + 1))
    return (h1 >> 11) * 2.0 ** -53, (h2 >> 11) * 2.0 ** -53


@dataclass
class Jitter:
    """Compute-path jitter of Sec. 7.6: e_t = 0.9 e_{t-1} + 0.1 c_t per stage over its F/B tasks in
    execution order; with probability p a delay alpha * max(base, e_t) * (0.5 + r_t), r_t ~ U(0,1),
    is added to the task.  Reading: e starts at the first measured c; W tasks are not delayed and do
    not enter the average (the paper delays F/B tasks)."""
    p: float = 0.0
    base: float = 0.0
    alpha: float = 0.0
    seed: int = 0


class JitterInjector:
    """The per-stage state of the jitter model: feed it the measured compute time of each F/B task in
    execution order, get the delay to add (0.0 when none is injected)."""

    def __init__(self, jitter: Jitter, stage: int, M: int, C: int = 1):
        self.j, self.stage, self.M, self.C = jitter, stage, M, C
        self.e = None

    def delay(self, d: int, microbatch: int, chunk: int, compute_seconds: float) -> float:
        self.e = compute_seconds if self.e is None else 0.9 * self.e + 0.1 * compute_seconds
        u1, u2 = task_uniforms(self.j.seed, self.stage, d, microbatch, chunk, self.M, self.C)
        if u1 < self.j.p:
            return self.j.alpha * max(self.j.base, self.e) * (0.5 + u2)
        return 0.0


# J0..J3 of the robustness table (Sec. 7.6): p_j, base delay in seconds, alpha
JITTER_LEVELS = {"J0": (0.0, 0.0, 0.0), "J1": (0.1, 5e-3, 0.5), "J2": (0.2, 10e-3, 1.0), "J3": (0.3, 15e-3, 1.5)}


def simulate(N: int, M: int, dur, *, C: int = 1, hint: int = HINT_BF, limit: int = 0, latency: float = 0.0,
             forward_only: bool = False, backward_only: bool = False, jitter: Jitter | None = None) -> SimResult:
    """N stages, M microbatches, C chunks per stage.  dur(direction, stage, chunk, microbatch) -> seconds.

    forward_only / backward_only give the reference executions of Sec. 6: all forward work available
    at stage 0 (all backward work available at stage N-1) at time 0, inter-stage dependencies kept,
    the other direction absent."""
    stages = []
    for s in range(N):
        a = StageArbiter(M=M, C=C, hint=hint, limit=limit)
        if hint == HINT_FIXED_1F1B:
            assert C == 1
            a.fixed = one_f_one_b_sequence(s, N, M)
        stages.append(a)
    only = forward_only or backward_only
    target = M * C if only else None
    running = [None] * N              # (task, start, end)
    arrivals = []                     # (time, stage, dir, microbatch, chunk)
    trace = [[] for _ in range(N)]
    busy = [0.0] * N
    fwd_held = [set() for _ in range(N)]
    bwd_held = [set() for _ in range(N)]
    max_f = [0] * N
    max_b = [0] * N
    max_D = [0] * N
    done = [0] * N
    injectors = [JitterInjector(jitter, s, M, C) for s in range(N)] if jitter is not None else None

    def deliver(s, d, j, c):
        if d == F:
            stages[s].Lf.add((j, c))
            fwd_held[s].add((j, c))
            max_f[s] = max(max_f[s], len(fwd_held[s]))
        else:
            stages[s].Lb.add((j, c))
            bwd_held[s].add((j, c))
            max_b[s] = max(max_b[s], len(bwd_held[s]))

    if backward_only:
        for j in range(M):
            deliver(N - 1, B, j, C - 1)
    else:
        # stage 0 has no forward-ready buffer for the first chunk (App. C.1): it admits a microbatch
        # by running its forward; the retained input is counted from that moment
        for j in range(M):
            stages[0].Lf.add((j, 0))

    def finish(s, task, t):
        d, j, c = task
        stages[s].complete(task)
        done[s] += 1
        if d == F:
            if s + 1 < N:
                arrivals.append((t + latency, s + 1, F, j, c))
            elif c + 1 < C:
                arrivals.append((t + latency, 0, F, j, c + 1))
            elif not forward_only:
                deliver(s, B, j, c)          # last stage, last chunk: local move
        elif d == B:
            fwd_held[s].discard((j, c))
            bwd_held[s].discard((j, c))
            if s > 0:
                arrivals.append((t + latency, s - 1, B, j, c))
            elif c > 0:
                arrivals.append((t + latency, N - 1, B, j, c - 1))

    def all_done():
        if only:
            return all(done[s] >= target for s in range(N))
        return all(stages[s].n_done() >= stages[s].n_target() for s in range(N))

    t = 0.0
    makespan = 0.0
    while True:
        # 1. completions at time t, in stage order
        for s in range(N):
            if running[s] is not None and running[s][2] <= t:
                task, t0, t1 = running[s]
                running[s] = None
                finish(s, task, t1)
        # 2. arrivals with time <= t
        keep = []
        for a in arrivals:
            if a[0] <= t:
                deliver(a[1], a[2], a[3], a[4])
            else:
                keep.append(a)
        arrivals[:] = keep
        # 3. idle stages arbitrate, in stage order
        for s in range(N):
            if running[s] is None:
                st = stages[s]
                if only and done[s] >= target:
                    continue
                max_D[s] = max(max_D[s], st.n_f - st.n_b)
                task = st.next()
                if task is not None:
                    d, j, c = task
                    if s == 0 and d == F and c == 0:
                        fwd_held[0].add((j, 0))
                        max_f[0] = max(max_f[0], len(fwd_held[0]))
                    p = dur(d, s, c, j)
                    if jitter is not None and d != W:
                        p = p + injectors[s].delay(d, j, c, p)
                    running[s] = (task, t, t + p)
                    trace[s].append((d, j, c, t, t + p))
                    busy[s] += p
                    makespan = max(makespan, t + p)
        if all_done() and all(r is None for r in running):
            break
        nxt = [r[2] for r in running if r is not None] + [a[0] for a in arrivals]
        if not nxt:
            return SimResult(makespan, trace, busy, max_f, max_b, max_D, deadlock=True)
        t = min(nxt)
    return SimResult(makespan, trace, busy, max_f, max_b, max_D, deadlock=False)


def flow_shop_makespan(times) -> float:
    """Permutation flow shop in index order: times[i][j] of job j on machine i (machines in
    pipeline order).  c[i][j] = max(c[i-1][j], c[i][j-1]) + times[i][j]."""
    n_mach, n_job = len(times), len(times[0])
    c = [[0.0] * n_job for _ in range(n_mach)]
    for i in range(n_mach):
        for j in range(n_job):
            up = c[i - 1][j] if i else 0.0
            left = c[i][j - 1] if j else 0.0
            c[i][j] = max(up, left) + times[i][j]
    return c[-1][-1]


def theorem_6_1_bound(Fd, Bd) -> float:
    """Right-hand side of Theorem 6.1 for forward / backward times Fd[i][j], Bd[i][j]."""
    N, M = len(Fd), len(Fd[0])
    calF = flow_shop_makespan(Fd)
    calB = flow_shop_makespan([Bd[i] for i in range(N - 1, -1, -1)])
    s1 = sum(max(Fd[i][j] for i in range(N)) - Fd[N - 1][j] for j in range(1, M))
    s2 = sum(max(Bd[i][j] for i in range(N)) - Bd[N - 1][j] for j in range(0, M - 1))
    return calF + calB + s1 + s2


def validate_schedule(N, M, C, trace, latency=0.0, with_w=False):
    """Checks a trace against the execution model of Sec. 3.1: each stage runs one task at a time,
    every task appears exactly once, and no task starts before its predecessors have ended (plus
    latency for inter-stage edges).  Returns a list of violations (empty = valid)."""
    bad = []
    end = {}
    start = {}
    for s in range(N):
        last_end = 0.0
        for (d, j, c, t0, t1) in trace[s]:
            key = (s, d, j, c)
            if key in end:
                bad.append(("duplicate", key))
            start[key], end[key] = t0, t1
            if t0 < last_end:
                bad.append(("overlap", key))
            last_end = t1
    for s in range(N):
        for c in range(C):
            for j in range(M):
                for d in (F, B) + ((W,) if with_w else ()):
                    if (s, d, j, c) not in end:
                        bad.append(("missing", (s, d, j, c)))
    if bad:
        return bad

    def need(key, pred, lat):
        if pred is not None and start[key] < end[pred] + lat:
            bad.append(("precedence", key, pred))

    for s in range(N):
        for c in range(C):
            for j in range(M):
                if s > 0:
                    need((s, F, j, c), (s - 1, F, j, c), latency)
                elif c > 0:
                    need((s, F, j, c), (N - 1, F, j, c - 1), latency)
                if s + 1 < N:
                    need((s, B, j, c), (s + 1, B, j, c), latency)
                elif c + 1 < C:
                    need((s, B, j, c), (0, B, j, c + 1), latency)
                need((s, B, j, c), (s, F, j, c), 0.0)
                if s == N - 1 and c == C - 1:
                    need((s, B, j, c), (s, F, j, c), 0.0)
                if with_w:
                    need((s, W, j, c), (s, B, j, c), 0.0)
    return bad
