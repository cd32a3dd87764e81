"""Pins of the arbiter / simulator oracle against what the paper and the execution model fix.

None of these checks re-types the oracle's own rules: they use the proven bound (Theorem 6.1), the
lower bound L of Sec. 6, the buffer corollary and the deadlock-freedom theorem of App. C, facts the
proofs state about the last stage, closed forms for uniform pipelines, and a schedule validator
that only knows the precedence model of Sec. 3.1.
"""
import random

import pytest

from oracle import arbiter_oracle as A


def rand_durations(N, M, C, seed, lo=0.5, hi=2.0, imbalance=None):
    rng = random.Random(seed)
    tab = {}
    for d in (A.F, A.B, A.W):
        for s in range(N):
            for c in range(C):
                for j in range(M):
                    x = rng.uniform(lo, hi)
                    if imbalance is not None:
                        x *= imbalance[s]
                    if d == A.B:
                        x *= 2.0
                    tab[(d, s, c, j)] = x
    return tab, (lambda d, s, c, j: tab[(d, s, c, j)])


def tables(tab, N, M):
    Fd = [[tab[(A.F, i, 0, j)] for j in range(M)] for i in range(N)]
    Bd = [[tab[(A.B, i, 0, j)] for j in range(M)] for i in range(N)]
    return Fd, Bd


@pytest.mark.parametrize("seed", range(40))
def test_theorem_6_1_upper_bound_and_last_stage_lower_bound(seed):
    rng = random.Random(1000 + seed)
    N, M = rng.randint(1, 6), rng.randint(1, 12)
    imb = [rng.uniform(0.5, 1.5) for _ in range(N)]
    if seed % 2:
        imb[-1] = 2.0          # last-stage-dominant instances (Corollary 6.2's regime)
    tab, dur = rand_durations(N, M, 1, seed, imbalance=imb)
    r = A.simulate(N, M, dur, hint=A.HINT_BF)
    assert not r.deadlock
    assert A.validate_schedule(N, M, 1, r.trace) == []
    Fd, Bd = tables(tab, N, M)
    bound = A.theorem_6_1_bound(Fd, Bd)
    L = sum(Fd[N - 1][j] + Bd[N - 1][j] for j in range(M))
    assert r.makespan <= bound * (1 + 1e-12)
    assert r.makespan >= L * (1 - 1e-12)
    for s in range(N):
        assert r.makespan >= r.busy[s] * (1 - 1e-12)


@pytest.mark.parametrize("N,M", [(1, 5), (3, 7), (4, 4), (6, 11)])
def test_reference_makespans_are_flow_shops(N, M):
    tab, dur = rand_durations(N, M, 1, 7 * N + M)
    Fd, Bd = tables(tab, N, M)
    rf = A.simulate(N, M, dur, forward_only=True)
    rb = A.simulate(N, M, dur, backward_only=True)
    assert rf.makespan == pytest.approx(A.flow_shop_makespan(Fd), rel=1e-12)
    assert rb.makespan == pytest.approx(A.flow_shop_makespan(Bd[::-1]), rel=1e-12)


@pytest.mark.parametrize("hint", [A.HINT_BF, A.HINT_FB, A.HINT_B_PRIO, A.HINT_F_PRIO, A.HINT_FIXED_1F1B])
@pytest.mark.parametrize("N,M", [(1, 1), (1, 6), (4, 8), (5, 3), (8, 16)])
def test_uniform_pipeline_closed_form(hint, N, M):
    # equal integer task times: every work-conserving order and 1F1B reach the textbook
    # (M + N - 1)(f + b); no schedule can beat it (ramp-up, last-stage work, ramp-down)
    f, b = 2.0, 4.0
    r = A.simulate(N, M, lambda d, s, c, j: f if d == A.F else b, hint=hint)
    assert not r.deadlock
    assert A.validate_schedule(N, M, 1, r.trace) == []
    assert r.makespan == (M + N - 1) * (f + b)


def test_single_microbatch_and_single_stage():
    tab, dur = rand_durations(5, 1, 1, 3)
    r = A.simulate(5, 1, dur)
    assert r.makespan == pytest.approx(sum(tab[(d, s, 0, 0)] for d in (A.F, A.B) for s in range(5)), rel=1e-12)
    tab, dur = rand_durations(1, 6, 1, 4)
    r = A.simulate(1, 6, dur)
    assert r.makespan == pytest.approx(sum(tab[(d, 0, 0, j)] for d in (A.F, A.B) for j in range(6)), rel=1e-12)
    # one stage under BF: the strict alternation F0 B0 F1 B1 ... of the last stage (App. C.4 proof)
    assert [(d, j) for d, j, c, _, _ in r.trace[0]] == [(d, j) for j in range(6) for d in (A.F, A.B)]


@pytest.mark.parametrize("seed", range(10))
def test_last_stage_follows_exact_1f1b_under_bf(seed):
    # App. C.4: under the BF hint the last stage has n_f - n_b in {0, 1} at all times
    N, M = 4, 9
    _, dur = rand_durations(N, M, 1, 50 + seed)
    r = A.simulate(N, M, dur, hint=A.HINT_BF)
    nf = nb = 0
    for d, j, c, _, _ in r.trace[N - 1]:
        nf += d == A.F
        nb += d == A.B
        assert nf - nb in (0, 1)


def test_hint_orders_at_stage_zero():
    # stage 0 has every forward ready at time 0 and no buffer limit
    N, M = 3, 5
    dur = lambda d, s, c, j: 1.0
    r = A.simulate(N, M, dur, hint=A.HINT_F_PRIO)
    assert [(d, j) for d, j, c, _, _ in r.trace[0]][:M] == [(A.F, j) for j in range(M)]
    r = A.simulate(N, M, dur, hint=A.HINT_B_PRIO)
    seq = [(d, j) for d, j, c, _, _ in r.trace[0]]
    # a backward is never passed over: whenever a B starts, it is the smallest-index ready one
    assert [j for d, j in seq if d == A.B] == list(range(M))
    # FB vs BF differ only in who goes first when both are ready: with one stage, FB gives F0 F1? no -
    # after F0 both B0 and F1 are ready and the round continues with B, so both alternate
    r1 = A.simulate(1, 4, dur, hint=A.HINT_FB)
    assert [(d, j) for d, j, c, _, _ in r1.trace[0]] == [(A.F, 0), (A.B, 0), (A.F, 1), (A.B, 1), (A.F, 2), (A.B, 2), (A.F, 3), (A.B, 3)]


@pytest.mark.parametrize("limit", [1, 2, 3, 8])
@pytest.mark.parametrize("seed", range(6))
def test_backpressure_bounds_buffers_and_never_deadlocks(limit, seed):
    # App. C.3 corollary: with limit L every buffer holds at most L entries (one chunk);
    # App. C.4: no deadlock for any positive limit
    rng = random.Random(seed)
    N, M = rng.randint(2, 6), rng.randint(4, 14)
    _, dur = rand_durations(N, M, 1, 200 + seed)
    for hint in (A.HINT_BF, A.HINT_FB, A.HINT_F_PRIO, A.HINT_BFW):
        r = A.simulate(N, M, dur, hint=hint, limit=limit)
        assert not r.deadlock
        assert A.validate_schedule(N, M, 1, r.trace, with_w=(hint == A.HINT_BFW)) == []
        for s in range(N):
            assert r.max_D[s] <= limit
            assert r.max_fwd_buffer[s] <= limit
            assert r.max_bwd_buffer[s] <= limit


def test_backpressure_changes_nothing_when_limit_is_large():
    N, M = 4, 10
    _, dur = rand_durations(N, M, 1, 9)
    a = A.simulate(N, M, dur, limit=0)
    b = A.simulate(N, M, dur, limit=M)
    assert a.trace == b.trace


@pytest.mark.parametrize("C", [2, 3])
@pytest.mark.parametrize("limit", [0, 1, 2, 4])
def test_interleaved_chunks_valid_bounded_and_deadlock_free(C, limit):
    # App. C.2/C.3: under backpressure D may overshoot the limit by at most C
    for seed in range(5):
        rng = random.Random(seed)
        N, M = rng.randint(2, 4), rng.randint(3, 8)
        _, dur = rand_durations(N, M, C, 300 + seed)
        r = A.simulate(N, M, dur, C=C, limit=limit)
        assert not r.deadlock
        assert A.validate_schedule(N, M, C, r.trace) == []
        if limit:
            for s in range(N):
                assert r.max_D[s] <= limit + C


def test_within_direction_priority_prefers_chunks_as_stated():
    # forward: smaller chunk first; backward: larger chunk first; ties: smaller microbatch (App. A)
    assert A.next_by_priority({(3, 0), (1, 1), (2, 0)}, A.F) == (2, 0)
    assert A.next_by_priority({(3, 0), (1, 1), (2, 1)}, A.B) == (1, 1)


def test_bfw_runs_weight_tasks_only_when_nothing_else_is_ready():
    N, M = 3, 6
    _, dur = rand_durations(N, M, 1, 77)
    r = A.simulate(N, M, dur, hint=A.HINT_BFW)
    assert A.validate_schedule(N, M, 1, r.trace, with_w=True) == []
    # same F/B times: splitting W off and filling gaps with it cannot lengthen the F/B critical path
    # beyond running W right after its B; weaker, model-free check: all 3*M tasks ran on every stage
    for s in range(N):
        assert len(r.trace[s]) == 3 * M
    # at stage N-1 a W is never dispatched while a backward input is present: after F_j completes
    # B_j is ready locally, so no W may start between F_j and B_j
    seq = [(d, j) for d, j, c, _, _ in r.trace[N - 1]]
    for k, (d, j) in enumerate(seq[:-1]):
        if d == A.F:
            assert seq[k + 1] == (A.B, j)


def test_readiness_first_beats_or_matches_fixed_order_on_the_papers_example_shape():
    # Sec. 2.2 / Fig. 2: when one backward takes longer than planned, the fixed order idles while a
    # ready forward exists.  Durations: unit tasks, B of microbatch 1 at the last stage is slow.
    N, M = 3, 6

    def dur(d, s, c, j):
        return 5.0 if (d == A.B and s == N - 1 and j == 1) else (1.0 if d == A.F else 2.0)
    fixed = A.simulate(N, M, dur, hint=A.HINT_FIXED_1F1B)
    rrfp = A.simulate(N, M, dur, hint=A.HINT_BF)
    assert A.validate_schedule(N, M, 1, fixed.trace) == []
    assert rrfp.makespan <= fixed.makespan


def _arb(hint, M=4, **kw):
    return A.StageArbiter(M=M, hint=hint, **kw)


def test_direction_rules_on_hand_worked_states():
    # Both directions become ready while the stage is idle: BF gives backward the first opportunity
    # (App. A "direction-level priority"), FB forward (Sec. 7.7).
    for hint, first in ((A.HINT_BF, A.B), (A.HINT_FB, A.F)):
        a = _arb(hint)
        assert a.next() is None
        a.Lf.add((2, 0)); a.Lb.add((0, 0))
        assert a.next()[0] == first
    # Inside a round BF moves on to forward after a backward even if more backward work is ready,
    # B-priority does not (Sec. 7.7), F-priority keeps taking forwards.
    a = _arb(A.HINT_BF)
    a.Lb |= {(0, 0), (1, 0)}; a.Lf |= {(2, 0), (3, 0)}
    assert [a.next() for _ in range(4)] == [(A.B, 0, 0), (A.F, 2, 0), (A.B, 1, 0), (A.F, 3, 0)]
    a = _arb(A.HINT_B_PRIO)
    a.Lb |= {(0, 0), (1, 0)}; a.Lf |= {(2, 0), (3, 0)}
    assert [a.next() for _ in range(4)] == [(A.B, 0, 0), (A.B, 1, 0), (A.F, 2, 0), (A.F, 3, 0)]
    a = _arb(A.HINT_F_PRIO)
    a.Lb |= {(0, 0), (1, 0)}; a.Lf |= {(2, 0), (3, 0)}
    assert [a.next() for _ in range(4)] == [(A.F, 2, 0), (A.F, 3, 0), (A.B, 0, 0), (A.B, 1, 0)]
    # An empty backward buffer is skipped at once, never waited for (App. A).
    a = _arb(A.HINT_BF)
    a.Lf |= {(1, 0), (0, 0)}
    assert a.next() == (A.F, 0, 0) and a.next() == (A.F, 1, 0) and a.next() is None


def test_backpressure_rule_on_hand_worked_states():
    # limit 2, two forwards executed, none backward: D = 2 >= limit, forward dispatch is off and
    # the stage waits although a forward is ready (App. C.2); a backward arrival is taken; once D
    # drops below the limit forwards flow again.
    a = _arb(A.HINT_BF, limit=2)
    a.Lf |= {(0, 0), (1, 0), (2, 0)}
    t = a.next(); a.complete(t)
    t = a.next(); a.complete(t)
    assert a.n_f == 2 and a.in_backpressure()
    assert a.next() is None
    a.Lb.add((0, 0))
    t = a.next(); assert t == (A.B, 0, 0); a.complete(t)
    assert not a.in_backpressure()
    assert a.next() == (A.F, 2, 0)


def test_interleaved_backpressure_drain_order_on_the_papers_example():
    # App. C.2, interleaved schedules, the paper's own example: C = 4 local chunks; a microbatch that
    # has completed F_0, F_1, F_2 while F_3 has not arrived -> the stage waits for F_3 (it does not
    # skip to other ready work), after F_3 it waits for B_3, then B_2, B_1, B_0; microbatches are
    # scanned from index 0 upward, so the next microbatch is touched only when the first is drained.
    C, M = 4, 3
    a = A.StageArbiter(M=M, C=C, hint=A.HINT_BF, limit=3)
    # normal mode: F_0, F_1, F_2 of microbatch 0 (forward prefers the smaller chunk, App. A)
    for c in range(3):
        a.Lf.add((0, c))
        t = a.next(); assert t == (A.F, 0, c); a.complete(t)
    assert a.n_f - a.n_b == 3 and a.in_backpressure()
    # ready work of LATER microbatches and a later task of microbatch 0 must not be taken
    a.Lf |= {(1, 0), (2, 0)}
    assert a.next() is None                      # waits for F_3 of microbatch 0
    a.Lf.add((0, 3))
    t = a.next(); assert t == (A.F, 0, 3); a.complete(t)
    assert a.n_f - a.n_b == 4                    # overshoot: at most limit + C (corollary of App. C.3)
    a.Lb.add((0, 1))                             # B_1 arrives early: not the next required task
    assert a.next() is None                      # waits for B_3
    want = [3, 2, 1]
    a.Lb |= {(0, 3), (0, 2)}
    for c in want:                               # B_3, B_2, B_1: after B_1 D = 4 - 3 = 1 < limit, mode ends
        t = a.next(); assert t == (A.B, 0, c), (t, c); a.complete(t)
        assert a.in_backpressure() == (a.n_f - a.n_b >= 3)
    assert not a.in_backpressure()
    # back in readiness order (BF round: backward first, none ready -> forward, smallest chunk, smallest microbatch)
    assert a.next() == (A.F, 1, 0)

    # scan order: with two unfinished microbatches under backpressure the LOWER index is served first
    # even when only the higher one has its required task ready
    a = A.StageArbiter(M=2, C=2, hint=A.HINT_BF, limit=2)
    for j in (0, 1):
        a.Lf.add((j, 0))
        t = a.next(); assert t == (A.F, j, 0); a.complete(t)
    assert a.in_backpressure()
    a.Lf.add((1, 1))                             # microbatch 1 could go on, microbatch 0 cannot
    assert a.next() is None
    a.Lf.add((0, 1))
    t = a.next(); assert t == (A.F, 0, 1); a.complete(t)
    a.Lb |= {(1, 1), (0, 0)}                     # neither is microbatch 0's next required task (B_1)
    assert a.next() is None
    a.Lb.add((0, 1))
    t = a.next(); assert t == (A.B, 0, 1); a.complete(t)
    assert a.in_backpressure()                   # D = 3 - 1 = 2
    t = a.next(); assert t == (A.B, 0, 0); a.complete(t)
    assert not a.in_backpressure()               # D = 1


def test_bfw_weight_task_rule_on_hand_worked_states():
    # W becomes ready when its B completes and runs only when neither B nor F is ready (Sec. 7.1)
    a = _arb(A.HINT_BFW, M=2)
    a.Lf |= {(0, 0), (1, 0)}
    t = a.next(); a.complete(t)                      # F0
    a.Lb.add((0, 0))
    t = a.next(); assert t == (A.B, 0, 0); a.complete(t)
    assert a.Lw == {(0, 0)}
    assert a.next() == (A.F, 1, 0)                   # a forward is ready: W waits
    a.complete((A.F, 1, 0))
    assert a.next() == (A.W, 0, 0)                   # nothing else ready
    a.complete((A.W, 0, 0))
    assert a.next() is None
    assert a.n_target() == 6


def test_jitter_model_statistics_and_pairing():
    # Sec. 7.6: constant compute time c -> the moving average stays at c; a delay is injected with
    # probability p and has mean alpha * max(base, c) * 1.0 (E[0.5 + r] = 1) and range [0.5, 1.5) of it
    N, M, c0 = 1, 4000, 2e-3
    p, base, alpha = A.JITTER_LEVELS["J2"]
    assert (p, base, alpha) == (0.2, 10e-3, 1.0)          # the table's J2 row
    jit = A.Jitter(p=p, base=base, alpha=alpha, seed=11)
    r = A.simulate(N, M, lambda d, s, c, j: c0, jitter=jit)
    extra = [(t1 - t0) - c0 for _, _, _, t0, t1 in r.trace[0]]
    hit = [x for x in extra if x > 1e-12]
    assert abs(len(hit) / len(extra) - p) < 0.02
    unit = alpha * max(base, c0)
    assert min(hit) >= 0.5 * unit * (1 - 1e-9) and max(hit) < 1.5 * unit
    assert abs(sum(hit) / len(hit) / unit - 1.0) < 0.03
    # p = 0 leaves the run untouched
    r0 = A.simulate(2, 5, lambda d, s, c, j: 1.0 + 0.1 * j, jitter=A.Jitter())
    r1 = A.simulate(2, 5, lambda d, s, c, j: 1.0 + 0.1 * j)
    assert r0.trace == r1.trace
    # the pattern is a function of the task, not of the execution order (paired patterns)
    u = A.task_uniforms(5, 2, A.B, 3, 0, 8, 1)
    assert u == A.task_uniforms(5, 2, A.B, 3, 0, 8, 1) and 0.0 <= u[0] < 1.0 and 0.0 <= u[1] < 1.0
    assert u != A.task_uniforms(5, 2, A.F, 3, 0, 8, 1)


def _golden(name):
    import os
    rows = []
    for line in open(os.path.join(os.path.dirname(__file__), "golden", name)):
        line = line.split("#")[0].split()
        if line:
            rows.append(line)
    return rows


def test_splitmix64_reference_values():
    # published outputs of splitmix64 (tests/golden/splitmix64.txt)
    for row in _golden("splitmix64.txt"):
        x = int(row[0], 0)
        for want in row[1:]:
            assert A.splitmix64(x) == int(want, 0)
            x = (x + 0x9E3779B97F4A7C15) & ((1 << 64) - 1)


def test_jitter_levels_are_the_papers_table():
    # Sec. 7.6 table, parameters only (tests/golden/jitter_levels.txt); base delay in seconds here
    rows = _golden("jitter_levels.txt")
    assert [r[0] for r in rows] == ["J0", "J1", "J2", "J3"]
    for name, p, b_ms, alpha in rows:
        assert A.JITTER_LEVELS[name] == (float(p), float(b_ms) * 1e-3, float(alpha))
