"""Native arbiter and simulator (C ABI, host code) against the plain oracle: identical decisions,
identical simulated times (bit for bit: both sides form every time as start + duration or
completion + latency), identical buffer peaks, on seeded scenarios that cover every hint order,
backpressure limits, interleaved chunks, message latency and the jitter model."""
import random

import numpy as np
import pytest

from oracle import arbiter_oracle as O
from paper_2605_18750_amd import arbiter as A


def durations(N, M, C, seed):
    rng = np.random.default_rng(seed)
    stage_scale = rng.uniform(0.6, 1.6, size=(N, 1, 1))
    f = rng.uniform(0.5, 2.0, size=(N, C, M)) * stage_scale
    b = rng.uniform(1.0, 4.0, size=(N, C, M)) * stage_scale
    w = rng.uniform(0.5, 2.0, size=(N, C, M)) * stage_scale
    return f, b, w


def run_both(N, M, C, hint, limit, latency, seed, jitter=None, mode=0):
    f, b, w = durations(N, M, C, seed)
    tab = {O.F: f, O.B: b, O.W: w}
    dur = lambda d, s, c, j: float(tab[d][s, c, j])
    oj = O.Jitter(*jitter) if jitter else None
    ref = O.simulate(N, M, dur, C=C, hint=hint, limit=limit, latency=latency, jitter=oj,
                     forward_only=(mode == 1), backward_only=(mode == 2))
    got = A.rrfp_sim_run(N, M, f, b, w, n_chunks=C, hint=hint, buffer_limit=limit, mode=mode, latency=latency,
                         jitter=jitter or (0.0, 0.0, 0.0, 0))
    return ref, got


def assert_same(ref, got, N):
    assert got["deadlock"] == ref.deadlock
    assert got["makespan"] == ref.makespan                     # bit-exact
    per_stage = [[] for _ in range(N)]
    for s, d, j, c, t0, t1 in got["trace"]:
        per_stage[s].append((d, j, c, t0, t1))
    assert per_stage == ref.trace                              # same tasks, same order, same times
    assert list(got["max_fwd_buffer"]) == ref.max_fwd_buffer
    assert list(got["max_bwd_buffer"]) == ref.max_bwd_buffer
    assert list(got["max_D"]) == ref.max_D
    np.testing.assert_allclose(got["busy"], ref.busy, rtol=1e-12)


HINTS = [O.HINT_BF, O.HINT_FB, O.HINT_B_PRIO, O.HINT_F_PRIO, O.HINT_BFW, O.HINT_FIXED_1F1B]


def test_hint_codes_agree_with_the_header():
    assert (A.ARB_HINT_BF, A.ARB_HINT_FB, A.ARB_HINT_B_PRIO, A.ARB_HINT_F_PRIO, A.ARB_HINT_BFW,
            A.ARB_HINT_FIXED_1F1B) == tuple(HINTS)
    assert (A.ARB_F, A.ARB_B, A.ARB_W) == (O.F, O.B, O.W)


@pytest.mark.parametrize("hint", HINTS)
@pytest.mark.parametrize("limit", [0, 1, 3])
def test_simulator_matches_oracle_one_chunk(hint, limit):
    if hint == O.HINT_FIXED_1F1B and limit:
        pytest.skip("the fixed order has no backpressure mode")
    for seed in range(6):
        rng = random.Random(seed * 31 + hint)
        N, M = rng.randint(1, 7), rng.randint(1, 17)
        latency = [0.0, 0.0, 0.25][seed % 3]
        ref, got = run_both(N, M, 1, hint, limit, latency, 1000 + seed)
        assert_same(ref, got, N)
        assert not got["deadlock"]


@pytest.mark.parametrize("C", [2, 3])
@pytest.mark.parametrize("hint", [O.HINT_BF, O.HINT_FB, O.HINT_B_PRIO, O.HINT_F_PRIO, O.HINT_BFW])
def test_simulator_matches_oracle_interleaved(C, hint):
    for seed in range(5):
        rng = random.Random(seed * 17 + C)
        N, M = rng.randint(2, 5), rng.randint(2, 9)
        limit = [0, 1, 2, 4, 0][seed]
        ref, got = run_both(N, M, C, hint, limit, 0.1 * (seed % 2), 2000 + seed)
        assert_same(ref, got, N)
        assert not got["deadlock"]


@pytest.mark.parametrize("level", ["J1", "J2", "J3"])
def test_simulator_matches_oracle_with_jitter(level):
    p, base, alpha = O.JITTER_LEVELS[level]
    for seed in range(4):
        for hint in (O.HINT_BF, O.HINT_FIXED_1F1B, O.HINT_BFW):
            # durations of O(1) with a base delay of O(1): scale the table's milliseconds to this unit
            ref, got = run_both(4, 12, 1, hint, 0, 0.0, 3000 + seed, jitter=(p, base * 100, alpha, 77 + seed))
            assert_same(ref, got, 4)


@pytest.mark.parametrize("mode", [1, 2])
def test_reference_executions_match(mode):
    for seed in range(4):
        ref, got = run_both(5, 9, 1, O.HINT_BF, 0, 0.0, 4000 + seed, mode=mode)
        assert got["makespan"] == ref.makespan
        assert not got["deadlock"]


def test_arbiter_api_random_event_streams_match_oracle():
    # one stage driven by a random interleaving of arrivals and arbitrations
    for seed in range(60):
        rng = random.Random(seed)
        M, C = rng.randint(1, 9), rng.randint(1, 3)
        hint = rng.choice([O.HINT_BF, O.HINT_FB, O.HINT_B_PRIO, O.HINT_F_PRIO, O.HINT_BFW])
        limit = rng.choice([0, 0, 1, 2, 5])
        N = 3
        stage = rng.choice([0, 1, 2])
        a = A.arbiter_create(M, C, hint, limit, stage, N)
        o = O.StageArbiter(M=M, C=C, hint=hint, limit=limit)
        if stage == 0:
            o.Lf |= {(j, 0) for j in range(M)}
        pending_f = [(j, c) for c in range(C) for j in range(M) if not (stage == 0 and c == 0)]
        rng.shuffle(pending_f)
        pending_b = []                     # backward inputs that may arrive (local forward done)
        steps = 0
        while o.n_done() < o.n_target():
            steps += 1
            assert steps < 10000
            r = rng.random()
            if pending_f and r < 0.35:
                j, c = pending_f.pop()
                o.Lf.add((j, c)); A.arbiter_post_ready(a, A.ARB_F, j, c)
            elif pending_b and r < 0.6:
                j, c = pending_b.pop(rng.randrange(len(pending_b)))
                o.Lb.add((j, c)); A.arbiter_post_ready(a, A.ARB_B, j, c)
            else:
                want = o.next()
                rc, got = A.arbiter_next(a)
                if want is None:
                    assert rc == A.ARB_WAIT and got is None
                    if not pending_f and not pending_b:
                        # nothing can arrive any more: only possible when everything is done
                        assert o.n_done() >= o.n_target()
                    continue
                assert rc == A.ARB_TASK and got == want
                o.complete(want); A.arbiter_complete(a, got)
                d, j, c = want
                if d == O.F:
                    if stage == N - 1 and c == C - 1:
                        o.Lb.add((j, c))   # the native side does this move inside arbiter_complete
                    else:
                        pending_b.append((j, c))
                cnt = A.arbiter_counters(a)
                assert (cnt["n_f"], cnt["n_b"], cnt["n_w"]) == (o.n_f, o.n_b, o.n_w)
                assert cnt["backpressure"] == o.in_backpressure()
        rc, _ = A.arbiter_next(a)
        assert rc == A.ARB_DONE
        A.arbiter_destroy(a)


def test_arbiter_rejects_misuse():
    with pytest.raises(A.ArbiterError):
        A.arbiter_create(0)
    with pytest.raises(A.ArbiterError):
        A.arbiter_create(4, 2, A.ARB_HINT_FIXED_1F1B)
    a = A.arbiter_create(4, 1, A.ARB_HINT_BF, 0, 1, 3)
    with pytest.raises(A.ArbiterError):
        A.arbiter_post_ready(a, A.ARB_B, 0, 0)          # backward input before the local forward ran
    with pytest.raises(A.ArbiterError):
        A.arbiter_post_ready(a, A.ARB_F, 4, 0)          # microbatch out of range
    A.arbiter_post_ready(a, A.ARB_F, 2, 0)
    with pytest.raises(A.ArbiterError):
        A.arbiter_post_ready(a, A.ARB_F, 2, 0)          # duplicate
    rc, t = A.arbiter_next(a)
    assert rc == A.ARB_TASK and t == (A.ARB_F, 2, 0)
    with pytest.raises(A.ArbiterError):
        A.arbiter_next(a)                               # one task in flight at a time
    with pytest.raises(A.ArbiterError):
        A.arbiter_complete(a, (A.ARB_F, 1, 0))          # not the task in flight
    A.arbiter_complete(a, t)
    assert "in flight" in A.arbiter_last_error(a) or A.arbiter_last_error(a)
    A.arbiter_reset(a)
    assert A.arbiter_counters(a)["completed"] == 0
    A.arbiter_destroy(a)


def test_large_pipeline_runs_and_respects_the_bounds():
    # 64 stages x 512 microbatches natively; Theorem 6.1 and the last-stage lower bound on the result
    N, M = 64, 512
    f, b, w = durations(N, M, 1, 5)
    got = A.rrfp_sim_run(N, M, f, b, None, want_trace=False)
    assert not got["deadlock"] and got["n_events"] == 2 * N * M
    Fd, Bd = f[:, 0, :].tolist(), b[:, 0, :].tolist()
    assert got["makespan"] <= O.theorem_6_1_bound(Fd, Bd) * (1 + 1e-12)
    assert got["makespan"] >= (f[N - 1, 0].sum() + b[N - 1, 0].sum()) * (1 - 1e-12)
    lim = A.rrfp_sim_run(N, M, f, b, None, buffer_limit=32, want_trace=False)
    assert not lim["deadlock"] and lim["max_D"].max() <= 32 and lim["max_fwd_buffer"].max() <= 32


def test_jitter_injector_matches_oracle_bit_for_bit():
    rng = random.Random(3)
    for level in ("J1", "J2", "J3"):
        p, base, alpha = O.JITTER_LEVELS[level]
        for stage in (0, 5):
            M, C, seed = 24, 2, 99 + stage
            nat = A.jitter_create(p, base, alpha, seed, stage, M, C)
            ref = O.JitterInjector(O.Jitter(p, base, alpha, seed), stage, M, C)
            hits = 0
            for _ in range(300):
                d, j, c = rng.choice((O.F, O.B)), rng.randrange(M), rng.randrange(C)
                comp = rng.uniform(1e-3, 30e-3)
                want = ref.delay(d, j, c, comp)
                got = A.jitter_next_delay(nat, d, j, c, comp)
                assert got == want
                hits += got > 0
            assert hits > 0
            A.jitter_destroy(nat)
    with pytest.raises(A.ArbiterError):
        A.jitter_create(1.5, 0.0, 1.0, 0, 0, 4)


@pytest.mark.parametrize("N,M,C,limit,jit", [(3, 6, 1, 0, None), (3, 6, 1, 2, (0.3, 0.5, 1.0, 9)), (2, 6, 2, 1, None),
                                            (4, 9, 3, 2, (0.2, 0.1, 0.7, 3)), (1, 4, 1, 0, None)])
def test_pipe_event_loop_one_dispatch_at_a_time_matches_oracle(N, M, C, limit, jit):
    # the resumable form of the event loop (rrfp_pipe_*), durations supplied task by task: trace, times and
    # delays identical to the oracle simulator; the named producer of every input is the routing rule of
    # Sec. 4.1 (neighbour stage, or the other end of the pipeline when the microbatch changes chunk)
    rng = random.Random(N * 100 + M)
    tab = {(d, s, c, j): rng.uniform(0.2, 3.0) for d in (0, 1, 2) for s in range(N) for c in range(C) for j in range(M)}
    pipe = A.rrfp_pipe_create(N, M, C, A.ARB_HINT_BFW, limit, 0.1, jit or (0.0, 0.0, 0.0, 0))
    tr = []
    while True:
        rc, d = A.rrfp_pipe_next(pipe)
        if rc == A.ARB_DONE:
            break
        s, dd, j, c, ss, sc, start = d
        if dd == A.ARB_F:
            want = (s - 1, c) if s > 0 else ((N - 1, c - 1) if c > 0 else (-1, -1))
        elif dd == A.ARB_B:
            want = (s + 1, c) if s + 1 < N else ((0, c + 1) if c + 1 < C else (-1, -1))
        else:
            want = (-1, -1)
        assert (ss, sc) == want
        with pytest.raises(A.ArbiterError):
            A.rrfp_pipe_next(pipe)                      # the duration is still owed
        delay, end = A.rrfp_pipe_set_duration(pipe, tab[(dd, s, c, j)])
        assert (delay > 0.0) <= (jit is not None and dd != A.ARB_W)
        tr.append((s, dd, j, c, start, end))
    with pytest.raises(A.ArbiterError):
        A.rrfp_pipe_set_duration(pipe, 1.0)             # nothing waits for a duration
    assert A.rrfp_pipe_next(pipe)[0] == A.ARB_DONE
    A.rrfp_pipe_destroy(pipe)
    ref = O.simulate(N, M, lambda d, s, c, j: tab[(d, s, c, j)], C=C, hint=O.HINT_BFW, limit=limit, latency=0.1,
                     jitter=O.Jitter(*jit) if jit else None)
    assert [[(d, j, c, t0, t1) for (s_, d, j, c, t0, t1) in tr if s_ == s] for s in range(N)] == ref.trace
    with pytest.raises(A.ArbiterError):
        A.rrfp_pipe_create(0, 4)
