"""The native arbiter driving the stage ABI: a chain of stages on one GPU, dispatched in readiness
order under seeded virtual task times, must produce bit-identical outputs and gradients to the
canonical stage-by-stage order (Sec. 7.1 'correctness validation': readiness-driven execution changes
only runtime ordering); its dispatch trace must be the one the ORACLE simulator (oracle/arbiter_oracle.py,
Algorithm 1 of App. A restated) produces for the same task times, and the outputs and reduced gradients of
the chain must match the chained fp64 stage oracle.  With the jitter model of Sec. 7.6 on measured task
times the results must stay bit-identical and the injected delays must be the oracle injector's."""
import random
import sys

import numpy as np
import pytest

import stage_inputs as SI
from tests import helpers as Hp

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _raw(t):
    import torch
    bits = torch.int16 if t.dtype == torch.bfloat16 else torch.int32
    return t.cpu().view(bits).numpy()


@pytest.mark.parametrize("N,C,limit", [(3, 1, 0), (3, 1, 2), (2, 2, 0), (2, 2, 1)])
def test_pipeline_in_readiness_order_is_bit_identical_to_canonical(N, C, limit):
    """C = 1: a plain pipeline of N stages.  C = 2: an interleaved pipeline, every physical stage owns
    two model chunks and a microbatch visits the stages twice (App. C.2)."""
    import torch
    import paper_2605_18750_amd as R
    from paper_2605_18750_amd import arbiter as A, harness as Hn, pipeline as P

    cus = [[0, 200], [0, 77, 333], [0, 64], [0, 130, 260], [0, 301], [0, 96, 97]]
    M = len(cus)
    V = N * C                      # virtual stages in model order: v = c * N + s
    shapes = [SI.StageShape(f"pipe_stage{v}", 1 + (v == 1), 128, 4, 2, 64, 192, M, w_std=0.05) for v in range(V)]
    works = [Hp.Workload(sh, cus, seed=SI.BASE_SEED + v) for v, sh in enumerate(shapes)]
    T_max = max(c[-1] for c in cus)
    _say(f"[pipeline] N={N} C={C} M={M} limit={limit}")

    def build():
        st = []
        for w in works:
            cfg = Hn.make_config(w.shape, T_max, 2, n_microbatches=M)
            st.append(Hn.Stage(cfg, Hn.pack_params(cfg, w.layers)))
        return st

    xs = [Hn.to_device(t.storage, "bf16") for t in works[0].x]
    dys = [Hn.to_device(t.storage, "bf16") for t in works[0].dy]
    cus_np = [np.asarray(c, dtype=np.int32) for c in cus]

    # canonical: one stream, virtual stage by virtual stage
    stages = build()
    s0 = torch.cuda.Stream()
    torch.cuda.synchronize()
    y = [list(xs)]
    for s in range(V):
        outs = []
        for j in range(M):
            o = torch.empty_like(xs[j])
            R.stage_F(stages[s].handle, j, y[-1][j], cus_np[j], o, s0)
            outs.append(o)
        y.append(outs)
    g = list(dys)
    for s in range(V - 1, -1, -1):
        outs = []
        for j in range(M):
            o = torch.empty_like(xs[j])
            R.stage_B(stages[s].handle, j, g[j], o, s0)
            R.stage_W(stages[s].handle, j, s0)
            outs.append(o)
        g = outs
        R.stage_grad_reduce(stages[s].handle, stages[s].grad_out, s0)
    torch.cuda.synchronize()
    ref_y = [_raw(t) for t in y[-1]]
    ref_dx = [_raw(t) for t in g]
    ref_grads = [st.grad_out.cpu().view(torch.int32).numpy().copy() for st in stages]
    for st in stages:
        st.close()

    # readiness order under seeded, strongly varying virtual task times
    rng = random.Random(5 + limit)
    tab = {(d, s, c, j): rng.uniform(0.2, 3.0) * (1 + (d == A.ARB_B))
           for d in (0, 1, 2) for s in range(N) for c in range(C) for j in range(M)}
    stages = build()
    grid = [[stages[c * N + s] for c in range(C)] for s in range(N)]
    pipe = P.Pipeline(grid, cus_np, hint=A.ARB_HINT_BFW, buffer_limit=limit)
    torch.cuda.synchronize()
    ys, dxs, trace = pipe.run_iteration(xs, dys, lambda d, s, j, c: tab[(d, s, c, j)], latency=0.1)
    for j in range(M):
        assert np.array_equal(_raw(ys[j]), ref_y[j]), f"y[{j}] differs"
        assert np.array_equal(_raw(dxs[j]), ref_dx[j]), f"dx[{j}] differs"
    for v, st in enumerate(stages):
        assert np.array_equal(st.grad_out.cpu().view(torch.int32).numpy(), ref_grads[v]), f"gradients of virtual stage {v} differ"

    # the dispatch order is what the oracle's event loop (App. A, Algorithm 1; App. C.2) gives for these task
    # times, bit for bit including the times; the native simulator agrees as well
    from oracle import arbiter_oracle as AO
    ref_sim = AO.simulate(N, M, lambda d, s, c, j: tab[(d, s, c, j)], C=C, hint=AO.HINT_BFW, limit=limit, latency=0.1)
    assert not ref_sim.deadlock
    assert AO.validate_schedule(N, M, C, ref_sim.trace, latency=0.1, with_w=True) == []
    per_stage = [[(d, j, c, t0, t1) for (s_, d, j, c, t0, t1) in trace if s_ == s] for s in range(N)]
    assert per_stage == ref_sim.trace, "dispatch trace differs from the oracle simulator's"
    dur = {d: np.array([[[tab[(d, s, c, j)] for j in range(M)] for c in range(C)] for s in range(N)]) for d in (0, 1, 2)}
    sim = A.rrfp_sim_run(N, M, dur[0], dur[1], dur[2], n_chunks=C, hint=A.ARB_HINT_BFW, buffer_limit=limit, latency=0.1)
    assert not sim["deadlock"]
    assert sim["trace"] == trace
    if C == 1:
        last = [(d, j) for (s, d, j, c, _, _) in trace if s == N - 1 and d != A.ARB_W]
        assert last == [(d, j) for j in range(M) for d in (A.ARB_F, A.ARB_B)]
    _say(f"[pipeline] stage 0 order: {[('FBW'[d], j, c) for (s, d, j, c, _, _) in trace if s == 0]}")

    # numerics of the chain against the chained fp64 stage oracle (no rounding between its stages)
    ref = _chained_oracle(works, cus_np)
    got = {"y": [Hn.to_f64(t) for t in ys], "dx": [Hn.to_f64(t) for t in dxs], "grads": [], "reduced": []}
    worst = Hp.compare(got, {"y": ref["y"], "dx": ref["dx"], "grads": [], "reduced": []}, 2e-2, "pipeline chain")
    for v, st in enumerate(stages):
        red = Hn.unpack_grads(st.cfg, st.grad_out.cpu().numpy())
        worst = max(worst, Hp.compare({"y": [], "dx": [], "grads": [], "reduced": red},
                                      {"y": [], "dx": [], "grads": [], "reduced": ref["reduced"][v]}, 2e-2,
                                      f"pipeline virtual stage {v}"))
    _say(f"[pipeline] chain vs chained oracle: worst max-norm rel err {worst:.3e}")
    pipe.close()
    for st in stages:
        st.close()


def _chained_oracle(works, cus_np):
    """y, dx and per-virtual-stage reduced gradients of the chain of stages, fp64 stage oracle throughout."""
    from oracle import stage_oracle as SO
    V, M = len(works), len(cus_np)
    cfgs = [Hp.oracle_config(w.shape) for w in works]
    params = [w.oracle_params() for w in works]
    ys, dxs = [], []
    grads = [[None] * M for _ in range(V)]
    for j in range(M):
        x = works[0].x[j].f64
        caches = []
        for v in range(V):
            x, ch = SO.stage_F(x, params[v], cus_np[j], cfgs[v])
            caches.append(ch)
        ys.append(x)
        g = works[0].dy[j].f64
        for v in range(V - 1, -1, -1):
            g, gains, wst = SO.stage_B(g, caches[v], params[v], cfgs[v])
            grads[v][j] = SO.merge_B_W(gains, SO.stage_W(caches[v], wst, cfgs[v]))
        dxs.append(g)
    return {"y": ys, "dx": dxs, "reduced": [SO.grad_reduce(grads[v]) for v in range(V)]}


def test_jitter_on_measured_task_times_leaves_results_bit_identical():
    """Sec. 7.6 on real streams: every F / B task is timed with HIP events on its stream, the measured time
    feeds the moving average, and the drawn delay is put behind the task as a device-side sleep.  J2 with a
    fixed seed must give y, dx and reduced gradients bit-identical to the J0 run of the same pipeline; the
    delays must be what the oracle injector returns for the same measured times, and the dispatch trace what
    the oracle simulator gives for them."""
    import torch
    from paper_2605_18750_amd import arbiter as A, harness as Hn, pipeline as P
    from oracle import arbiter_oracle as AO

    N, C = 3, 1
    cus = [[0, 200], [0, 77, 333], [0, 64], [0, 130, 260], [0, 301], [0, 96, 97], [0, 256], [0, 33, 190]]
    M = len(cus)
    shapes = [SI.StageShape(f"jit_stage{v}", 1 + (v == 1), 128, 4, 2, 64, 192, M, w_std=0.05) for v in range(N)]
    works = [Hp.Workload(sh, cus, seed=SI.BASE_SEED + 40 + v) for v, sh in enumerate(shapes)]
    T_max = max(c[-1] for c in cus)
    xs = [Hn.to_device(t.storage, "bf16") for t in works[0].x]
    dys = [Hn.to_device(t.storage, "bf16") for t in works[0].dy]
    cus_np = [np.asarray(c, dtype=np.int32) for c in cus]
    p_j, base, alpha = AO.JITTER_LEVELS["J2"]
    base *= 0.02                   # these tasks take ~0.1 ms, not the paper's tens of ms: keep delays short
    seed = 77

    def run(jitter):
        stages = []
        for w in works:
            cfg = Hn.make_config(w.shape, T_max, 2, n_microbatches=M)
            stages.append(Hn.Stage(cfg, Hn.pack_params(cfg, w.layers)))
        pipe = P.Pipeline(stages, cus_np, hint=A.ARB_HINT_BFW, buffer_limit=4)
        torch.cuda.synchronize()
        _say(f"[jitter] run with jitter={jitter}")
        ys, dxs, trace = pipe.run_iteration(xs, dys, None, latency=1e-5, jitter=jitter)
        out = ([_raw(t) for t in ys], [_raw(t) for t in dxs],
               [st.grad_out.cpu().view(torch.int32).numpy().copy() for st in stages], trace, list(pipe.delays))
        for st in stages:
            st.close()
        return out

    y0, dx0, g0, trace0, delays0 = run((0.0, 0.0, 0.0, 0))
    assert all(d[5] == 0.0 for d in delays0)
    y1, dx1, g1, trace1, delays1 = run((p_j, base, alpha, seed))
    for j in range(M):
        assert np.array_equal(y0[j], y1[j]), f"y[{j}] changed under jitter"
        assert np.array_equal(dx0[j], dx1[j]), f"dx[{j}] changed under jitter"
    for v in range(N):
        assert np.array_equal(g0[v], g1[v]), f"reduced gradients of stage {v} changed under jitter"
    # delays: the oracle injector fed the same measured times in the same per-stage execution order
    inj = [AO.JitterInjector(AO.Jitter(p=p_j, base=base, alpha=alpha, seed=seed), s, M, C) for s in range(N)]
    n_hit = 0
    for (s, d, j, c, seconds, delay) in delays1:
        if d == A.ARB_W:
            assert delay == 0.0
            continue
        want = inj[s].delay(d, j, c, seconds)
        assert delay == want, (s, d, j, c, seconds, delay, want)
        n_hit += delay > 0
    assert 0 < n_hit < 2 * N * M
    # trace: the oracle's event loop on the measured times (W tasks included) reproduces it bit for bit
    meas = {(s, d, j, c): sec for (s, d, j, c, sec, _) in delays1}
    ref_sim = AO.simulate(N, M, lambda d, s, c, j: meas[(s, d, j, c)], C=C, hint=AO.HINT_BFW, limit=4, latency=1e-5,
                          jitter=AO.Jitter(p=p_j, base=base, alpha=alpha, seed=seed))
    per_stage = [[(d, j, c, t0, t1) for (s_, d, j, c, t0, t1) in trace1 if s_ == s] for s in range(N)]
    assert per_stage == ref_sim.trace
    assert AO.validate_schedule(N, M, C, per_stage, latency=1e-5, with_w=True) == []
    _say(f"[jitter] {n_hit} of {2 * N * M} F/B tasks delayed; results bit-identical")
