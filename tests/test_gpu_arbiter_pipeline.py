"""The native arbiter driving the stage ABI: a chain of stages on one GPU, dispatched in readiness
order under seeded virtual task times, must produce bit-identical outputs and gradients to the
canonical stage-by-stage order (Sec. 7.1 'correctness validation': readiness-driven execution changes
only runtime ordering), and its dispatch trace must be the one the native simulator predicts."""
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

    # the dispatch order is the simulator's prediction for these task times, and it interleaves the
    # task kinds (the last stage alternates F and B) instead of the canonical all-F-then-B/W order
    dur = {d: np.array([[[tab[(d, s, c, j)] for j in range(M)] for c in range(C)] for s in range(N)]) for d in (0, 1, 2)}
    sim = A.rrfp_sim_run(N, M, dur[0], dur[1], dur[2], n_chunks=C, hint=A.ARB_HINT_BFW, buffer_limit=limit, latency=0.1)
    assert not sim["deadlock"]
    assert sim["trace"] == trace
    if C == 1:
        last = [(d, j) for (s, d, j, c, _, _) in trace if s == N - 1 and d != A.ARB_W]
        assert last == [(d, j) for j in range(M) for d in (A.ARB_F, A.ARB_B)]
    _say(f"[pipeline] stage 0 order: {[('FBW'[d], j, c) for (s, d, j, c, _, _) in trace if s == 0]}")
    pipe.close()
    for st in stages:
        st.close()
