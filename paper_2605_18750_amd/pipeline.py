"""A miniature of the runtime of Sec. 4.1 / Sec. 5 on ONE GPU: N stage handles chained into a pipeline,
one native ready-set arbiter per stage, one HIP stream per stage, and messages (tensor, microbatch id,
direction) between neighbours.  Every stage dispatches whatever its arbiter selects among READY tasks;
the tasks themselves are the stage_F / stage_B / stage_W calls of the library.

All stages share one device here, so wall-clock readiness would just mirror the enqueue order.  To
exercise out-of-order dispatch deterministically the loop runs on a VIRTUAL clock: the caller gives a
duration per task, a message becomes visible to the receiving arbiter at completion + latency of that
clock, and an idle stage arbitrates whenever something changed (the event loop of the simulator).  The
GPU work is enqueued at dispatch on the stage's own stream; data dependencies between stages are
enforced with HIP events recorded by the producer and waited on by the consumer stream, so the device
executes a valid order whatever the virtual clock says.  No arithmetic of the method lives here.
"""
from __future__ import annotations

import heapq

import paper_2605_18750_amd as R
from . import arbiter as A


class Pipeline:
    def __init__(self, stages, cus, hint: int = A.ARB_HINT_BFW, buffer_limit: int = 0):
        """stages: harness.Stage objects in pipeline order (same hidden size), or, for an interleaved
        pipeline, a list per physical stage with one Stage per model chunk (a microbatch then visits
        stage 0..N-1 with chunk 0, again with chunk 1, ...); cus: cu_seqlens per microbatch."""
        import torch
        self.torch = torch
        self.stages = [list(st) if isinstance(st, (list, tuple)) else [st] for st in stages]
        self.N = len(self.stages)
        self.C = len(self.stages[0])
        assert all(len(st) == self.C for st in self.stages)
        self.M = len(cus)
        self.cus = cus
        self.hint = hint
        self.with_w = hint == A.ARB_HINT_BFW
        self.arbiters = [A.arbiter_create(self.M, self.C, hint, buffer_limit, s, self.N) for s in range(self.N)]
        self.streams = [torch.cuda.Stream() for _ in range(self.N)]

    def close(self):
        for a in self.arbiters:
            A.arbiter_destroy(a)
        self.arbiters = []

    def run_iteration(self, xs, dys, duration, latency: float = 0.0):
        """xs[j]: input of microbatch j to (stage 0, chunk 0); dys[j]: gradient w.r.t. the output of
        (stage N-1, chunk C-1).  duration(dir, stage, microbatch, chunk) -> virtual seconds.  Returns
        (final outputs, input gradients, trace) with trace = [(stage, dir, microbatch, chunk, start, end)]
        in dispatch order; the reduced gradients are in each Stage's grad_out."""
        torch = self.torch
        N, M, C = self.N, self.M, self.C
        y = {}
        dx = {}
        ev_f = {}
        ev_b = {}
        for a in self.arbiters:
            A.arbiter_reset(a)
        if not self.with_w:
            raise ValueError("the stage library needs W tasks before the reduce: use the BFW hint")
        running = [None] * N
        arrivals = []          # heap of (time, seq, stage, dir, microbatch, chunk)
        seq = 0
        trace = []
        t = 0.0

        def f_source(s, c):    # producer of the forward input of (stage s, chunk c), None = the caller
            if s > 0:
                return (s - 1, c)
            return (N - 1, c - 1) if c > 0 else None

        def b_source(s, c):    # producer of the backward input of (stage s, chunk c), None = the caller
            if s < N - 1:
                return (s + 1, c)
            return (0, c + 1) if c < C - 1 else None

        def enqueue(s, d, j, c):
            st, stream = self.stages[s][c], self.streams[s]
            if d == A.ARB_F:
                src = f_source(s, c)
                if src is None:
                    inp = xs[j]
                else:
                    inp = y[(src[0], src[1], j)]
                    stream.wait_event(ev_f[(src[0], src[1], j)])
                y[(s, c, j)] = torch.empty_like(inp)
                R.stage_F(st.handle, j, inp, self.cus[j], y[(s, c, j)], stream)
                ev_f[(s, c, j)] = torch.cuda.Event()
                ev_f[(s, c, j)].record(stream)
            elif d == A.ARB_B:
                src = b_source(s, c)
                if src is None:
                    inp = dys[j]
                else:
                    inp = dx[(src[0], src[1], j)]
                    stream.wait_event(ev_b[(src[0], src[1], j)])
                dx[(s, c, j)] = torch.empty_like(inp)
                R.stage_B(st.handle, j, inp, dx[(s, c, j)], stream)
                ev_b[(s, c, j)] = torch.cuda.Event()
                ev_b[(s, c, j)].record(stream)
            else:
                R.stage_W(st.handle, j, stream)

        while True:
            for s in range(N):
                if running[s] is not None and running[s][1] <= t:
                    task, t_end = running[s]
                    running[s] = None
                    A.arbiter_complete(self.arbiters[s], task)
                    d, j, c = task
                    if d == A.ARB_F:
                        if s + 1 < N:
                            heapq.heappush(arrivals, (t_end + latency, seq, s + 1, A.ARB_F, j, c)); seq += 1
                        elif c + 1 < C:
                            heapq.heappush(arrivals, (t_end + latency, seq, 0, A.ARB_F, j, c + 1)); seq += 1
                    elif d == A.ARB_B:
                        if s > 0:
                            heapq.heappush(arrivals, (t_end + latency, seq, s - 1, A.ARB_B, j, c)); seq += 1
                        elif c > 0:
                            heapq.heappush(arrivals, (t_end + latency, seq, N - 1, A.ARB_B, j, c - 1)); seq += 1
            while arrivals and arrivals[0][0] <= t:
                _, _, s, d, j, c = heapq.heappop(arrivals)
                A.arbiter_post_ready(self.arbiters[s], d, j, c)
            all_done = True
            for s in range(N):
                if running[s] is not None:
                    all_done = False
                    continue
                rc, task = A.arbiter_next(self.arbiters[s])
                if rc == A.ARB_TASK:
                    d, j, c = task
                    p = float(duration(d, s, j, c))
                    enqueue(s, d, j, c)
                    running[s] = (task, t + p)
                    trace.append((s, d, j, c, t, t + p))
                    all_done = False
                elif rc != A.ARB_DONE:
                    all_done = False
            if all_done:
                break
            nxt = [r[1] for r in running if r is not None] + ([arrivals[0][0]] if arrivals else [])
            if not nxt:
                raise RuntimeError("pipeline stalled: no task in flight and no message pending")
            t = min(nxt)
        for s in range(N):
            for c in range(C):
                R.stage_grad_reduce(self.stages[s][c].handle, self.stages[s][c].grad_out, self.streams[s])
        torch.cuda.synchronize()
        return [y[(N - 1, C - 1, j)] for j in range(M)], [dx[(0, 0, j)] for j in range(M)], trace
