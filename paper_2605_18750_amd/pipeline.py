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
        """stages: harness.Stage objects in pipeline order (same hidden size); cus: cu_seqlens per microbatch."""
        import torch
        self.torch = torch
        self.stages = stages
        self.N = len(stages)
        self.M = len(cus)
        self.cus = cus
        self.hint = hint
        self.with_w = hint == A.ARB_HINT_BFW
        self.arbiters = [A.arbiter_create(self.M, 1, hint, buffer_limit, s, self.N) for s in range(self.N)]
        self.streams = [torch.cuda.Stream() for _ in range(self.N)]

    def close(self):
        for a in self.arbiters:
            A.arbiter_destroy(a)
        self.arbiters = []

    def run_iteration(self, xs, dys, duration, latency: float = 0.0):
        """xs[j]: stage-0 input of microbatch j; dys[j]: gradient w.r.t. the last stage's output.
        duration(dir, stage, microbatch) -> virtual seconds.  Returns (ys of the last stage, dxs of
        stage 0, trace) with trace = [(stage, dir, microbatch, start, end)] in dispatch order; the
        reduced gradients are in each stage's grad_out."""
        torch = self.torch
        N, M = self.N, self.M
        y = [[None] * M for _ in range(N)]
        dx = [[None] * M for _ in range(N)]
        ev_f = [[None] * M for _ in range(N)]
        ev_b = [[None] * M for _ in range(N)]
        for a in self.arbiters:
            A.arbiter_reset(a)
        if not self.with_w:
            raise ValueError("the stage library needs W tasks before the reduce: use the BFW hint")
        running = [None] * N
        arrivals = []          # heap of (time, seq, stage, dir, microbatch)
        seq = 0
        trace = []
        t = 0.0

        def enqueue(s, d, j):
            st, stream = self.stages[s], self.streams[s]
            if d == A.ARB_F:
                src = xs[j] if s == 0 else y[s - 1][j]
                if s > 0:
                    stream.wait_event(ev_f[s - 1][j])
                y[s][j] = torch.empty_like(src)
                R.stage_F(st.handle, j, src, self.cus[j], y[s][j], stream)
                ev_f[s][j] = torch.cuda.Event()
                ev_f[s][j].record(stream)
            elif d == A.ARB_B:
                src = dys[j] if s == N - 1 else dx[s + 1][j]
                if s < N - 1:
                    stream.wait_event(ev_b[s + 1][j])
                dx[s][j] = torch.empty_like(src)
                R.stage_B(st.handle, j, src, dx[s][j], stream)
                ev_b[s][j] = torch.cuda.Event()
                ev_b[s][j].record(stream)
            else:
                R.stage_W(st.handle, j, stream)

        while True:
            for s in range(N):
                if running[s] is not None and running[s][1] <= t:
                    task, t_end = running[s]
                    running[s] = None
                    A.arbiter_complete(self.arbiters[s], task)
                    d, j, _ = task
                    if d == A.ARB_F and s + 1 < N:
                        heapq.heappush(arrivals, (t_end + latency, seq, s + 1, A.ARB_F, j)); seq += 1
                    elif d == A.ARB_B and s > 0:
                        heapq.heappush(arrivals, (t_end + latency, seq, s - 1, A.ARB_B, j)); seq += 1
            while arrivals and arrivals[0][0] <= t:
                _, _, s, d, j = heapq.heappop(arrivals)
                A.arbiter_post_ready(self.arbiters[s], d, j, 0)
            all_done = True
            for s in range(N):
                if running[s] is not None:
                    all_done = False
                    continue
                rc, task = A.arbiter_next(self.arbiters[s])
                if rc == A.ARB_TASK:
                    d, j, _ = task
                    p = float(duration(d, s, j))
                    enqueue(s, d, j)
                    running[s] = (task, t + p)
                    trace.append((s, d, j, t, t + p))
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
            R.stage_grad_reduce(self.stages[s].handle, self.stages[s].grad_out, self.streams[s])
        torch.cuda.synchronize()
        return y[N - 1], dx[0], trace
