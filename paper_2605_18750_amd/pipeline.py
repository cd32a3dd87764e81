"""A miniature of the runtime of Sec. 4.1 / Sec. 5 on ONE GPU: N stage handles chained into a pipeline,
one HIP stream per stage, and messages (tensor, microbatch id, direction) between neighbours.  Which task
every stage dispatches, when, and whose output it consumes is decided by the native event loop of the
library (rrfp_pipe_* of include/rrfp_arbiter.h: one ready-set arbiter per stage, message routing, virtual
clock); the tasks themselves are the stage_F / stage_B / stage_W calls of the library.  This module only
keeps the tensors and HIP events that go with the dispatches.

All stages share one device here, so wall-clock readiness would just mirror the enqueue order.  The loop
therefore runs on a VIRTUAL clock: a message becomes visible to the receiving arbiter at the sender's
completion + latency on that clock, and a task's duration is either given by the caller or MEASURED (HIP
events around the task on its stream).  The GPU work is enqueued at dispatch on the stage's own stream;
data dependencies between stages are enforced with HIP events recorded by the producer and waited on by
the consumer stream, so the device executes a valid order whatever the virtual clock says.  With a jitter
level (Sec. 7.6) the library draws the delay of each F / B task from its measured time and the delay is
put behind the task on its stream as a device-side sleep (rrfp_delay).  No arithmetic of the method lives
here.
"""
from __future__ import annotations

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
        self.buffer_limit = buffer_limit
        if hint != A.ARB_HINT_BFW:
            raise ValueError("the stage library needs W tasks before the reduce: use the BFW hint")
        self.streams = [torch.cuda.Stream() for _ in range(self.N)]

    def close(self):
        pass

    def run_iteration(self, xs, dys, duration=None, latency: float = 0.0, jitter=(0.0, 0.0, 0.0, 0)):
        """xs[j]: input of microbatch j to (stage 0, chunk 0); dys[j]: gradient w.r.t. the output of
        (stage N-1, chunk C-1).  duration(dir, stage, microbatch, chunk) -> virtual seconds, or None to
        measure every task with HIP events on its stream (the host then waits for each task).
        jitter = (p, base seconds, alpha, seed) of Sec. 7.6.  Returns (final outputs, input gradients,
        trace) with trace = [(stage, dir, microbatch, chunk, start, end)] in dispatch order; the reduced
        gradients are in each Stage's grad_out; self.delays lists (stage, dir, microbatch, chunk, compute
        seconds, injected delay seconds) for every task in dispatch order (W tasks are never delayed)."""
        torch = self.torch
        N, M, C = self.N, self.M, self.C
        y, dx, ev = {}, {}, {}
        trace = []
        self.delays = []
        pipe = A.rrfp_pipe_create(N, M, C, self.hint, self.buffer_limit, latency, jitter)
        try:
            while True:
                rc, disp = A.rrfp_pipe_next(pipe)
                if rc == A.ARB_DONE:
                    break
                s, d, j, c, src_s, src_c, start = disp
                st, stream = self.stages[s][c], self.streams[s]
                t0 = t1 = None
                if duration is None:
                    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                if d == A.ARB_W:
                    if t0 is not None:
                        t0.record(stream)
                    R.stage_W(st.handle, j, stream)
                else:
                    store = y if d == A.ARB_F else dx
                    if src_s < 0:
                        inp = xs[j] if d == A.ARB_F else dys[j]
                    else:
                        inp = store[(src_s, src_c, j)]
                        stream.wait_event(ev[(d, src_s, src_c, j)])
                    out = torch.empty_like(inp)
                    store[(s, c, j)] = out
                    if t0 is not None:
                        t0.record(stream)
                    if d == A.ARB_F:
                        R.stage_F(st.handle, j, inp, self.cus[j], out, stream)
                    else:
                        R.stage_B(st.handle, j, inp, out, stream)
                if t1 is not None:
                    t1.record(stream)
                    t1.synchronize()
                    seconds = t0.elapsed_time(t1) * 1e-3
                else:
                    seconds = float(duration(d, s, j, c))
                delay, end = A.rrfp_pipe_set_duration(pipe, seconds)
                if d != A.ARB_W:
                    if delay > 0.0:      # the device-side sleep sits behind the task, before its "sent" event
                        A.rrfp_delay(min(delay, 1.0), stream)
                    e = torch.cuda.Event()
                    e.record(stream)
                    ev[(d, s, c, j)] = e
                self.delays.append((s, d, j, c, seconds, delay))
                trace.append((s, d, j, c, start, end))
        finally:
            A.rrfp_pipe_destroy(pipe)
        for s in range(N):
            for c in range(C):
                R.stage_grad_reduce(self.stages[s][c].handle, self.stages[s][c].grad_out, self.streams[s])
        torch.cuda.synchronize()
        return [y[(N - 1, C - 1, j)] for j in range(M)], [dx[(0, 0, j)] for j in range(M)], trace
