"""Thin ctypes binding of the arbiter and simulator entry points of include/rrfp_arbiter.h:
argument marshalling only, the decisions and the event loop run in the native library."""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import lib as _stage_lib

ARB_F, ARB_B, ARB_W = 0, 1, 2
ARB_HINT_BF, ARB_HINT_FB, ARB_HINT_B_PRIO, ARB_HINT_F_PRIO, ARB_HINT_BFW, ARB_HINT_FIXED_1F1B = range(6)
ARB_OK, ARB_WAIT, ARB_TASK, ARB_DONE, ARB_EINVAL, ARB_ESTATE = 0, 0, 1, 2, -1, -2
HINT_NAMES = {"bf": ARB_HINT_BF, "fb": ARB_HINT_FB, "b-prio": ARB_HINT_B_PRIO, "f-prio": ARB_HINT_F_PRIO,
              "bfw": ARB_HINT_BFW, "1f1b": ARB_HINT_FIXED_1F1B}


class arbiter_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_microbatches", "n_chunks", "hint", "buffer_limit", "stage", "n_stages")]


class arbiter_task(C.Structure):
    _fields_ = [("dir", C.c_int32), ("microbatch", C.c_int32), ("chunk", C.c_int32)]


class rrfp_sim_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_stages", "n_microbatches", "n_chunks", "hint", "buffer_limit", "mode")] + [
        ("latency", C.c_double), ("jitter_p", C.c_double), ("jitter_base", C.c_double), ("jitter_alpha", C.c_double),
        ("jitter_seed", C.c_uint64)]


class rrfp_sim_event(C.Structure):
    _fields_ = [("stage", C.c_int32), ("dir", C.c_int32), ("microbatch", C.c_int32), ("chunk", C.c_int32),
                ("start", C.c_double), ("end", C.c_double)]


class rrfp_pipe_dispatch(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("stage", "dir", "microbatch", "chunk", "src_stage", "src_chunk")] + [
        ("start", C.c_double)]


class rrfp_sim_result(C.Structure):
    _fields_ = [("makespan", C.c_double), ("n_events", C.c_int64), ("deadlock", C.c_int32)]


class ArbiterError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"arbiter error {code}: {msg}")
        self.code = code


_ready = False


def _lib():
    global _ready
    L = _stage_lib()
    if not _ready:
        vp = C.c_void_p
        L.arbiter_create.argtypes = [C.POINTER(arbiter_config)]
        L.arbiter_create.restype = vp
        L.arbiter_destroy.argtypes = [vp]
        L.arbiter_destroy.restype = None
        L.arbiter_reset.argtypes = [vp]
        L.arbiter_post_ready.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32]
        L.arbiter_next.argtypes = [vp, C.POINTER(arbiter_task)]
        L.arbiter_complete.argtypes = [vp, C.POINTER(arbiter_task)]
        L.arbiter_counters.argtypes = [vp, C.POINTER(C.c_int64)]
        L.arbiter_last_error.argtypes = [vp]
        L.arbiter_last_error.restype = C.c_char_p
        L.rrfp_sim_run.argtypes = [C.POINTER(rrfp_sim_config), vp, vp, vp, C.POINTER(rrfp_sim_result), vp,
                                   C.POINTER(rrfp_sim_event), C.c_int64]
        L.rrfp_pipe_create.argtypes = [C.POINTER(rrfp_sim_config)]
        L.rrfp_pipe_create.restype = vp
        L.rrfp_pipe_destroy.argtypes = [vp]
        L.rrfp_pipe_destroy.restype = None
        L.rrfp_pipe_next.argtypes = [vp, C.POINTER(rrfp_pipe_dispatch)]
        L.rrfp_pipe_next.restype = C.c_int
        L.rrfp_pipe_set_duration.argtypes = [vp, C.c_double, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.rrfp_pipe_set_duration.restype = C.c_int
        L.jitter_create.argtypes = [C.c_double, C.c_double, C.c_double, C.c_uint64, C.c_int32, C.c_int32, C.c_int32]
        L.jitter_create.restype = vp
        L.jitter_destroy.argtypes = [vp]
        L.jitter_destroy.restype = None
        L.jitter_next_delay.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_double]
        L.jitter_next_delay.restype = C.c_double
        L.rrfp_delay.argtypes = [C.c_double, vp]
        L.rrfp_delay.restype = C.c_int
        L.rrfp_delay_last_error.argtypes = []
        L.rrfp_delay_last_error.restype = C.c_char_p
        for f in ("arbiter_reset", "arbiter_post_ready", "arbiter_next", "arbiter_complete", "arbiter_counters",
                  "rrfp_sim_run"):
            getattr(L, f).restype = C.c_int
        _ready = True
    return L


def arbiter_last_error(a=None) -> str:
    return (_lib().arbiter_last_error(a) or b"").decode()


def _check(rc: int, a=None) -> int:
    if rc < 0:
        raise ArbiterError(rc, arbiter_last_error(a))
    return rc


def arbiter_create(n_microbatches: int, n_chunks: int = 1, hint: int = ARB_HINT_BF, buffer_limit: int = 0,
                   stage: int = 0, n_stages: int = 1):
    cfg = arbiter_config(n_microbatches, n_chunks, hint, buffer_limit, stage, n_stages)
    a = _lib().arbiter_create(C.byref(cfg))
    if not a:
        raise ArbiterError(ARB_EINVAL, arbiter_last_error(None))
    return a


def arbiter_destroy(a):
    _lib().arbiter_destroy(a)


def arbiter_reset(a):
    _check(_lib().arbiter_reset(a), a)


def arbiter_post_ready(a, direction: int, microbatch: int, chunk: int = 0):
    _check(_lib().arbiter_post_ready(a, direction, microbatch, chunk), a)


def arbiter_next(a):
    """(ARB_TASK, (dir, microbatch, chunk)) | (ARB_WAIT, None) | (ARB_DONE, None)."""
    t = arbiter_task()
    rc = _check(_lib().arbiter_next(a, C.byref(t)), a)
    return (rc, (t.dir, t.microbatch, t.chunk)) if rc == ARB_TASK else (rc, None)


def arbiter_complete(a, task):
    t = arbiter_task(*task)
    _check(_lib().arbiter_complete(a, C.byref(t)), a)


def arbiter_counters(a):
    out = (C.c_int64 * 5)()
    _check(_lib().arbiter_counters(a, out), a)
    return {"n_f": out[0], "n_b": out[1], "n_w": out[2], "backpressure": bool(out[3]), "completed": out[4]}


def rrfp_sim_run(n_stages: int, n_microbatches: int, dur_f, dur_b, dur_w=None, *, n_chunks: int = 1,
                 hint: int = ARB_HINT_BF, buffer_limit: int = 0, mode: int = 0, latency: float = 0.0,
                 jitter=(0.0, 0.0, 0.0, 0), want_trace: bool = True):
    """dur_* : float64 arrays [stage][chunk][microbatch].  Returns a dict with makespan, deadlock,
    per-stage busy / peak buffers / peak D, and (optionally) the trace as a structured array."""
    N, M, Cc = n_stages, n_microbatches, n_chunks
    arrs = []
    for d in (dur_f, dur_b, dur_w):
        if d is None:
            arrs.append(None)
            continue
        a = np.ascontiguousarray(d, dtype=np.float64).reshape(N, Cc, M)
        arrs.append(a)
    cfg = rrfp_sim_config(N, M, Cc, hint, buffer_limit, mode, latency, jitter[0], jitter[1], jitter[2], jitter[3])
    res = rrfp_sim_result()
    per_stage = np.zeros((N, 4), dtype=np.float64)
    cap = (3 if hint == ARB_HINT_BFW else 2) * N * M * Cc if want_trace else 0
    trace = (rrfp_sim_event * max(cap, 1))()
    ptr = lambda a: None if a is None else a.ctypes.data_as(C.c_void_p)
    _check(_lib().rrfp_sim_run(C.byref(cfg), ptr(arrs[0]), ptr(arrs[1]), ptr(arrs[2]), C.byref(res),
                               per_stage.ctypes.data_as(C.c_void_p), trace if want_trace else None, cap))
    out = {"makespan": res.makespan, "deadlock": bool(res.deadlock), "n_events": res.n_events,
           "busy": per_stage[:, 0].copy(), "max_fwd_buffer": per_stage[:, 1].astype(int),
           "max_bwd_buffer": per_stage[:, 2].astype(int), "max_D": per_stage[:, 3].astype(int)}
    if want_trace:
        n = min(res.n_events, cap)
        out["trace"] = [(e.stage, e.dir, e.microbatch, e.chunk, e.start, e.end) for e in trace[:n]]
    return out


def rrfp_pipe_create(n_stages: int, n_microbatches: int, n_chunks: int = 1, hint: int = ARB_HINT_BFW,
                     buffer_limit: int = 0, latency: float = 0.0, jitter=(0.0, 0.0, 0.0, 0)):
    """The pipeline event loop as an object; jitter = (p, base seconds, alpha, seed)."""
    cfg = rrfp_sim_config(n_stages, n_microbatches, n_chunks, hint, buffer_limit, 0, latency,
                          jitter[0], jitter[1], jitter[2], jitter[3])
    p = _lib().rrfp_pipe_create(C.byref(cfg))
    if not p:
        raise ArbiterError(ARB_EINVAL, arbiter_last_error(None))
    return p


def rrfp_pipe_destroy(p):
    _lib().rrfp_pipe_destroy(p)


def rrfp_pipe_next(p):
    """(ARB_TASK, dispatch) with dispatch = (stage, dir, microbatch, chunk, src_stage, src_chunk, start),
    or (ARB_DONE, None)."""
    d = rrfp_pipe_dispatch()
    rc = _check(_lib().rrfp_pipe_next(p, C.byref(d)))
    if rc == ARB_TASK:
        return rc, (d.stage, d.dir, d.microbatch, d.chunk, d.src_stage, d.src_chunk, d.start)
    return rc, None


def rrfp_pipe_set_duration(p, seconds: float):
    """-> (injected delay in seconds, virtual completion time) of the task rrfp_pipe_next returned last."""
    delay, end = C.c_double(), C.c_double()
    _check(_lib().rrfp_pipe_set_duration(p, seconds, C.byref(delay), C.byref(end)))
    return delay.value, end.value


def jitter_create(p: float, base_seconds: float, alpha: float, seed: int, stage: int, n_microbatches: int,
                  n_chunks: int = 1):
    j = _lib().jitter_create(p, base_seconds, alpha, seed, stage, n_microbatches, n_chunks)
    if not j:
        raise ArbiterError(ARB_EINVAL, arbiter_last_error(None))
    return j


def jitter_destroy(j):
    _lib().jitter_destroy(j)


def jitter_next_delay(j, direction: int, microbatch: int, chunk: int, compute_seconds: float) -> float:
    return _lib().jitter_next_delay(j, direction, microbatch, chunk, compute_seconds)


def rrfp_delay(seconds: float, stream=None):
    """Enqueues the device-side sleep on `stream` (a torch stream, a raw handle, or None)."""
    h = 0 if stream is None else getattr(stream, "cuda_stream", stream)
    rc = _lib().rrfp_delay(seconds, h)
    if rc < 0:
        raise ArbiterError(rc, (_lib().rrfp_delay_last_error() or b"").decode())
