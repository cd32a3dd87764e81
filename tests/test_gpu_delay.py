"""The device-side sleep of the jitter protocol (Sec. 7.6): timed with HIP events on its stream, it
lasts at least the requested time and not much longer, and rejects requests outside [0, 1] s."""
import sys

import pytest

pytestmark = pytest.mark.gpu


def test_delay_kernel_sleeps_for_the_requested_time():
    import torch
    from paper_2605_18750_amd import arbiter as A
    s = torch.cuda.Stream()
    A.rrfp_delay(1e-4, s)                      # warm-up (module load)
    torch.cuda.synchronize()
    for want_ms in (0.5, 2.0, 10.0):
        print(f"[delay] {want_ms} ms", flush=True)
        sys.stdout.flush()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(s)
        A.rrfp_delay(want_ms * 1e-3, s)
        e1.record(s)
        torch.cuda.synchronize()
        got = e0.elapsed_time(e1)
        assert got >= want_ms * 0.98, (want_ms, got)
        assert got <= want_ms * 1.1 + 0.2, (want_ms, got)
    with pytest.raises(A.ArbiterError):
        A.rrfp_delay(1.5, s)
    with pytest.raises(A.ArbiterError):
        A.rrfp_delay(-1.0, s)
