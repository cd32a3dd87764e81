"""Full-size GPU checks, in the launch configuration bench.py times (same stage_config, same
kernels and grids).  The oracle computes sampled microbatches of every bf16 workload at the size the
workload states (language: two microbatches; wide GQA: 2 layers, T = 4096; multimodal: depth 4 at
the largest token count of the seeded draw and a two-sample packed microbatch; vision); the other
full-size claims are properties that hold at any size: bit-identical results under two dispatch
orders (language and vision) and grad_out == the index-ordered fp32 sum of the slots."""
import time

import numpy as np
import pytest

import stage_inputs as SI
from tests import helpers as Hp

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def _say(msg):
    print(msg, flush=True)


def _run_one_mb(shape, cu, M_slots, mb, seed=SI.BASE_SEED):
    """F, B, W of microbatch `mb` on a stage created with M_slots slots; returns GPU and oracle results."""
    import torch
    import paper_2605_18750_amd as R
    from paper_2605_18750_amd import harness as Hn
    from oracle import stage_oracle as O
    t0 = time.time()
    w = Hp.Workload(shape, [cu], seed=seed)
    _say(f"  inputs generated in {time.time() - t0:.1f} s")
    T = int(cu[-1])
    cfg = Hn.make_config(shape, T, len(cu) - 1, n_microbatches=M_slots)
    stage = Hn.Stage(cfg, Hn.pack_params(cfg, w.layers))
    x = Hn.to_device(w.x[0].storage, shape.dtype)
    dy = Hn.to_device(w.dy[0].storage, shape.dtype)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    s = torch.cuda.Stream()
    R.stage_F(stage.handle, mb, x, cu, y, s)
    R.stage_B(stage.handle, mb, dy, dx, s)
    R.stage_W(stage.handle, mb, s)
    torch.cuda.synchronize()
    got = {"y": [Hn.to_f64(y)], "dx": [Hn.to_f64(dx)],
           "grads": [Hn.unpack_grads(cfg, stage.slot(mb).cpu().numpy())]}
    stage.close()
    del stage
    torch.cuda.empty_cache()
    t0 = time.time()
    ocfg = Hp.oracle_config(shape)
    params = w.oracle_params()
    yr, caches = O.stage_F(w.x[0].f64, params, cu, ocfg)
    dxr, gains, wst = O.stage_B(w.dy[0].f64, caches, params, ocfg)
    gr = O.merge_B_W(gains, O.stage_W(caches, wst, ocfg))
    _say(f"  oracle F+B+W in {time.time() - t0:.1f} s")
    ref = {"y": [yr], "dx": [dxr], "grads": [gr]}
    got["reduced"], ref["reduced"] = [], []
    return got, ref


def _compare_and_report(got, ref, what):
    """compare() at the bf16 tolerance; prints the largest per-tensor errors whether it passes or not."""
    rep = []
    try:
        worst = Hp.compare(got, ref, 2e-2, what, report=rep)
    finally:
        for name, e in sorted(rep, key=lambda t: -t[1])[:10]:
            _say(f"    {name}: {e:.3e}")
    _say(f"[full] {what}: worst rel err {worst:.3e}")
    return worst


@pytest.mark.parametrize("mb,seed", [(3, SI.BASE_SEED), (6, SI.BASE_SEED + 1)])
def test_language_stage_full_size_sampled_microbatch(mb, seed):
    """4 layers, hidden 4096, 32 heads x 128, FFN 11008, causal seq 4096, 8 slots; two sampled microbatches
    (slots 3 and 6) with different seeded inputs."""
    shape = SI.LANGUAGE
    _say(f"[full] language stage, microbatch {mb} of 8, T=4096, seed {seed}")
    got, ref = _run_one_mb(shape, np.array([0, SI.LANGUAGE_SEQ], dtype=np.int32), shape.n_microbatches, mb, seed)
    _compare_and_report(got, ref, f"language full size mb {mb}")


def test_wide_gqa_stage_full_size_sampled_microbatch():
    """The wide GQA stage as stated: 2 layers, hidden 8192, 64 query / 8 KV heads x 128, FFN 28672, causal
    seq 4096, 4 slots; microbatch 2."""
    shape = SI.WIDE_GQA
    _say("[full] wide GQA stage, 2 layers, microbatch 2 of 4, T=4096")
    got, ref = _run_one_mb(shape, np.array([0, SI.WIDE_SEQ], dtype=np.int32), shape.n_microbatches, 2)
    _compare_and_report(got, ref, "wide gqa full size")


def test_multimodal_stage_full_depth_largest_microbatch():
    """The multimodal stage as stated: 4 layers, 16 slots; the microbatch with the largest token count of the
    seeded draw (text uniform on [512, 2048] + image tokens from {256, 1024, 2304, 4096}), one causal segment."""
    shape = SI.MULTIMODAL
    text, img = SI.multimodal_lengths(shape)
    T_all = (text + img).astype(int)
    mb = int(np.argmax(T_all))
    _say(f"[full] multimodal stage, 4 layers, microbatch {mb} of 16, T={T_all[mb]} (text {text[mb]} + image {img[mb]})")
    assert T_all[mb] > 6000
    got, ref = _run_one_mb(shape, np.array([0, T_all[mb]], dtype=np.int32), shape.n_microbatches, mb)
    _compare_and_report(got, ref, "multimodal full depth, largest microbatch")


def test_multimodal_stage_full_depth_packed_two_samples():
    """Depth 4, two samples of the seeded draw packed into one microbatch (per-sample boundaries: attention
    must not cross the join), ragged lengths."""
    shape = SI.MULTIMODAL
    text, img = SI.multimodal_lengths(shape)
    a, b = int(text[1] + img[1]), int(text[4] + img[4])
    _say(f"[full] multimodal stage, 4 layers, packed microbatch {a} + {b} tokens")
    got, ref = _run_one_mb(shape, np.array([0, a, a + b], dtype=np.int32), shape.n_microbatches, 1)
    _compare_and_report(got, ref, "multimodal full depth, packed")


def test_vision_stage_full_size_sampled_microbatch():
    """8 bidirectional layers, hidden 1280, 16 heads x 80, GELU 5120, 8 images x 784 tokens."""
    shape = SI.VISION
    _say("[full] vision stage, microbatch 5 of 8, T=6272 in 8 segments")
    got, ref = _run_one_mb(shape, SI.default_cu_seqlens(shape), shape.n_microbatches, 5)
    worst = Hp.compare(got, ref, 2e-2, "vision full size")
    _say(f"[full] vision: worst rel err {worst:.3e}")


def _order_and_reduce_properties(shape, cu, order_seed):
    """All microbatches of a workload at full size (device-generated inputs, as in bench.py): a seeded random
    ready order on 3 streams gives y, dx, slots and grad_out bit-identical to the canonical order on one
    stream, and grad_out is exactly ((s0+s1)+s2)+... in fp32."""
    import torch
    import paper_2605_18750_amd as R
    from paper_2605_18750_amd import harness as Hn
    M, T = shape.n_microbatches, int(cu[-1])
    cfg = Hn.make_config(shape, T, len(cu) - 1)
    pb, gb, ab = R.stage_query(cfg)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(7)
    params = torch.empty(pb // 2, dtype=torch.bfloat16, device="cuda:0").normal_(0.0, 0.02, generator=gen)
    for l in range(cfg.n_layers):
        for which in (R.STAGE_P_G1, R.STAGE_P_G2):
            off, (r, _) = R.stage_param_layout(cfg, l, which)
            params[off:off + r] += 1.0
    arena = torch.empty(ab, dtype=torch.uint8, device="cuda:0")
    grad_out = torch.empty(gb // 4, dtype=torch.float32, device="cuda:0")
    st = R.stage_create(cfg, params, arena, ab)
    xs = [torch.empty((T, shape.hidden), dtype=torch.bfloat16, device="cuda:0").normal_(0, 1, generator=gen) for _ in range(M)]
    dys = [torch.empty((T, shape.hidden), dtype=torch.bfloat16, device="cuda:0").normal_(0, 1, generator=gen) for _ in range(M)]
    cu = [int(v) for v in cu]
    # tensor regions of a flat gradient buffer (padding between tensors is never written)
    regions = []
    for l in range(cfg.n_layers):
        for which in range(R.STAGE_P_COUNT):
            off, (r, c) = R.stage_param_layout(cfg, l, which)
            if r * c:
                regions.append((off, off + r * c))
    slot_off = [R.stage_grad_slot(st, j) - arena.data_ptr() for j in range(M)]

    def run(order, n_streams):
        ys = [torch.empty_like(x) for x in xs]
        dxs = [torch.empty_like(x) for x in xs]
        streams = [torch.cuda.Stream() for _ in range(n_streams)]
        for i, (kind, j) in enumerate(order):
            s = streams[i % n_streams]
            if kind == "F":
                R.stage_F(st, j, xs[j], cu, ys[j], s)
            elif kind == "B":
                R.stage_B(st, j, dys[j], dxs[j], s)
            else:
                R.stage_W(st, j, s)
        R.stage_grad_reduce(st, grad_out, streams[0])
        torch.cuda.synchronize()
        return ys, dxs

    _say("[full] canonical order, 1 stream")
    ys0, dxs0 = run(Hp.canonical_order(M), 1)
    assert all(bool(torch.isfinite(t.float()).all()) for t in ys0 + dxs0)
    # grad_out == index-ordered fp32 sum of the slots, region by region, bit for bit
    for (a, b) in regions:
        acc = arena[slot_off[0] + 4 * a: slot_off[0] + 4 * b].view(torch.float32).clone()
        for j in range(1, M):
            acc += arena[slot_off[j] + 4 * a: slot_off[j] + 4 * b].view(torch.float32)
        assert torch.equal(acc.view(torch.int32), grad_out[a:b].view(torch.int32)), "grad_out is not the index-ordered sum"
    keep_y = [t.clone() for t in ys0]
    keep_dx = [t.clone() for t in dxs0]
    keep_g = grad_out.clone()
    keep_slots = [arena[slot_off[j]: slot_off[j] + gb].clone() for j in range(M)] if gb * M < (8 << 30) else None
    order = SI.ready_order(M, order_seed)
    _say(f"[full] seeded ready order on 3 streams: {order}")
    ys1, dxs1 = run(order, 3)
    for a, b in zip(keep_y + keep_dx, ys1 + dxs1):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)), "y/dx differ between dispatch orders"
    for (a, b) in regions:
        assert torch.equal(keep_g[a:b].view(torch.int32), grad_out[a:b].view(torch.int32)), "grad_out differs between dispatch orders"
        if keep_slots is not None:
            for j in range(M):
                assert torch.equal(keep_slots[j][4 * a:4 * b], arena[slot_off[j] + 4 * a: slot_off[j] + 4 * b]), f"slot {j} differs"
    R.stage_destroy(st)


def test_language_stage_full_size_order_and_reduce_properties():
    _order_and_reduce_properties(SI.LANGUAGE, [0, SI.LANGUAGE_SEQ], 11)


def test_vision_stage_full_size_seeded_ready_order_is_bit_exact():
    """The vision workload as stated: 8 microbatches of 8 images x 784 tokens, split B/W tasks interleaved
    across microbatches in a seeded random ready order on 3 streams, against the canonical order."""
    order = SI.ready_order(SI.VISION.n_microbatches, 23)
    kinds = [k for k, _ in order]
    # the drawn order really interleaves: some W runs before another microbatch's F, some B before a later F
    assert kinds.index("W") < len(kinds) - 1 - kinds[::-1].index("F")
    _order_and_reduce_properties(SI.VISION, SI.default_cu_seqlens(SI.VISION), 23)
