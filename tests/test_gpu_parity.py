"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the same
seeded inputs.  Bar: max-norm relative error per tensor <= 1e-4 (fp32 path) / 2e-2 (bf16
path) for y, dx, every per-microbatch gradient tensor and the reduced gradients; bit-exact
across dispatch orders (paper Section 7.1: reordering must preserve training semantics)."""
import sys

import numpy as np
import pytest

import stage_inputs as SI
from tests import helpers as Hp

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


SMALL = {
    # fp32, odd hidden (scalar norm path), GQA, several segments, ragged tiles, causal
    "fp32_ragged_causal_gqa": (SI.StageShape("s_fp32_a", 2, 100, 4, 2, 16, 36, 3, dtype="fp32", x_std=1.0, dy_std=1.0, w_std=0.1),
                               [[0, 37, 150], [0, 70], [0, 1, 3, 131]]),
    # fp32, bidirectional + GELU, MQA
    "fp32_bidir_gelu_mqa": (SI.StageShape("s_fp32_b", 2, 64, 4, 1, 32, 48, 2, dtype="fp32", mlp_kind="gelu", causal=False,
                                          x_std=1.0, dy_std=1.0, w_std=0.1),
                            [[0, 65, 130], [0, 129]]),
    # bf16, causal SwiGLU, GQA, ragged
    "bf16_ragged_causal_gqa": (SI.StageShape("s_bf16_a", 2, 128, 4, 2, 64, 192, 3, w_std=0.05),
                               [[0, 200], [0, 77, 333], [0, 64]]),
    # bf16, bidirectional GELU, head_dim 80
    "bf16_bidir_gelu_d80": (SI.StageShape("s_bf16_b", 2, 320, 4, 4, 80, 256, 2, mlp_kind="gelu", causal=False, w_std=0.05),
                            [[0, 100, 200, 300], [0, 259]]),
    # bf16 degenerate lengths: a single token, single-token segments, one row past a query tile
    "bf16_single_tokens": (SI.StageShape("s_bf16_d", 1, 128, 4, 2, 64, 192, 3, w_std=0.05),
                           [[0, 1], [0, 1, 2, 3], [0, 257]]),
    # fp32 degenerate lengths
    "fp32_single_tokens": (SI.StageShape("s_fp32_c", 1, 64, 2, 1, 32, 48, 3, dtype="fp32", x_std=1.0, dy_std=1.0, w_std=0.1),
                           [[0, 1], [0, 1, 2, 3], [0, 65]]),
    # rotary position embedding variant: bf16 d = 128 GQA ragged causal; fp32 d = 32 bidirectional GELU
    "bf16_rope_d128": (SI.StageShape("s_bf16_rope", 2, 512, 4, 2, 128, 320, 3, w_std=0.03, rope=True),
                       [[0, 300], [0, 130, 391], [0, 5]]),
    "bf16_rope_d80": (SI.StageShape("s_bf16_rope80", 1, 320, 4, 4, 80, 256, 2, mlp_kind="gelu", causal=False, w_std=0.05,
                                    rope=True, rope_base=500.0),
                      [[0, 100, 200, 300], [0, 259]]),
    "fp32_rope": (SI.StageShape("s_fp32_rope", 2, 64, 2, 1, 32, 48, 2, dtype="fp32", mlp_kind="gelu", causal=False,
                                x_std=1.0, dy_std=1.0, w_std=0.1, rope=True),
                  [[0, 65, 130], [0, 129]]),
    # LayerNorm + projection biases (GPT / ViT style layers): bf16 GELU bidirectional d = 80 (vision-like),
    # bf16 SwiGLU causal with rope on top, fp32 GELU
    "bf16_layernorm_bias_gelu": (SI.StageShape("s_bf16_ln", 2, 320, 4, 4, 80, 256, 2, mlp_kind="gelu", causal=False, w_std=0.05,
                                               norm_kind="layer", bias=True),
                                 [[0, 100, 200, 300], [0, 259]]),
    "bf16_layernorm_bias_swiglu_rope": (SI.StageShape("s_bf16_ln2", 2, 512, 4, 2, 128, 384, 2, w_std=0.03,
                                                      norm_kind="layer", bias=True, rope=True),
                                        [[0, 300], [0, 130, 391]]),
    "bf16_qk_norm_rope": (SI.StageShape("s_bf16_qkn", 2, 512, 4, 2, 128, 384, 2, w_std=0.03, qk_norm=True, rope=True),
                          [[0, 130, 300], [0, 257]]),
    "bf16_qk_norm_d80_bias": (SI.StageShape("s_bf16_qkn80", 1, 320, 4, 4, 80, 256, 2, mlp_kind="gelu", causal=False, w_std=0.05,
                                            qk_norm=True, bias=True), [[0, 96, 97], [0, 301]]),
    "fp32_qk_norm": (SI.StageShape("s_fp32_qkn", 2, 100, 4, 2, 16, 36, 2, dtype="fp32", x_std=1.0, dy_std=1.0, qk_norm=True,
                                   rope=True), [[0, 50, 130], [0, 33]]),
    "bf16_bias_only": (SI.StageShape("s_bf16_b", 1, 128, 4, 2, 64, 192, 2, w_std=0.05, bias=True), [[0, 200], [0, 77, 333]]),
    "fp32_layernorm_bias": (SI.StageShape("s_fp32_ln", 2, 100, 4, 2, 16, 36, 2, dtype="fp32", mlp_kind="gelu", x_std=1.0, dy_std=1.0,
                                          w_std=0.1, norm_kind="layer", bias=True),
                            [[0, 37, 150], [0, 70]]),
    # bf16, many tokens on a narrow stage: the weight-gradient GEMMs (K = tokens) take the split-K path
    "bf16_long_tokens_splitk": (SI.StageShape("s_bf16_e", 1, 128, 4, 2, 64, 192, 2, w_std=0.05),
                                [[0, 1100], [0, 600, 1163]]),
    # bf16, head_dim 128, GQA 4:1
    "bf16_d128_gqa4": (SI.StageShape("s_bf16_c", 1, 512, 4, 1, 128, 320, 2, w_std=0.03),
                       [[0, 300], [0, 130, 260]]),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_small_stage_matches_oracle(name):
    shape, cus = SMALL[name]
    _say(f"[parity] {name}: {shape}")
    w = Hp.Workload(shape, cus)
    ref = Hp.run_oracle(w)
    got = Hp.run_gpu(w)
    worst = Hp.compare(got, ref, Hp.TOL[shape.dtype], name)
    _say(f"[parity] {name}: worst rel err {worst:.3e} (tol {Hp.TOL[shape.dtype]})")


def test_tiny_fp32_config_matches_oracle():
    """The tiny fp32 configuration at its full size: 1 layer, hidden 256, 4 heads of 64, FFN 688,
    seq 128, 4 microbatches, everything N(0, 0.02)."""
    shape = SI.TINY
    w = Hp.Workload(shape, [SI.default_cu_seqlens(shape, j) for j in range(shape.n_microbatches)])
    _say(f"[parity] tiny fp32 full config")
    ref = Hp.run_oracle(w)
    got = Hp.run_gpu(w)
    worst = Hp.compare(got, ref, 1e-4, "tiny")
    _say(f"[parity] tiny: worst rel err {worst:.3e}")


@pytest.mark.parametrize("name", ["fp32_ragged_causal_gqa", "bf16_ragged_causal_gqa", "bf16_bidir_gelu_d80", "bf16_rope_d128",
                                  "bf16_long_tokens_splitk", "bf16_layernorm_bias_gelu", "bf16_qk_norm_rope"])
def test_dispatch_order_is_bit_exact(name):
    shape, cus = SMALL[name]
    w = Hp.Workload(shape, cus)
    _say(f"[order] {name}: canonical order, one stream")
    base = Hp.run_gpu(w, keep_raw=True)
    for seed in (1, 2):
        order = SI.ready_order(w.M, seed)
        _say(f"[order] {name}: seed {seed} order {order} on 3 streams")
        other = Hp.run_gpu(w, order=order, n_streams=3, keep_raw=True)
        Hp.assert_bit_identical(base, other)


def test_second_iteration_reuses_slots_and_matches():
    """Two iterations on one handle (slots are recycled by stage_grad_reduce): same results."""
    import torch
    import paper_2605_18750_amd as R
    from paper_2605_18750_amd import harness as Hn
    shape, cus = SMALL["bf16_ragged_causal_gqa"]
    w = Hp.Workload(shape, cus)
    cfg = Hn.make_config(shape, 333, 2, n_microbatches=w.M)
    stage = Hn.Stage(cfg, Hn.pack_params(cfg, w.layers))
    xs = [Hn.to_device(t.storage, shape.dtype) for t in w.x]
    dys = [Hn.to_device(t.storage, shape.dtype) for t in w.dy]
    results = []
    for it in range(2):
        ys = [torch.empty_like(x) for x in xs]
        dxs = [torch.empty_like(x) for x in xs]
        s = torch.cuda.Stream()
        order = Hp.canonical_order(w.M) if it == 0 else SI.ready_order(w.M, 9)
        _say(f"[iter {it}] order {order}")
        for kind, j in order:
            if kind == "F":
                R.stage_F(stage.handle, j, xs[j], w.cus[j], ys[j], s)
            elif kind == "B":
                R.stage_B(stage.handle, j, dys[j], dxs[j], s)
            else:
                R.stage_W(stage.handle, j, s)
        R.stage_grad_reduce(stage.handle, stage.grad_out, s)
        torch.cuda.synchronize()
        results.append(([y.cpu() for y in ys], [d.cpu() for d in dxs], stage.grad_out.cpu().clone()))
    for a, b in zip(results[0][0] + results[0][1], results[1][0] + results[1][1]):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    ga = Hn.unpack_grads(cfg, results[0][2].numpy().view(np.int32))
    gb = Hn.unpack_grads(cfg, results[1][2].numpy().view(np.int32))
    for la, lb in zip(ga, gb):
        for k in la:
            assert np.array_equal(la[k], lb[k]), k
    stage.close()


@pytest.mark.parametrize("log2_scale", [-24, 18])
def test_backward_is_exactly_homogeneous_in_the_output_gradient(log2_scale):
    """B and W are linear in dy.  The bf16 path keeps its attention-internal copy of dO as IEEE halves behind a
    per-microbatch power-of-two scale taken from max|dy|, so multiplying dy by 2^k (exact in bf16) must multiply
    dx and every gradient by 2^k EXACTLY: with gradients of order 1e-7 (an un-scaled mean loss) or 1e+5 the half
    copy would otherwise lose its digits or overflow.  The scaled run is also compared with the oracle."""
    import torch
    import paper_2605_18750_amd as R
    from paper_2605_18750_amd import harness as Hn
    shape, cus = SMALL["bf16_ragged_causal_gqa"]
    w = Hp.Workload(shape, cus)
    cfg = Hn.make_config(shape, 333, 2, n_microbatches=w.M)
    stage = Hn.Stage(cfg, Hn.pack_params(cfg, w.layers))
    xs = [Hn.to_device(t.storage, shape.dtype) for t in w.x]
    factor = 2.0 ** log2_scale
    runs = []
    for f in (1.0, factor):
        dys = [Hn.to_device(t.storage, shape.dtype) * f for t in w.dy]      # exact: a power of two
        ys = [torch.empty_like(x) for x in xs]
        dxs = [torch.empty_like(x) for x in xs]
        _say(f"[homogeneous] dy x 2^{0 if f == 1.0 else log2_scale}")
        for j in range(w.M):
            R.stage_F(stage.handle, j, xs[j], w.cus[j], ys[j])
        for j in range(w.M):
            R.stage_B(stage.handle, j, dys[j], dxs[j])
            R.stage_W(stage.handle, j)
        R.stage_grad_reduce(stage.handle, stage.grad_out)
        torch.cuda.synchronize()
        runs.append(([d.float().cpu() for d in dxs], stage.grad_out.cpu().clone()))
    (dx1, g1), (dx2, g2) = runs
    for a, b in zip(dx1, dx2):
        assert torch.equal(a * factor, b), "dx is not exactly homogeneous in dy"
    assert torch.equal(g1 * factor, g2), "the gradients are not exactly homogeneous in dy"
    assert float(g1.abs().max()) > 0
    # and the scaled run against the oracle (linear in dy as well)
    ref = Hp.run_oracle(w)
    got_red = Hn.unpack_grads(cfg, (g2 / factor).numpy())
    worst = Hp.compare({"y": [], "dx": [Hn.to_f64(d / factor) for d in dx2], "grads": [], "reduced": got_red},
                       {"y": [], "dx": ref["dx"], "grads": [], "reduced": ref["reduced"]}, 2e-2, f"dy x 2^{log2_scale}")
    _say(f"[homogeneous] 2^{log2_scale}: exact; against the oracle {worst:.3e}")
    stage.close()
