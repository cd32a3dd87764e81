"""Step-by-step parity: every tensor a task keeps per microbatch and layer (stage_intermediate) against the
oracle's value of the same tensor, so that the error of each step of the F and B tasks is seen on its own
(RMSNorm, QKV projection, attention and its log-sum-exp, output projection + residual, gate|up projection,
activation, and in B the activation backward, the norm backward, the attention backward)."""
import numpy as np
import pytest

import stage_inputs as SI
from tests import helpers as Hp

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _lse(q, k, cu, cfg):
    """log sum_j exp(q_i . k_j / sqrt(d)) over the allowed keys of row i, per query head: [n_q, T]."""
    nq, nkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    T = q.shape[0]
    out = np.empty((nq, T))
    for s, e in zip(cu[:-1], cu[1:]):
        for a in range(nq):
            b = a // (nq // nkv)
            S = q[s:e, a * d:(a + 1) * d] @ k[s:e, b * d:(b + 1) * d].T / np.sqrt(float(d))
            if cfg.causal:
                S = np.where(np.tril(np.ones(S.shape, dtype=bool)), S, -np.inf)
            mx = S.max(axis=1, keepdims=True)
            out[a, s:e] = (mx + np.log(np.exp(S - mx).sum(axis=1, keepdims=True))).reshape(-1)
    return out


@pytest.mark.parametrize("name,shape,cu", [
    ("swiglu_gqa_d128", SI.StageShape("inter_a", 2, 512, 8, 2, 128, 768, 2, w_std=0.04), [0, 300, 777]),
    ("gelu_d80_bidir", SI.StageShape("inter_b", 2, 320, 4, 4, 80, 640, 2, mlp_kind="gelu", causal=False, w_std=0.05), [0, 260, 530]),
])
def test_every_stashed_tensor_against_the_oracle(name, shape, cu):
    import torch
    import paper_2605_18750_amd as R
    from paper_2605_18750_amd import harness as Hn
    from oracle import stage_oracle as O
    cu = np.asarray(cu, dtype=np.int32)
    T = int(cu[-1])
    w = Hp.Workload(shape, [cu])
    cfg = Hn.make_config(shape, T, len(cu) - 1, n_microbatches=2)
    stage = Hn.Stage(cfg, Hn.pack_params(cfg, w.layers))
    x = Hn.to_device(w.x[0].storage, "bf16")
    dy = Hn.to_device(w.dy[0].storage, "bf16")
    y, dx = torch.empty_like(x), torch.empty_like(x)
    mb = 1
    _say(f"[inter] {name}: F, B on slot {mb}")
    R.stage_F(stage.handle, mb, x, cu, y)
    R.stage_B(stage.handle, mb, dy, dx)
    torch.cuda.synchronize()
    ocfg = Hp.oracle_config(shape)
    params = w.oracle_params()
    _, caches = O.stage_F(w.x[0].f64, params, cu, ocfg)
    _, _, wst = O.stage_B(w.dy[0].f64, caches, params, ocfg)
    worst = {}
    swiglu = shape.mlp_kind == "swiglu"
    for l in range(shape.n_layers):
        c, b = caches[l], wst[l]
        ref = {
            R.STAGE_T_X: c["x"], R.STAGE_T_H1: c["h1"], R.STAGE_T_QKV: np.concatenate([c["q"], c["k"], c["v"]], axis=1),
            R.STAGE_T_O: c["o"], R.STAGE_T_X1: c["x1"], R.STAGE_T_H2: c["h2"],
            R.STAGE_T_UP: np.concatenate([c["gt"], c["up"]], axis=1) if swiglu else c["u"], R.STAGE_T_M: c["m"],
            R.STAGE_T_DY: b["dy"], R.STAGE_T_DUP: np.concatenate([b["dgt"], b["dup"]], axis=1) if swiglu else b["du"],
            R.STAGE_T_DX1: b["dx1"], R.STAGE_T_DQKV: np.concatenate([b["dq"], b["dk"], b["dv"]], axis=1),
            R.STAGE_T_LSE: _lse(c["q"], c["k"], cu, ocfg), R.STAGE_T_H1_HALF: c["h1"],
        }
        names = {R.STAGE_T_X: "x", R.STAGE_T_H1: "h1", R.STAGE_T_QKV: "qkv", R.STAGE_T_O: "o", R.STAGE_T_X1: "x1",
                 R.STAGE_T_H2: "h2", R.STAGE_T_UP: "up", R.STAGE_T_M: "m", R.STAGE_T_DY: "dy", R.STAGE_T_DUP: "dup",
                 R.STAGE_T_DX1: "dx1", R.STAGE_T_DQKV: "dqkv", R.STAGE_T_LSE: "lse", R.STAGE_T_H1_HALF: "h1h"}
        for which, r in ref.items():
            got = Hn.to_f64(stage.intermediate(mb, l, which, T))
            assert got.shape == r.shape, (names[which], got.shape, r.shape)
            e = Hp.max_norm_rel_err(got, r)
            worst[(l, names[which])] = e
            _say(f"[inter] {name} layer {l} {names[which]:5s}: {e:.3e}")
    # one storage rounding is 2^-9 = 2e-3 of the value; the bound of the path applies to every step
    for key, e in worst.items():
        assert e <= 2e-2, (name, key, e)
    # the first step of each task sees only the rounding of its own output
    for key in ((0, "h1"), (shape.n_layers - 1, "dy")):
        assert worst[key] <= 4e-3, (name, key, worst[key])
    # the IEEE-half copies on the path into the scores round to 2^-12: h1 as the QKV projection reads it, q|k|v
    assert worst[(0, "h1h")] <= 5e-4 and worst[(0, "qkv")] <= 1e-3, (name, worst[(0, "h1h")], worst[(0, "qkv")])
    assert worst[(0, "x")] == 0.0          # the widened input is exact
    stage.close()
