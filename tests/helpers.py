"""Shared by the tests: runs the same seeded workload through the oracle and through the
HIP library (via the C ABI binding) and compares them with the max-norm relative error."""
from __future__ import annotations

import numpy as np

import stage_inputs as SI
from oracle import stage_oracle as O

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def oracle_config(shape: SI.StageShape) -> O.OracleConfig:
    return O.OracleConfig(n_layers=shape.n_layers, hidden=shape.hidden, n_q_heads=shape.n_q_heads,
                          n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn,
                          mlp_kind=shape.mlp_kind, causal=shape.causal, norm_eps=shape.norm_eps,
                          rope=shape.rope, rope_base=shape.rope_base, norm_kind=shape.norm_kind, bias=shape.bias, qk_norm=shape.qk_norm)


def max_norm_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max|got - ref| / max|ref| over one tensor."""
    den = float(np.max(np.abs(ref)))
    num = float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref)))
    return num / den if den > 0 else num


class Workload:
    """Seeded inputs of one stage: parameters, and x / dy / cu_seqlens per microbatch."""

    def __init__(self, shape: SI.StageShape, cus: list, seed: int = SI.BASE_SEED):
        self.shape = shape
        self.cus = [np.asarray(c, dtype=np.int32) for c in cus]
        self.M = len(cus)
        if shape.hidden >= 1024:     # big stages: generate the tensors on a thread pool (numpy releases the GIL)
            from concurrent.futures import ThreadPoolExecutor
            jobs = [(l, nm, shp) for l in range(shape.n_layers) for nm, shp in SI.layer_param_shapes(shape).items()]

            def gen(job):
                l, nm, shp = job
                return SI.make_tensor(seed, f"{shape.name}/L{l}/{nm}", shp, shape.w_std, shape.dtype,
                                      mean=1.0 if nm in ("g1", "g2") else 0.0)
            with ThreadPoolExecutor(max_workers=8) as ex:
                out = list(ex.map(gen, jobs))
            self.layers = [dict() for _ in range(shape.n_layers)]
            for (l, nm, _), t in zip(jobs, out):
                self.layers[l][nm] = t
        else:
            self.layers = SI.make_stage_params(shape, seed)
        self.x = [SI.make_x(shape, j, int(c[-1]), seed) for j, c in enumerate(self.cus)]
        self.dy = [SI.make_dy(shape, j, int(c[-1]), seed) for j, c in enumerate(self.cus)]

    def oracle_params(self):
        return [{k: v.f64 for k, v in layer.items()} for layer in self.layers]


def run_oracle(w: Workload):
    """-> dict(y=[...], dx=[...], grads=[per-mb list of per-layer dicts], reduced=[per-layer dicts])"""
    cfg = oracle_config(w.shape)
    params = w.oracle_params()
    ys, dxs, per_mb = [], [], []
    for j in range(w.M):
        y, caches = O.stage_F(w.x[j].f64, params, w.cus[j], cfg)
        dx, gains, wst = O.stage_B(w.dy[j].f64, caches, params, cfg)
        per_mb.append(O.merge_B_W(gains, O.stage_W(caches, wst, cfg)))
        ys.append(y)
        dxs.append(dx)
    return {"y": ys, "dx": dxs, "grads": per_mb, "reduced": O.grad_reduce(per_mb)}


def canonical_order(M: int):
    return [("F", j) for j in range(M)] + [("B", j) for j in range(M)] + [("W", j) for j in range(M)]


def run_gpu(w: Workload, order=None, n_streams: int = 1, max_tokens=None, keep_raw: bool = False):
    """Runs the workload through the HIP library in the given task order (default canonical),
    round-robin over n_streams streams.  Returns the same dict as run_oracle (fp64 numpy), plus
    raw bit-level copies when keep_raw is set."""
    import torch
    import paper_2605_18750_amd as R
    from paper_2605_18750_amd import harness as Hn

    shape = w.shape
    T_max = max(int(c[-1]) for c in w.cus) if max_tokens is None else max_tokens
    cfg = Hn.make_config(shape, T_max, max(len(c) - 1 for c in w.cus), n_microbatches=w.M)
    stage = Hn.Stage(cfg, Hn.pack_params(cfg, w.layers))
    tdt = torch.float32 if shape.dtype == "fp32" else torch.bfloat16
    xs = [Hn.to_device(t.storage, shape.dtype) for t in w.x]
    dys = [Hn.to_device(t.storage, shape.dtype) for t in w.dy]
    ys = [torch.empty_like(x) for x in xs]
    dxs = [torch.empty_like(x) for x in xs]
    streams = [torch.cuda.Stream() for _ in range(n_streams)]
    torch.cuda.synchronize()
    order = canonical_order(w.M) if order is None else order
    for i, (kind, j) in enumerate(order):
        s = streams[i % n_streams]
        if kind == "F":
            R.stage_F(stage.handle, j, xs[j], w.cus[j], ys[j], s)
        elif kind == "B":
            R.stage_B(stage.handle, j, dys[j], dxs[j], s)
        else:
            R.stage_W(stage.handle, j, s)
    R.stage_grad_reduce(stage.handle, stage.grad_out, streams[0])
    torch.cuda.synchronize()
    out = {"y": [Hn.to_f64(t) for t in ys], "dx": [Hn.to_f64(t) for t in dxs]}
    slots = [stage.slot(j).cpu().numpy() for j in range(w.M)]
    red = stage.grad_out.cpu().numpy()
    out["grads"] = [Hn.unpack_grads(cfg, s) for s in slots]
    out["reduced"] = Hn.unpack_grads(cfg, red)
    if keep_raw:   # bit patterns, for order-independence checks (tensor regions only, no padding)
        bits = torch.int16 if tdt == torch.bfloat16 else torch.int32
        out["raw"] = {"y": [t.cpu().view(bits).numpy() for t in ys],
                      "dx": [t.cpu().view(bits).numpy() for t in dxs],
                      "grads": [Hn.unpack_grads(cfg, s.view(np.int32)) for s in slots],
                      "reduced": Hn.unpack_grads(cfg, red.view(np.int32))}
    stage.close()
    return out


def assert_bit_identical(a: dict, b: dict):
    """Every output of two runs (raw bit patterns) must agree exactly."""
    ra, rb = a["raw"], b["raw"]
    for key in ("y", "dx"):
        for j, (u, v) in enumerate(zip(ra[key], rb[key])):
            assert np.array_equal(u, v), f"{key}[mb {j}] differs between dispatch orders"
    for j, (gm, hm) in enumerate(zip(ra["grads"], rb["grads"])):
        for l, (gl, hl) in enumerate(zip(gm, hm)):
            for k in gl:
                assert np.array_equal(gl[k], hl[k]), f"grad {k} layer {l} mb {j} differs between dispatch orders"
    for l, (gl, hl) in enumerate(zip(ra["reduced"], rb["reduced"])):
        for k in gl:
            assert np.array_equal(gl[k], hl[k]), f"reduced grad {k} layer {l} differs between dispatch orders"


def fuse_grads(layer: dict) -> dict:
    """Per-layer gradient dict keyed by logical names -> the library's own gradient tensors
    (include/rrfp_stage.h, STAGE_P_*): g1, Wqkv = [Wq|Wk|Wv], Wo, g2, Wup = [Wg|Wu] (or W1), Wd."""
    out = {"g1": layer["g1"], "g2": layer["g2"], "Wo": layer["Wo"], "Wd": layer["Wd"],
           "Wqkv": np.concatenate([layer["Wq"], layer["Wk"], layer["Wv"]], axis=1)}
    out["Wup"] = np.concatenate([layer["Wg"], layer["Wu"]], axis=1) if "Wg" in layer else layer["W1"]
    for k in ("b1", "b2", "bo", "bd", "gq", "gk"):
        if k in layer:
            out[k] = layer[k]
    if "bq" in layer:
        out["bqkv"] = np.concatenate([layer["bq"], layer["bk"], layer["bv"]])
        out["bup"] = np.concatenate([layer["bg"], layer["bu"]]) if "bg" in layer else layer["bf"]
    return out


def compare(got: dict, ref: dict, tol: float, what: str = "", report=None):
    """Asserts the max-norm relative error bound for y, dx, every per-microbatch gradient tensor
    and the reduced gradients.  A gradient tensor is checked both as the library stores it
    (STAGE_P_*: the fused Wqkv = [Wq|Wk|Wv], Wup = [Wg|Wu], bqkv, bup) and block by block (Wq, Wk,
    Wv, Wg, Wu, bq, bk, bv, bg, bu each against its own maximum), so a small-magnitude block cannot
    hide behind a large neighbour.  Returns the worst error seen.  `report`, if given, receives
    (name, error) for every tensor checked."""
    worst = 0.0
    failures = []

    def check(name, g, r):
        nonlocal worst
        e = max_norm_rel_err(g, r)
        worst = max(worst, e)
        if report is not None:
            report.append((name, e))
        if not e <= tol:
            failures.append(f"{what} {name}: rel err {e:.3e} > {tol}")

    for key in ("y", "dx"):
        for j, (g, r) in enumerate(zip(got[key], ref[key])):
            check(f"{key}[mb {j}]", g, r)

    parent = {"Wq": "Wqkv", "Wk": "Wqkv", "Wv": "Wqkv", "Wg": "Wup", "Wu": "Wup",
              "bq": "bqkv", "bk": "bqkv", "bv": "bqkv", "bg": "bup", "bu": "bup"}

    def layers(gl_list, rl_list, tag):
        nonlocal worst
        for l, (gl, rl) in enumerate(zip(gl_list, rl_list)):
            gf, rf = fuse_grads(gl), fuse_grads(rl)
            for k in rl:                              # every logical tensor on its own
                den = float(np.max(np.abs(rl[k])))
                big = float(np.max(np.abs(rf[parent[k]]))) if k in parent else den
                if den < 1e-9 * big:
                    # A block whose true value is identically zero (the key bias: softmax does not change when
                    # every key score of a row moves by the same amount, so its gradient vanishes) has no scale
                    # of its own; the oracle holds fp64 round-off there.  It is measured on the fused tensor's scale.
                    e = float(np.max(np.abs(np.asarray(gl[k], dtype=np.float64) - rl[k]))) / big
                    worst = max(worst, e)
                    if report is not None:
                        report.append((f"{tag} {k} layer {l} (zero block, fused scale)", e))
                    if not e <= tol:
                        failures.append(f"{what} {tag} {k} layer {l}: abs err / fused max {e:.3e} > {tol}")
                    continue
                check(f"{tag} {k} layer {l}", gl[k], rl[k])
            for k in rf:                              # the fused tensors of the ABI
                if k not in rl:
                    check(f"{tag} {k} layer {l}", gf[k], rf[k])

    for j, (gm, rm) in enumerate(zip(got["grads"], ref["grads"])):
        layers(gm, rm, f"grad mb {j}")
    if ref["reduced"]:
        layers(got["reduced"], ref["reduced"], "reduced grad")
    assert not failures, "; ".join(failures[:8]) + (f" (+{len(failures) - 8} more)" if len(failures) > 8 else "")
    return worst
