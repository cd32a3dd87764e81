"""Plumbing around the C ABI for tests, smoke() and bench.py: stage_config from a StageShape,
packing logical parameter tensors into the parameter buffer per stage_param_layout, splitting
a flat fp32 gradient buffer back into logical tensors, and device buffers via torch.  No layer
arithmetic lives here."""
from __future__ import annotations

import numpy as np

import paper_2605_18750_amd as R


def make_config(shape, max_tokens: int, max_segments: int = 1, n_microbatches: int | None = None):
    return R.stage_config(
        n_layers=shape.n_layers, hidden=shape.hidden, n_q_heads=shape.n_q_heads,
        n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn,
        max_tokens=max_tokens,
        n_microbatches=shape.n_microbatches if n_microbatches is None else n_microbatches,
        max_segments=max_segments,
        dtype=R.STAGE_DTYPE_FP32 if shape.dtype == "fp32" else R.STAGE_DTYPE_BF16,
        mlp_kind=R.STAGE_MLP_SWIGLU if shape.mlp_kind == "swiglu" else R.STAGE_MLP_GELU,
        causal=1 if shape.causal else 0, norm_kind=1 if getattr(shape, "norm_kind", "rms") == "layer" else 0,
        norm_eps=shape.norm_eps, rope=1 if getattr(shape, "rope", False) else 0,
        rope_base=getattr(shape, "rope_base", 10000.0), bias=1 if getattr(shape, "bias", False) else 0,
        qk_norm=1 if getattr(shape, "qk_norm", False) else 0)


def _fused(layer: dict, which: int, swiglu: bool) -> np.ndarray:
    """Storage array of fused tensor `which` from the logical tensors of one layer."""
    st = lambda n: layer[n].storage
    if which == R.STAGE_P_G1:
        return st("g1")
    if which == R.STAGE_P_WQKV:
        return np.concatenate([st("Wq"), st("Wk"), st("Wv")], axis=1)
    if which == R.STAGE_P_WO:
        return st("Wo")
    if which == R.STAGE_P_G2:
        return st("g2")
    if which == R.STAGE_P_WUP:
        return np.concatenate([st("Wg"), st("Wu")], axis=1) if swiglu else st("W1")
    if which == R.STAGE_P_WD:
        return st("Wd")
    empty = np.zeros(0, dtype=st("g1").dtype)
    if which in (R.STAGE_P_B1, R.STAGE_P_B2):
        nm = "b1" if which == R.STAGE_P_B1 else "b2"
        return st(nm) if nm in layer else empty
    if which in (R.STAGE_P_GQ, R.STAGE_P_GK):
        nm = "gq" if which == R.STAGE_P_GQ else "gk"
        return st(nm) if nm in layer else empty
    if "bo" not in layer:
        return empty
    if which == R.STAGE_P_BQKV:
        return np.concatenate([st("bq"), st("bk"), st("bv")])
    if which == R.STAGE_P_BO:
        return st("bo")
    if which == R.STAGE_P_BUP:
        return np.concatenate([st("bg"), st("bu")]) if swiglu else st("bf")
    if which == R.STAGE_P_BD:
        return st("bd")
    raise ValueError(which)


def pack_params(cfg, layers: list) -> np.ndarray:
    """Flat parameter buffer (float32, or uint16 bf16 bit patterns) in the library's layout."""
    param_bytes, _, _ = R.stage_query(cfg)
    esz = 4 if cfg.dtype == R.STAGE_DTYPE_FP32 else 2
    flat = np.zeros(param_bytes // esz, dtype=np.float32 if esz == 4 else np.uint16)
    swiglu = cfg.mlp_kind == R.STAGE_MLP_SWIGLU
    for l, layer in enumerate(layers):
        for which in range(R.STAGE_P_COUNT):
            off, (r, c) = R.stage_param_layout(cfg, l, which)
            a = np.ascontiguousarray(_fused(layer, which, swiglu)).reshape(-1)
            assert a.size == r * c, (which, a.size, r, c)
            flat[off:off + a.size] = a
    return flat


def unpack_grads(cfg, flat: np.ndarray) -> list:
    """Flat fp32 gradient buffer -> per-layer dicts keyed by the logical tensor names."""
    d, nq, nkv = cfg.head_dim, cfg.n_q_heads, cfg.n_kv_heads
    F = cfg.ffn
    swiglu = cfg.mlp_kind == R.STAGE_MLP_SWIGLU
    out = []
    for l in range(cfg.n_layers):
        t = {}
        for which in range(R.STAGE_P_COUNT):
            off, (r, c) = R.stage_param_layout(cfg, l, which)
            t[which] = flat[off:off + r * c].reshape(r, c)
        g = {"g1": t[R.STAGE_P_G1].reshape(-1), "g2": t[R.STAGE_P_G2].reshape(-1),
             "Wq": t[R.STAGE_P_WQKV][:, :nq * d], "Wk": t[R.STAGE_P_WQKV][:, nq * d:(nq + nkv) * d],
             "Wv": t[R.STAGE_P_WQKV][:, (nq + nkv) * d:], "Wo": t[R.STAGE_P_WO], "Wd": t[R.STAGE_P_WD]}
        if swiglu:
            g["Wg"] = t[R.STAGE_P_WUP][:, :F]
            g["Wu"] = t[R.STAGE_P_WUP][:, F:]
        else:
            g["W1"] = t[R.STAGE_P_WUP]
        if cfg.norm_kind == 1:
            g["b1"], g["b2"] = t[R.STAGE_P_B1].reshape(-1), t[R.STAGE_P_B2].reshape(-1)
        if cfg.qk_norm:
            g["gq"], g["gk"] = t[R.STAGE_P_GQ].reshape(-1), t[R.STAGE_P_GK].reshape(-1)
        if cfg.bias:
            bqkv, bup = t[R.STAGE_P_BQKV].reshape(-1), t[R.STAGE_P_BUP].reshape(-1)
            g["bq"], g["bk"], g["bv"] = bqkv[:nq * d], bqkv[nq * d:(nq + nkv) * d], bqkv[(nq + nkv) * d:]
            g["bo"], g["bd"] = t[R.STAGE_P_BO].reshape(-1), t[R.STAGE_P_BD].reshape(-1)
            if swiglu:
                g["bg"], g["bu"] = bup[:F], bup[F:]
            else:
                g["bf"] = bup
        out.append(g)
    return out


def to_device(storage: np.ndarray, dtype: str, device="cuda:0"):
    """numpy storage (float32, or uint16 bf16 bits) -> torch device tensor of that dtype."""
    import torch
    if dtype == "fp32":
        return torch.from_numpy(np.ascontiguousarray(storage, dtype=np.float32)).to(device)
    t = torch.from_numpy(np.ascontiguousarray(storage).view(np.int16)).to(device)
    return t.view(torch.bfloat16)


def to_f64(t) -> np.ndarray:
    """torch device tensor (fp32 or bf16) -> numpy fp64 on the host."""
    import torch
    return t.detach().to("cpu", torch.float64).numpy()


class Stage:
    """Owns the device buffers of one stage (parameters, arena, grad_out) and the handle."""

    def __init__(self, cfg, params_flat: np.ndarray, device="cuda:0"):
        import torch
        self.cfg = cfg
        self.device = device
        self.param_bytes, self.grad_bytes, self.arena_bytes = R.stage_query(cfg)
        self.dtype = "fp32" if cfg.dtype == R.STAGE_DTYPE_FP32 else "bf16"
        self.params = to_device(params_flat, self.dtype, device)
        self.arena = torch.empty(self.arena_bytes, dtype=torch.uint8, device=device)
        self.grad_out = torch.empty(self.grad_bytes // 4, dtype=torch.float32, device=device)
        self.handle = R.stage_create(cfg, self.params, self.arena, self.arena_bytes)

    def slot(self, mb: int):
        """Gradient slot mb as a torch fp32 tensor aliasing the arena."""
        import torch
        addr = R.stage_grad_slot(self.handle, mb)
        off = addr - self.arena.data_ptr()
        return self.arena[off:off + self.grad_bytes].view(torch.float32)

    def intermediate(self, mb: int, layer: int, which: int, T: int):
        """Intermediate tensor `which` (R.STAGE_T_*) of a layer as a torch tensor aliasing the arena."""
        import torch
        c = self.cfg
        nqkv = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim
        nup = (2 if c.mlp_kind == R.STAGE_MLP_SWIGLU else 1) * c.ffn
        cols = {R.STAGE_T_X: c.hidden, R.STAGE_T_H1: c.hidden, R.STAGE_T_QKV: nqkv, R.STAGE_T_O: c.n_q_heads * c.head_dim,
                R.STAGE_T_X1: c.hidden, R.STAGE_T_H2: c.hidden, R.STAGE_T_UP: nup, R.STAGE_T_M: c.ffn,
                R.STAGE_T_DY: c.hidden, R.STAGE_T_DUP: nup, R.STAGE_T_DX1: c.hidden, R.STAGE_T_DQKV: nqkv,
                R.STAGE_T_H1_HALF: c.hidden}
        off = R.stage_intermediate(self.handle, mb, layer, which) - self.arena.data_ptr()
        if which == R.STAGE_T_LSE:
            return self.arena[off:off + 4 * c.n_q_heads * T].view(torch.float32).view(c.n_q_heads, T)
        f32 = which in (R.STAGE_T_X, R.STAGE_T_X1) or self.dtype == "fp32"
        half = not f32 and which in (R.STAGE_T_QKV, R.STAGE_T_H1_HALF)     # IEEE-half copies of the bf16 path
        esz = 4 if f32 else 2
        n = T * cols[which]
        tdt = torch.float32 if f32 else (torch.float16 if half else torch.bfloat16)
        return self.arena[off:off + esz * n].view(tdt).view(T, cols[which])

    def close(self):
        if self.handle is not None:
            R.stage_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
