"""fp64 CPU oracle for the per-microbatch stage tasks F, B and W.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file; it is
used by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg.  It
shares no code with the HIP path.

What it computes.  The paper (Section 3.1, Section 4.1, Section 7.1 "Baselines")
fixes only the task model: F_j is the forward of the stage's layers for microbatch j,
the backward of j needs the local F_j and the upstream gradient, and under the BFW
variant the backward is decomposed into a part that produces the input gradient (B)
and a part that produces the weight gradients (W).  The paper changes only the order
in which tasks run ("preserving training semantics", Section 7.1), so the result of
every task is the ordinary forward value / gradient of ordinary pre-norm transformer
layers.  The oracle is therefore the plain definition of those layers and of their
gradient, written with numpy in fp64 with no blocking, fusion or reordering:

  forward of one layer (x [T,H], packed segments given by cu_seqlens):
    h1 = RMSNorm(x; g1)                        r = (mean_c x^2 + eps)^-1/2, h = x*r*g
    q,k,v = h1 Wq, h1 Wk, h1 Wv
    o = per segment, per query head a (KV head a // G): softmax(q k^T / sqrt(d)) v,
        the softmax running over the keys of the same segment (and j <= i if causal)
    x1 = x + o Wo
    h2 = RMSNorm(x1; g2)
    m  = silu(h2 Wg) * (h2 Wu)        (SwiGLU)   or   gelu_erf(h2 W1)   (GELU)
    y  = x1 + m Wd

  The backward is the chain rule applied to exactly these lines.  "unsplit" returns
  every gradient; B returns dx, the two norm-gain gradients and the GEMM
  output-gradients W needs; W returns the GEMM-shaped weight gradients.

Readings where the paper is silent (all layer math is): W computes gradients, not an
optimizer update; norm-gain gradients are produced in B; no biases, no positional
encoding; eps inside the square root; masked keys are excluded from the softmax;
query head a uses KV head a // (n_q / n_kv); GELU is the exact erf form.

Model-fidelity variants (off in the five workloads; the paper names GPT3-Large and ViT models,
which use them, without printing layer details): rope = rotary embedding on q and k;
qk_norm = RMSNorm over head_dim of every query and key head (gains gq, gk of length head_dim shared
by all heads, same eps), applied to the projection output before the rotary embedding;
norm_kind = "layer" replaces both RMSNorms by LayerNorm with gain and bias,
h = (x - mean) * (var + eps)^-1/2 * g + b; bias = True adds a bias vector to each of the four
projections.  All vector-shaped gradients (gains and biases) are produced in B.

Every function is pinned by tests/test_oracle_pins.py (finite differences, brute-force
loops, closed forms, exact causality, split == unsplit, microbatch-sum == packed batch,
an independent autograd cross-check).  Nothing here is "parity unpinned".
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
from scipy.special import erf as _erf


@dataclass(frozen=True)
class OracleConfig:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    mlp_kind: str = "swiglu"      # "swiglu" | "gelu"
    causal: bool = True
    norm_eps: float = 1e-5
    norm_kind: str = "rms"        # "rms" | "layer" (LayerNorm with gain and bias; model-fidelity variant)
    bias: bool = False            # bias vectors on the four projections (model-fidelity variant)
    qk_norm: bool = False         # RMSNorm over head_dim on every q and k head, before rope (model-fidelity variant)
    rope: bool = False            # rotary position embedding on q and k (model-fidelity variant)
    rope_base: float = 10000.0
    rope_offset: int = 0          # added to every position (test hook for the relative-position property)


# ----------------------------------------------------------------------------- pieces

def layernorm_fwd(x, g, b, eps):
    """h = xhat * g + b with xhat = (x - mean_c x) * r, r = (var_c x + eps)^(-1/2) (biased variance)."""
    mu = np.mean(x, axis=1, keepdims=True)
    xc = x - mu
    r = 1.0 / np.sqrt(np.mean(xc * xc, axis=1, keepdims=True) + eps)
    xhat = xc * r
    return xhat * g + b, xhat, r


def layernorm_bwd(dh, xhat, r, g):
    """Gradient of h = xhat * g + b.  Returns dx, dg, db."""
    w = dh * g
    dx = r * (w - np.mean(w, axis=1, keepdims=True) - xhat * np.mean(w * xhat, axis=1, keepdims=True))
    return dx, np.sum(dh * xhat, axis=0), np.sum(dh, axis=0)


def _norm_fwd(x, p, which, cfg):
    if cfg.norm_kind == "layer":
        return layernorm_fwd(x, p["g" + which], p["b" + which], cfg.norm_eps)
    return rmsnorm_fwd(x, p["g" + which], cfg.norm_eps)


def _norm_bwd(dh, xhat, r, p, which, cfg, out):
    """Norm backward; stores the vector-shaped parameter gradients in `out`, returns dx."""
    if cfg.norm_kind == "layer":
        dx, out["g" + which], out["b" + which] = layernorm_bwd(dh, xhat, r, p["g" + which])
    else:
        dx, out["g" + which] = rmsnorm_bwd(dh, xhat, r, p["g" + which])
    return dx


def _b(p, name, cfg):
    """Bias vector `name` when the variant is on, else 0."""
    return p[name] if cfg.bias else 0.0


def rope_positions(cu_seqlens, offset=0):
    """Position of every token inside its own segment, plus offset."""
    cu = np.asarray(cu_seqlens)
    pos = np.empty(int(cu[-1]), dtype=np.float64)
    for s in range(len(cu) - 1):
        pos[cu[s]:cu[s + 1]] = np.arange(cu[s + 1] - cu[s]) + offset
    return pos


def rope_rotate(x, pos, n_heads, d, base, sign=1.0):
    """Rotary embedding in the split-half convention (Su et al. 2021, as used by LLaMA / Qwen
    implementations): for every head and i < d/2 the pair (x_i, x_{i+d/2}) is rotated by the angle
    pos * base^(-2i/d).  sign = -1 applies the inverse (= transpose) rotation, which is what maps a
    gradient w.r.t. the rotated vector back to the un-rotated one."""
    T = x.shape[0]
    half = d // 2
    theta = base ** (-2.0 * np.arange(half) / d)
    ang = pos[:, None] * theta[None, :]
    cs, sn = np.cos(ang)[:, None, :], sign * np.sin(ang)[:, None, :]
    xh = x.reshape(T, n_heads, d)
    a, b = xh[:, :, :half], xh[:, :, half:]
    out = np.concatenate([a * cs - b * sn, b * cs + a * sn], axis=2)
    return out.reshape(T, n_heads * d)


def _head_norm_fwd(x, g, n_heads, d, eps):
    """RMSNorm of every head's d-vector with the gain g [d]: the rows are the (token, head) pairs."""
    T = x.shape[0]
    h, xhat, r = rmsnorm_fwd(x.reshape(T * n_heads, d), g, eps)
    return h.reshape(T, n_heads * d), xhat, r


def _qk_for_attention(c, cfg, p=None):
    """q, k as the attention sees them: head-normalised and rotated when those variants are on
    (computed once per layer and cached)."""
    if not (cfg.rope or cfg.qk_norm):
        return c["q"], c["k"]
    if "q_att" not in c:
        q, k = c["q"], c["k"]
        if cfg.qk_norm:
            q, c["q_hat"], c["q_r"] = _head_norm_fwd(q, p["gq"], cfg.n_q_heads, cfg.head_dim, cfg.norm_eps)
            k, c["k_hat"], c["k_r"] = _head_norm_fwd(k, p["gk"], cfg.n_kv_heads, cfg.head_dim, cfg.norm_eps)
        if cfg.rope:
            pos = rope_positions(c["cu"], cfg.rope_offset)
            q = rope_rotate(q, pos, cfg.n_q_heads, cfg.head_dim, cfg.rope_base)
            k = rope_rotate(k, pos, cfg.n_kv_heads, cfg.head_dim, cfg.rope_base)
        c["q_att"], c["k_att"] = q, k
    return c["q_att"], c["k_att"]


def _attention_bwd_qk(do, c, cfg, p=None, out=None):
    """Gradients w.r.t. the projection outputs q, k, v (rotation and head norm undone for q and k);
    the head-norm gain gradients go into `out`."""
    q, k = _qk_for_attention(c, cfg, p)
    dq, dk, dv = attention_bwd(do, q, k, c["v"], c["cu"], cfg)
    if cfg.rope:
        pos = rope_positions(c["cu"], cfg.rope_offset)
        dq = rope_rotate(dq, pos, cfg.n_q_heads, cfg.head_dim, cfg.rope_base, sign=-1.0)
        dk = rope_rotate(dk, pos, cfg.n_kv_heads, cfg.head_dim, cfg.rope_base, sign=-1.0)
    if cfg.qk_norm:
        T, d = dq.shape[0], cfg.head_dim
        dqh, out["gq"] = rmsnorm_bwd(dq.reshape(T * cfg.n_q_heads, d), c["q_hat"], c["q_r"], p["gq"])
        dkh, out["gk"] = rmsnorm_bwd(dk.reshape(T * cfg.n_kv_heads, d), c["k_hat"], c["k_r"], p["gk"])
        dq, dk = dqh.reshape(T, cfg.n_q_heads * d), dkh.reshape(T, cfg.n_kv_heads * d)
    return dq, dk, dv

def rmsnorm_fwd(x, g, eps):
    """h = x * r * g with r = (mean_c x^2 + eps)^(-1/2).  Returns h, xhat = x*r, r."""
    r = 1.0 / np.sqrt(np.mean(x * x, axis=1, keepdims=True) + eps)
    xhat = x * r
    return xhat * g, xhat, r


def rmsnorm_bwd(dh, xhat, r, g):
    """Gradient of h = xhat * g, xhat = x * r(x).  Returns dx, dg."""
    w = dh * g
    dx = r * (w - xhat * np.mean(w * xhat, axis=1, keepdims=True))
    dg = np.sum(dh * xhat, axis=0)
    return dx, dg


def _segments(cu_seqlens):
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    return [(int(cu[i]), int(cu[i + 1])) for i in range(len(cu) - 1)]


def _probabilities(qa, kb, d, causal):
    """Softmax over allowed keys of S = qa kb^T / sqrt(d) for one head of one segment."""
    S = (qa @ kb.T) / np.sqrt(float(d))
    if causal:
        n = S.shape[0]
        allowed = np.tril(np.ones((n, n), dtype=bool))
        S = np.where(allowed, S, -np.inf)
    S = S - np.max(S, axis=1, keepdims=True)
    E = np.exp(S)                      # exp(-inf) = 0: masked keys get weight exactly 0
    return E / np.sum(E, axis=1, keepdims=True)


def attention_fwd(q, k, v, cu_seqlens, cfg):
    """q [T, nq*d], k and v [T, nkv*d] (head-major within a row) -> o [T, nq*d]."""
    nq, nkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    G = nq // nkv
    o = np.zeros_like(q)
    for (s, e) in _segments(cu_seqlens):
        for a in range(nq):
            b = a // G
            P = _probabilities(q[s:e, a * d:(a + 1) * d], k[s:e, b * d:(b + 1) * d], d, cfg.causal)
            o[s:e, a * d:(a + 1) * d] = P @ v[s:e, b * d:(b + 1) * d]
    return o


def attention_bwd(do, q, k, v, cu_seqlens, cfg):
    """Gradient of attention_fwd.  Returns dq, dk, dv."""
    nq, nkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    G = nq // nkv
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    scale = 1.0 / np.sqrt(float(d))
    for (s, e) in _segments(cu_seqlens):
        for a in range(nq):
            b = a // G
            qa = q[s:e, a * d:(a + 1) * d]
            kb = k[s:e, b * d:(b + 1) * d]
            vb = v[s:e, b * d:(b + 1) * d]
            doa = do[s:e, a * d:(a + 1) * d]
            P = _probabilities(qa, kb, d, cfg.causal)
            dP = doa @ vb.T
            dS = P * (dP - np.sum(P * dP, axis=1, keepdims=True))     # softmax Jacobian
            dq[s:e, a * d:(a + 1) * d] = (dS @ kb) * scale
            dk[s:e, b * d:(b + 1) * d] += (dS.T @ qa) * scale
            dv[s:e, b * d:(b + 1) * d] += P.T @ doa
    return dq, dk, dv


def _sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def _Phi(u):
    return 0.5 * (1.0 + _erf(u / np.sqrt(2.0)))


def _phi(u):
    return np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi)


# ----------------------------------------------------------------------------- one layer

def layer_forward(x, p, cu_seqlens, cfg):
    """Forward of one pre-norm layer.  p: dict of logical fp64 weights (y = x @ W).
    Returns y and a cache of every intermediate the backward uses."""
    c = {"x": x, "cu": np.asarray(cu_seqlens)}
    c["h1"], c["xhat"], c["r1"] = _norm_fwd(x, p, "1", cfg)
    c["q"] = c["h1"] @ p["Wq"] + _b(p, "bq", cfg)
    c["k"] = c["h1"] @ p["Wk"] + _b(p, "bk", cfg)
    c["v"] = c["h1"] @ p["Wv"] + _b(p, "bv", cfg)
    q, k = _qk_for_attention(c, cfg, p)
    c["o"] = attention_fwd(q, k, c["v"], cu_seqlens, cfg)
    c["x1"] = x + c["o"] @ p["Wo"] + _b(p, "bo", cfg)
    c["h2"], c["x1hat"], c["r2"] = _norm_fwd(c["x1"], p, "2", cfg)
    if cfg.mlp_kind == "swiglu":
        c["gt"] = c["h2"] @ p["Wg"] + _b(p, "bg", cfg)
        c["up"] = c["h2"] @ p["Wu"] + _b(p, "bu", cfg)
        c["m"] = c["gt"] * _sigmoid(c["gt"]) * c["up"]
    elif cfg.mlp_kind == "gelu":
        c["u"] = c["h2"] @ p["W1"] + _b(p, "bf", cfg)
        c["m"] = c["u"] * _Phi(c["u"])
    else:
        raise ValueError(cfg.mlp_kind)
    y = c["x1"] + c["m"] @ p["Wd"] + _b(p, "bd", cfg)
    return y, c


def layer_backward_unsplit(dy, c, p, cfg):
    """All gradients of one layer in one pass: returns dx and a dict of parameter grads."""
    g = {}
    dm = dy @ p["Wd"].T
    g["Wd"] = c["m"].T @ dy
    dx1 = dy.copy()
    if cfg.mlp_kind == "swiglu":
        sg = _sigmoid(c["gt"])
        dgt = dm * c["up"] * sg * (1.0 + c["gt"] * (1.0 - sg))
        dup = dm * c["gt"] * sg
        dh2 = dgt @ p["Wg"].T + dup @ p["Wu"].T
        g["Wg"] = c["h2"].T @ dgt
        g["Wu"] = c["h2"].T @ dup
        if cfg.bias:
            g["bg"], g["bu"] = dgt.sum(axis=0), dup.sum(axis=0)
    else:
        du = dm * (_Phi(c["u"]) + c["u"] * _phi(c["u"]))
        dh2 = du @ p["W1"].T
        g["W1"] = c["h2"].T @ du
        if cfg.bias:
            g["bf"] = du.sum(axis=0)
    dn = _norm_bwd(dh2, c["x1hat"], c["r2"], p, "2", cfg, g)
    dx1 = dx1 + dn
    do = dx1 @ p["Wo"].T
    g["Wo"] = c["o"].T @ dx1
    dq, dk, dv = _attention_bwd_qk(do, c, cfg, p, g)
    dh1 = dq @ p["Wq"].T + dk @ p["Wk"].T + dv @ p["Wv"].T
    g["Wq"] = c["h1"].T @ dq
    g["Wk"] = c["h1"].T @ dk
    g["Wv"] = c["h1"].T @ dv
    if cfg.bias:
        g["bd"], g["bo"] = dy.sum(axis=0), dx1.sum(axis=0)
        g["bq"], g["bk"], g["bv"] = dq.sum(axis=0), dk.sum(axis=0), dv.sum(axis=0)
    dn = _norm_bwd(dh1, c["xhat"], c["r1"], p, "1", cfg, g)
    dx = dx1 + dn
    return dx, g


def layer_B(dy, c, p, cfg):
    """Backward-to-inputs of one layer.  Returns dx, the norm-gain grads, and the GEMM
    output-gradients that the W task of the same microbatch consumes."""
    w = {"dy": dy}
    dm = dy @ p["Wd"].T
    if cfg.mlp_kind == "swiglu":
        sg = _sigmoid(c["gt"])
        w["dgt"] = dm * c["up"] * sg * (1.0 + c["gt"] * (1.0 - sg))
        w["dup"] = dm * c["gt"] * sg
        dh2 = w["dgt"] @ p["Wg"].T + w["dup"] @ p["Wu"].T
    else:
        w["du"] = dm * (_Phi(c["u"]) + c["u"] * _phi(c["u"]))
        dh2 = w["du"] @ p["W1"].T
    gains = {}
    dn = _norm_bwd(dh2, c["x1hat"], c["r2"], p, "2", cfg, gains)
    w["dx1"] = dy + dn
    do = w["dx1"] @ p["Wo"].T
    w["dq"], w["dk"], w["dv"] = _attention_bwd_qk(do, c, cfg, p, gains)
    dh1 = w["dq"] @ p["Wq"].T + w["dk"] @ p["Wk"].T + w["dv"] @ p["Wv"].T
    dn = _norm_bwd(dh1, c["xhat"], c["r1"], p, "1", cfg, gains)
    if cfg.bias:     # column sums of the GEMM output-gradients: vector-shaped, produced in B like the gains
        gains["bd"], gains["bo"] = dy.sum(axis=0), w["dx1"].sum(axis=0)
        gains["bq"], gains["bk"], gains["bv"] = w["dq"].sum(axis=0), w["dk"].sum(axis=0), w["dv"].sum(axis=0)
        if cfg.mlp_kind == "swiglu":
            gains["bg"], gains["bu"] = w["dgt"].sum(axis=0), w["dup"].sum(axis=0)
        else:
            gains["bf"] = w["du"].sum(axis=0)
    return w["dx1"] + dn, gains, w


def layer_W(c, w, cfg):
    """Backward-to-weights of one layer: every GEMM-shaped gradient, dW = input^T @ dOut."""
    g = {"Wd": c["m"].T @ w["dy"], "Wo": c["o"].T @ w["dx1"],
         "Wq": c["h1"].T @ w["dq"], "Wk": c["h1"].T @ w["dk"], "Wv": c["h1"].T @ w["dv"]}
    if cfg.mlp_kind == "swiglu":
        g["Wg"] = c["h2"].T @ w["dgt"]
        g["Wu"] = c["h2"].T @ w["dup"]
    else:
        g["W1"] = c["h2"].T @ w["du"]
    return g


# ----------------------------------------------------------------------------- the stage tasks

def stage_F(x, params, cu_seqlens, cfg):
    """F task: forward through the stage's layers.  Returns y and the per-layer caches."""
    caches = []
    for p in params:
        x, c = layer_forward(x, p, cu_seqlens, cfg)
        caches.append(c)
    return x, caches


def stage_backward_unsplit(dy, caches, params, cfg):
    """Unsplit backward: dx and per-layer dicts of all parameter gradients."""
    grads = [None] * len(params)
    for l in reversed(range(len(params))):
        dy, grads[l] = layer_backward_unsplit(dy, caches[l], params[l], cfg)
    return dy, grads


def stage_B(dy, caches, params, cfg):
    """B task: dx, per-layer norm-gain grads, per-layer output-gradient stash for W."""
    gains = [None] * len(params)
    wst = [None] * len(params)
    for l in reversed(range(len(params))):
        dy, gains[l], wst[l] = layer_B(dy, caches[l], params[l], cfg)
    return dy, gains, wst


def stage_W(caches, wst, cfg):
    """W task: per-layer dicts of GEMM-shaped weight gradients."""
    return [layer_W(c, w, cfg) for c, w in zip(caches, wst)]


def grad_reduce(per_microbatch):
    """Index-ordered sum ((s_0 + s_1) + s_2) + ... of per-microbatch gradient lists."""
    total = [{k: v.copy() for k, v in layer.items()} for layer in per_microbatch[0]]
    for mb in per_microbatch[1:]:
        for tl, layer in zip(total, mb):
            for k in tl:
                tl[k] = tl[k] + layer[k]
    return total


def merge_B_W(gains, wgrads):
    """Join B's gain grads and W's GEMM grads into the per-layer dicts unsplit returns."""
    return [{**g, **w} for g, w in zip(gains, wgrads)]
