"""Pins for the fp64 oracle: every check here is something other than the oracle itself
(finite differences, brute-force loops, closed forms, invariants, an autograd library)."""
import math

import numpy as np
import pytest

from oracle import stage_oracle as O
import stage_inputs as SI


def _rand_params(cfg, rng, std=0.3):
    H, d, F = cfg.hidden, cfg.head_dim, cfg.ffn
    nq, nkv = cfg.n_q_heads, cfg.n_kv_heads
    ps = []
    for _ in range(cfg.n_layers):
        p = {"g1": 1 + 0.2 * rng.standard_normal(H), "g2": 1 + 0.2 * rng.standard_normal(H),
             "Wq": std * rng.standard_normal((H, nq * d)), "Wk": std * rng.standard_normal((H, nkv * d)),
             "Wv": std * rng.standard_normal((H, nkv * d)), "Wo": std * rng.standard_normal((nq * d, H)),
             "Wd": std * rng.standard_normal((F, H))}
        if cfg.mlp_kind == "swiglu":
            p["Wg"] = std * rng.standard_normal((H, F))
            p["Wu"] = std * rng.standard_normal((H, F))
        else:
            p["W1"] = std * rng.standard_normal((H, F))
        if cfg.norm_kind == "layer":
            p["b1"] = 0.3 * rng.standard_normal(H)
            p["b2"] = 0.3 * rng.standard_normal(H)
        if cfg.qk_norm:
            p["gq"] = 1 + 0.3 * rng.standard_normal(d)
            p["gk"] = 1 + 0.3 * rng.standard_normal(d)
        if cfg.bias:
            for nm, n in (("bq", nq * d), ("bk", nkv * d), ("bv", nkv * d), ("bo", H), ("bd", H)):
                p[nm] = 0.3 * rng.standard_normal(n)
            for nm in (("bg", "bu") if cfg.mlp_kind == "swiglu" else ("bf",)):
                p[nm] = 0.3 * rng.standard_normal(F)
        ps.append(p)
    return ps


CASES = [
    dict(mlp_kind="swiglu", causal=True, n_kv_heads=2),
    dict(mlp_kind="swiglu", causal=False, n_kv_heads=4),
    dict(mlp_kind="gelu", causal=False, n_kv_heads=2),
    dict(mlp_kind="gelu", causal=True, n_kv_heads=1),
    dict(mlp_kind="swiglu", causal=True, n_kv_heads=2, rope=True),
    dict(mlp_kind="gelu", causal=False, n_kv_heads=4, rope=True, rope_base=50.0),
    dict(mlp_kind="gelu", causal=False, n_kv_heads=4, norm_kind="layer", bias=True),
    dict(mlp_kind="swiglu", causal=True, n_kv_heads=2, norm_kind="layer", bias=True, rope=True),
    dict(mlp_kind="gelu", causal=True, n_kv_heads=2, bias=True),
    dict(mlp_kind="swiglu", causal=True, n_kv_heads=2, qk_norm=True, rope=True),
    dict(mlp_kind="gelu", causal=False, n_kv_heads=1, qk_norm=True, bias=True),
]


def _cfg(**kw):
    base = dict(n_layers=2, hidden=16, n_q_heads=4, n_kv_heads=2, head_dim=4, ffn=24)
    base.update(kw)
    return O.OracleConfig(**base)


# ------------------------------------------------------------------ finite differences

@pytest.mark.parametrize("case", CASES)
def test_backward_matches_central_finite_differences(case):
    cfg = _cfg(**case)
    rng = np.random.default_rng(7)
    T, cu = 7, [0, 3, 7]
    params = _rand_params(cfg, rng)
    x = rng.standard_normal((T, cfg.hidden))
    dy = rng.standard_normal((T, cfg.hidden))

    def loss(xv, ps):
        y, _ = O.stage_F(xv, ps, cu, cfg)
        return float(np.sum(y * dy))

    y, caches = O.stage_F(x, params, cu, cfg)
    dx, grads = O.stage_backward_unsplit(dy, caches, params, cfg)

    def fd(arr, setter, n_probe=12):
        flat_idx = rng.choice(arr.size, size=min(n_probe, arr.size), replace=False)
        out = []
        for fi in flat_idx:
            idx = np.unravel_index(fi, arr.shape)
            h = 1e-6 * max(1.0, abs(arr[idx]))
            old = arr[idx]
            arr[idx] = old + h
            lp = setter()
            arr[idx] = old - h
            lm = setter()
            arr[idx] = old
            out.append((idx, (lp - lm) / (2 * h)))
        return out

    xs = x.copy()
    for idx, num in fd(xs, lambda: loss(xs, params), n_probe=24):
        assert abs(num - dx[idx]) <= 1e-6 * max(1.0, abs(num)), ("dx", idx, num, dx[idx])
    for l in range(cfg.n_layers):
        for name in params[l]:
            arr = params[l][name]
            for idx, num in fd(arr, lambda: loss(x, params)):
                an = grads[l][name][idx]
                assert abs(num - an) <= 1e-6 * max(1.0, abs(num)), (l, name, idx, num, an)


# ------------------------------------------------------------------ split == unsplit

@pytest.mark.parametrize("case", CASES)
def test_B_plus_W_equals_unsplit(case):
    cfg = _cfg(**case)
    rng = np.random.default_rng(11)
    T, cu = 9, [0, 4, 9]
    params = _rand_params(cfg, rng)
    x = rng.standard_normal((T, cfg.hidden))
    dy = rng.standard_normal((T, cfg.hidden))
    _, caches = O.stage_F(x, params, cu, cfg)
    dx_u, g_u = O.stage_backward_unsplit(dy, caches, params, cfg)
    dx_b, gains, wst = O.stage_B(dy, caches, params, cfg)
    g_s = O.merge_B_W(gains, O.stage_W(caches, wst, cfg))
    np.testing.assert_allclose(dx_b, dx_u, rtol=0, atol=1e-13 * np.abs(dx_u).max())
    for l in range(cfg.n_layers):
        assert set(g_s[l]) == set(g_u[l]) == set(params[l])
        for k in g_u[l]:
            np.testing.assert_allclose(g_s[l][k], g_u[l][k], rtol=0, atol=1e-13 * np.abs(g_u[l][k]).max())


# ------------------------------------------------------------------ microbatch sum == packed batch

@pytest.mark.parametrize("case", CASES[:3])
def test_sum_of_microbatch_grads_equals_packed_batch(case):
    cfg = _cfg(**case)
    rng = np.random.default_rng(13)
    params = _rand_params(cfg, rng)
    lens = [3, 5, 2, 6]
    xs = [rng.standard_normal((n, cfg.hidden)) for n in lens]
    dys = [rng.standard_normal((n, cfg.hidden)) for n in lens]
    per_mb, dxs = [], []
    for x, dy in zip(xs, dys):
        _, caches = O.stage_F(x, params, [0, len(x)], cfg)
        dx, gains, wst = O.stage_B(dy, caches, params, cfg)
        per_mb.append(O.merge_B_W(gains, O.stage_W(caches, wst, cfg)))
        dxs.append(dx)
    red = O.grad_reduce(per_mb)
    cu = np.concatenate([[0], np.cumsum(lens)])
    X, DY = np.concatenate(xs), np.concatenate(dys)
    _, caches = O.stage_F(X, params, cu, cfg)
    dX, g_all = O.stage_backward_unsplit(DY, caches, params, cfg)
    np.testing.assert_allclose(np.concatenate(dxs), dX, rtol=0, atol=1e-12 * np.abs(dX).max())
    for l in range(cfg.n_layers):
        for k in g_all[l]:
            np.testing.assert_allclose(red[l][k], g_all[l][k], rtol=0, atol=1e-12 * np.abs(g_all[l][k]).max())


def test_grad_reduce_is_left_to_right_in_index_order():
    # Values chosen so that fp64 addition is order-sensitive: (1 + 2^-53) + 2^-53 != 1 + (2^-53 + 2^-53)
    e = 2.0 ** -53
    mbs = [[{"w": np.array([1.0])}], [{"w": np.array([e])}], [{"w": np.array([e])}]]
    assert O.grad_reduce(mbs)[0]["w"][0] == (1.0 + e) + e == 1.0
    assert O.grad_reduce(mbs[::-1])[0]["w"][0] == (e + e) + 1.0 != 1.0


# ------------------------------------------------------------------ exact causality / segment isolation

def test_causality_and_segment_isolation_are_exact():
    cfg = _cfg(mlp_kind="swiglu", causal=True)
    rng = np.random.default_rng(17)
    T, cu = 10, [0, 6, 10]
    params = _rand_params(cfg, rng)
    x = rng.standard_normal((T, cfg.hidden))
    dy = rng.standard_normal((T, cfg.hidden))
    y, caches = O.stage_F(x, params, cu, cfg)
    dx, _, _ = O.stage_B(dy, caches, params, cfg)
    t = 3
    x2 = x.copy(); x2[t] += 1.0
    y2, _ = O.stage_F(x2, params, cu, cfg)
    assert np.array_equal(y2[:t], y[:t])            # earlier tokens: bit-identical
    assert not np.array_equal(y2[t], y[t])
    assert np.all(np.any(y2[t:6] != y[t:6], axis=1))  # later tokens of the same segment do change
    assert np.array_equal(y2[6:], y[6:])            # other segment: bit-identical
    dy2 = dy.copy(); dy2[t] += 1.0
    dx2, _, _ = O.stage_B(dy2, caches, params, cfg)
    assert np.array_equal(dx2[t + 1:], dx[t + 1:])   # gradient flows only to tokens <= t
    assert np.all(np.any(dx2[:t + 1] != dx[:t + 1], axis=1))
    # a perturbation in the second segment never reaches the first, in either direction
    x3 = x.copy(); x3[7] += 1.0
    y3, _ = O.stage_F(x3, params, cu, cfg)
    assert np.array_equal(y3[:7], y[:7])
    dy3 = dy.copy(); dy3[8] += 1.0
    dx3, _, _ = O.stage_B(dy3, caches, params, cfg)
    assert np.array_equal(dx3[:6], dx[:6]) and np.array_equal(dx3[9:], dx[9:])


def test_bidirectional_mixes_whole_segment_but_not_across():
    cfg = _cfg(mlp_kind="gelu", causal=False)
    rng = np.random.default_rng(19)
    T, cu = 8, [0, 5, 8]
    params = _rand_params(cfg, rng)
    x = rng.standard_normal((T, cfg.hidden))
    y, _ = O.stage_F(x, params, cu, cfg)
    x2 = x.copy(); x2[3] += 1.0
    y2, _ = O.stage_F(x2, params, cu, cfg)
    assert np.all(np.any(y2[:5] != y[:5], axis=1))
    assert np.array_equal(y2[5:], y[5:])


# ------------------------------------------------------------------ brute force attention

def _attention_loops(q, k, v, cu, nq, nkv, d, causal):
    T = q.shape[0]
    o = np.zeros((T, nq * d))
    G = nq // nkv
    seg_of = np.zeros(T, dtype=int)
    for s in range(len(cu) - 1):
        seg_of[cu[s]:cu[s + 1]] = s
    for a in range(nq):
        b = a // G
        for i in range(T):
            js = [j for j in range(T) if seg_of[j] == seg_of[i] and (j <= i or not causal)]
            sc = [sum(q[i, a * d + c] * k[j, b * d + c] for c in range(d)) / math.sqrt(d) for j in js]
            mx = max(sc)
            w = [math.exp(s_ - mx) for s_ in sc]
            z = sum(w)
            for c in range(d):
                o[i, a * d + c] = sum(w_ * v[j, b * d + c] for w_, j in zip(w, js)) / z
    return o


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("nkv", [1, 2, 4])
def test_attention_forward_against_python_loops(causal, nkv):
    cfg = _cfg(n_kv_heads=nkv, causal=causal)
    rng = np.random.default_rng(23)
    T, cu = 9, [0, 2, 6, 9]
    d, nq = cfg.head_dim, cfg.n_q_heads
    q = rng.standard_normal((T, nq * d)); k = rng.standard_normal((T, nkv * d)); v = rng.standard_normal((T, nkv * d))
    ref = _attention_loops(q, k, v, cu, nq, nkv, d, causal)
    np.testing.assert_allclose(O.attention_fwd(q, k, v, cu, cfg), ref, rtol=1e-12, atol=1e-13)


def test_attention_backward_finite_differences_and_invariants():
    cfg = _cfg(n_kv_heads=2, causal=True)
    rng = np.random.default_rng(29)
    T, cu = 8, [0, 5, 8]
    d, nq, nkv = cfg.head_dim, cfg.n_q_heads, cfg.n_kv_heads
    q = rng.standard_normal((T, nq * d)); k = rng.standard_normal((T, nkv * d)); v = rng.standard_normal((T, nkv * d))
    do = rng.standard_normal((T, nq * d))
    dq, dk, dv = O.attention_bwd(do, q, k, v, cu, cfg)
    for arr, grad in ((q, dq), (k, dk), (v, dv)):
        for _ in range(10):
            idx = (rng.integers(arr.shape[0]), rng.integers(arr.shape[1]))
            old = arr[idx]; h = 1e-6
            arr[idx] = old + h; lp = np.sum(O.attention_fwd(q, k, v, cu, cfg) * do)
            arr[idx] = old - h; lm = np.sum(O.attention_fwd(q, k, v, cu, cfg) * do)
            arr[idx] = old
            assert abs((lp - lm) / (2 * h) - grad[idx]) < 1e-7
    # softmax rows sum to one and masked keys carry exactly zero weight
    P = O._probabilities(q[:5, :d], k[:5, :d], d, True)
    np.testing.assert_allclose(P.sum(1), 1.0, atol=1e-15)
    assert np.all(np.triu(P, 1) == 0.0)


def test_closed_forms():
    rng = np.random.default_rng(31)
    # T = 1: P = 1, o = v (repeated over the query heads of the group)
    cfg = _cfg(n_kv_heads=2)
    d, nq, nkv = cfg.head_dim, cfg.n_q_heads, cfg.n_kv_heads
    q = rng.standard_normal((1, nq * d)); k = rng.standard_normal((1, nkv * d)); v = rng.standard_normal((1, nkv * d))
    o = O.attention_fwd(q, k, v, [0, 1], cfg)
    np.testing.assert_array_equal(o.reshape(nq, d), np.repeat(v.reshape(nkv, d), nq // nkv, axis=0))
    # all keys equal -> uniform probabilities -> o = running mean of v (causal)
    T = 6
    q = rng.standard_normal((T, nq * d)); k = np.tile(rng.standard_normal((1, nkv * d)), (T, 1))
    v = rng.standard_normal((T, nkv * d))
    o = O.attention_fwd(q, k, v, [0, T], cfg)
    run_mean = np.cumsum(v, 0) / np.arange(1, T + 1)[:, None]
    np.testing.assert_allclose(o.reshape(T, nq, d), np.repeat(run_mean.reshape(T, nkv, d), nq // nkv, axis=1), atol=1e-14)
    # Wo = 0 and Wd = 0 -> y = x and dx = dy
    cfg = _cfg()
    params = _rand_params(cfg, rng)
    for p in params:
        p["Wo"][:] = 0; p["Wd"][:] = 0
    x = rng.standard_normal((T, cfg.hidden)); dy = rng.standard_normal((T, cfg.hidden))
    y, caches = O.stage_F(x, params, [0, T], cfg)
    dx, _, _ = O.stage_B(dy, caches, params, cfg)
    np.testing.assert_array_equal(y, x); np.testing.assert_array_equal(dx, dy)
    # unit gain, eps = 0, rows of unit RMS -> RMSNorm is the identity
    xr = rng.standard_normal((5, 16)); xr /= np.sqrt(np.mean(xr * xr, 1, keepdims=True))
    h, xhat, r = O.rmsnorm_fwd(xr, np.ones(16), 0.0)
    np.testing.assert_allclose(h, xr, atol=1e-15); np.testing.assert_allclose(r, 1.0, atol=1e-15)
    # RMSNorm bwd with unit gain is orthogonal to xhat when eps = 0 (scale invariance of the norm)
    dh = rng.standard_normal((5, 16))
    dxn, dg = O.rmsnorm_bwd(dh, xhat, r, np.ones(16))
    np.testing.assert_allclose(np.sum(dxn * xhat, 1), 0.0, atol=1e-13)
    np.testing.assert_allclose(dg, np.sum(dh * xhat, 0))
    # eps sits inside the square root, added to the mean of squares
    h, _, r = O.rmsnorm_fwd(np.full((1, 4), 2.0), np.ones(4), 5.0)
    assert abs(r[0, 0] - 1.0 / 3.0) < 1e-15 and abs(h[0, 0] - 2.0 / 3.0) < 1e-15


def test_key_shift_invariance_and_scale():
    # Adding the same vector c to every key leaves the softmax (hence o) unchanged only up to q.c per
    # row, which is constant along the row: o is exactly shift invariant in exact arithmetic.
    cfg = _cfg(n_kv_heads=4, causal=False)
    rng = np.random.default_rng(37)
    T = 7; d, nq = cfg.head_dim, cfg.n_q_heads
    q = rng.standard_normal((T, nq * d)); k = rng.standard_normal((T, nq * d)); v = rng.standard_normal((T, nq * d))
    o1 = O.attention_fwd(q, k, v, [0, T], cfg)
    o2 = O.attention_fwd(q, k + np.tile(rng.standard_normal(d), nq), v, [0, T], cfg)
    np.testing.assert_allclose(o1, o2, atol=1e-13)
    # scale is 1/sqrt(d): q scaled by sqrt(d) with two keys gives the logistic of the raw score gap
    qq = np.zeros((2, nq * d)); kk = np.zeros((2, nq * d)); vv = np.zeros((2, nq * d))
    qq[:, 0] = math.sqrt(d); kk[0, 0] = 0.3; kk[1, 0] = -0.4; vv[0, 0] = 1.0
    o = O.attention_fwd(qq, kk, vv, [0, 2], cfg)
    assert abs(o[0, 0] - 1.0 / (1.0 + math.exp(-0.7))) < 1e-15


def test_gqa_equals_mha_with_duplicated_kv_heads():
    rng = np.random.default_rng(41)
    gqa = _cfg(n_kv_heads=2, causal=True)
    mha = _cfg(n_kv_heads=4, causal=True)
    T, cu = 6, [0, 6]; d = gqa.head_dim
    q = rng.standard_normal((T, 4 * d)); k = rng.standard_normal((T, 2 * d)); v = rng.standard_normal((T, 2 * d))
    do = rng.standard_normal((T, 4 * d))
    dup = lambda a: np.repeat(a.reshape(T, 2, d), 2, axis=1).reshape(T, 4 * d)
    np.testing.assert_array_equal(O.attention_fwd(q, k, v, cu, gqa), O.attention_fwd(q, dup(k), dup(v), cu, mha))
    dq1, dk1, dv1 = O.attention_bwd(do, q, k, v, cu, gqa)
    dq2, dk2, dv2 = O.attention_bwd(do, q, dup(k), dup(v), cu, mha)
    fold = lambda a: a.reshape(T, 2, 2, d).sum(2).reshape(T, 2 * d)
    np.testing.assert_allclose(dq1, dq2, atol=1e-14)
    np.testing.assert_allclose(dk1, fold(dk2), atol=1e-14)
    np.testing.assert_allclose(dv1, fold(dv2), atol=1e-14)


def test_activation_closed_forms():
    # silu(z) = z * sigmoid(z); gelu(u) = u * Phi(u); values from the definitions at hand-picked points
    cfg = _cfg(n_layers=1, mlp_kind="swiglu")
    assert abs(O._sigmoid(0.0) - 0.5) < 1e-16 and abs(O._sigmoid(math.log(3.0)) - 0.75) < 1e-15
    assert abs(O._Phi(0.0) - 0.5) < 1e-16
    assert abs(O._Phi(1.0) - 0.8413447460685429) < 1e-15      # standard normal CDF at 1
    assert abs(O._phi(0.0) - 0.3989422804014327) < 1e-16      # 1/sqrt(2 pi)


# ------------------------------------------------------------------ library second opinion

@pytest.mark.parametrize("case", CASES)
def test_against_torch_autograd(case):
    torch = pytest.importorskip("torch")
    cfg = _cfg(**case)
    rng = np.random.default_rng(43)
    T, cu = 11, [0, 4, 11]
    params = _rand_params(cfg, rng)
    x = rng.standard_normal((T, cfg.hidden)); dy = rng.standard_normal((T, cfg.hidden))
    y, caches = O.stage_F(x, params, cu, cfg)
    dx, grads = O.stage_backward_unsplit(dy, caches, params, cfg)

    tp = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()} for p in params]
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    seg = torch.zeros(T, dtype=torch.long)
    for s in range(len(cu) - 1):
        seg[cu[s]:cu[s + 1]] = s
    mask = seg[:, None] == seg[None, :]
    if cfg.causal:
        mask = mask & torch.tril(torch.ones(T, T, dtype=torch.bool))
    d, nq, nkv = cfg.head_dim, cfg.n_q_heads, cfg.n_kv_heads

    def norm(z, p, which):
        if cfg.norm_kind == "layer":
            return torch.nn.functional.layer_norm(z, (cfg.hidden,), p["g" + which], p["b" + which], cfg.norm_eps)
        return z * torch.rsqrt(z.pow(2).mean(-1, keepdim=True) + cfg.norm_eps) * p["g" + which]

    def lin(z, p, w, b):
        return torch.nn.functional.linear(z, p[w].T, p[b] if cfg.bias else None)

    h = tx
    for p in tp:
        a = norm(h, p, "1")
        q = lin(a, p, "Wq", "bq").view(T, nq, d)
        k = lin(a, p, "Wk", "bk").view(T, nkv, d)
        if cfg.qk_norm:
            q = q * torch.rsqrt(q.pow(2).mean(-1, keepdim=True) + cfg.norm_eps) * p["gq"]
            k = k * torch.rsqrt(k.pow(2).mean(-1, keepdim=True) + cfg.norm_eps) * p["gk"]
        if cfg.rope:
            # independent formulation: pairs (x_i, x_{i+d/2}) as complex numbers times e^{i pos theta_i}
            pos = torch.tensor(np.concatenate([np.arange(cu[s + 1] - cu[s]) for s in range(len(cu) - 1)]), dtype=torch.float64)
            theta = torch.tensor(cfg.rope_base, dtype=torch.float64) ** (-2.0 * torch.arange(d // 2, dtype=torch.float64) / d)
            rot = torch.polar(torch.ones(T, d // 2, dtype=torch.float64), pos[:, None] * theta[None, :])[:, None, :]

            def rope(z):
                zc = torch.complex(z[..., :d // 2], z[..., d // 2:]) * rot
                return torch.cat([zc.real, zc.imag], dim=-1)
            q, k = rope(q), rope(k)
        q = q.transpose(0, 1)
        k = k.transpose(0, 1).repeat_interleave(nq // nkv, 0)
        v = lin(a, p, "Wv", "bv").view(T, nkv, d).transpose(0, 1).repeat_interleave(nq // nkv, 0)
        o = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask)
        h = h + lin(o.transpose(0, 1).reshape(T, nq * d), p, "Wo", "bo")
        b = norm(h, p, "2")
        if cfg.mlp_kind == "swiglu":
            m = torch.nn.functional.silu(lin(b, p, "Wg", "bg")) * lin(b, p, "Wu", "bu")
        else:
            m = torch.nn.functional.gelu(lin(b, p, "W1", "bf"))
        h = h + lin(m, p, "Wd", "bd")
    (h * torch.tensor(dy)).sum().backward()
    np.testing.assert_allclose(y, h.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-11)
    for l in range(cfg.n_layers):
        for k_ in grads[l]:
            np.testing.assert_allclose(grads[l][k_], tp[l][k_].grad.numpy(), rtol=1e-10, atol=1e-11)


# ------------------------------------------------------------------ LayerNorm / bias variants

def test_layernorm_closed_forms():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((5, 12)) * 3 + 2
    g, b = rng.standard_normal(12), rng.standard_normal(12)
    h, xhat, r = O.layernorm_fwd(x, g, b, 0.0)
    # normalised rows: zero mean, unit (biased) variance; shift and scale of the input do not matter
    np.testing.assert_allclose(xhat.mean(axis=1), 0, atol=1e-14)
    np.testing.assert_allclose((xhat ** 2).mean(axis=1), 1, rtol=1e-13)
    h2, _, _ = O.layernorm_fwd(7.0 * x - 11.0, g, b, 0.0)
    np.testing.assert_allclose(h2, h, rtol=1e-11, atol=1e-12)
    # against the library definition
    np.testing.assert_allclose(h, (x - x.mean(1, keepdims=True)) / x.std(1, keepdims=True) * g + b, rtol=1e-12)
    # eps inside the square root: a constant row maps to the bias
    hc, _, _ = O.layernorm_fwd(np.full((1, 12), 3.0), g, b, 1e-5)
    np.testing.assert_allclose(hc[0], b, atol=1e-12)
    # the input gradient is orthogonal to constants and to xhat (projections removed)
    dh = rng.standard_normal((5, 12))
    dx, dg, db = O.layernorm_bwd(dh, xhat, r, g)
    np.testing.assert_allclose(dx.sum(axis=1), 0, atol=1e-12)
    np.testing.assert_allclose((dx * xhat).sum(axis=1), 0, atol=1e-12)
    np.testing.assert_allclose(db, dh.sum(axis=0), rtol=1e-14)


def test_bias_variant_reduces_to_plain_layer_at_zero_bias():
    rng = np.random.default_rng(9)
    cfg_b, cfg_0 = _cfg(bias=True, mlp_kind="gelu"), _cfg(mlp_kind="gelu")
    params = _rand_params(cfg_b, rng)
    for p in params:
        for k in list(p):
            if k.startswith("b"):
                p[k] = np.zeros_like(p[k])
    x = rng.standard_normal((9, cfg_0.hidden))
    ya, _ = O.stage_F(x, params, [0, 9], cfg_b)
    yb, _ = O.stage_F(x, params, [0, 9], cfg_0)
    np.testing.assert_array_equal(ya, yb)


def test_key_bias_gradient_vanishes_without_rope_or_head_norm():
    # Adding the same vector to every key of a segment moves all scores of a query row by one constant, which
    # the softmax removes: the loss does not depend on the key bias, so its gradient is exactly zero in exact
    # arithmetic (fp64 round-off here), while the other projection biases have ordinary gradients.
    cfg = _cfg(mlp_kind="gelu", causal=True, n_kv_heads=2, bias=True)
    rng = np.random.default_rng(3)
    T, cu = 9, [0, 4, 9]
    params = _rand_params(cfg, rng)
    x, dy = rng.standard_normal((T, cfg.hidden)), rng.standard_normal((T, cfg.hidden))
    _, caches = O.stage_F(x, params, cu, cfg)
    _, grads = O.stage_backward_unsplit(dy, caches, params, cfg)
    for g in grads:
        assert np.max(np.abs(g["bk"])) < 1e-12 * np.max(np.abs(g["bq"]))
        assert np.max(np.abs(g["bv"])) > 1e-3
    # with the rotary embedding the bias is rotated per position and the invariance is gone
    cfg_r = _cfg(mlp_kind="gelu", causal=True, n_kv_heads=2, bias=True, rope=True)
    _, caches = O.stage_F(x, params, cu, cfg_r)
    _, grads = O.stage_backward_unsplit(dy, caches, params, cfg_r)
    assert all(np.max(np.abs(g["bk"])) > 1e-6 for g in grads)


def test_qk_norm_makes_scores_independent_of_the_projection_scale():
    # with head normalisation (eps = 0) scaling Wq or Wk by a positive constant changes nothing
    rng = np.random.default_rng(10)
    cfg = O.OracleConfig(n_layers=1, hidden=16, n_q_heads=4, n_kv_heads=2, head_dim=4, ffn=24, qk_norm=True, norm_eps=0.0)
    params = _rand_params(cfg, rng)
    x = rng.standard_normal((9, 16))
    y0, _ = O.stage_F(x, params, [0, 9], cfg)
    scaled = [dict(p, Wq=3.0 * p["Wq"], Wk=0.25 * p["Wk"]) for p in params]
    y1, _ = O.stage_F(x, scaled, [0, 9], cfg)
    np.testing.assert_allclose(y1, y0, rtol=1e-10, atol=1e-12)
    # unit gains: every normalised head has RMS 1 (checked through the cache)
    unit = [dict(p, gq=np.ones(4), gk=np.ones(4)) for p in params]
    _, caches = O.stage_F(x, unit, [0, 9], cfg)
    q = caches[0]["q_att"].reshape(9, 4, 4)
    np.testing.assert_allclose(np.sqrt((q ** 2).mean(-1)), 1.0, rtol=1e-12)


# ------------------------------------------------------------------ rotary embedding variant

def test_rope_rotation_properties():
    rng = np.random.default_rng(5)
    # one pair, angle pi/2 at position 1 with base 1 -> theta = 1; use pos = pi/2 directly
    out = O.rope_rotate(np.array([[1.0, 0.0]]), np.array([np.pi / 2]), 1, 2, base=7.0)
    np.testing.assert_allclose(out, [[0.0, 1.0]], atol=1e-15)
    # frequencies base^(-2i/d): pair i of a d = 8 head at position 1 turns by base^(-i/4)
    x = np.zeros((1, 8)); x[0, :4] = 1.0
    out = O.rope_rotate(x, np.array([1.0]), 1, 8, base=16.0)
    np.testing.assert_allclose(out[0, :4], np.cos(16.0 ** (-np.arange(4) / 4.0)), atol=1e-15)
    np.testing.assert_allclose(out[0, 4:], np.sin(16.0 ** (-np.arange(4) / 4.0)), atol=1e-15)
    # a rotation: norms per head are kept, the inverse undoes it, position 0 is the identity
    x = rng.standard_normal((9, 3 * 8)); pos = np.arange(9.0) * 3
    y = O.rope_rotate(x, pos, 3, 8, 100.0)
    np.testing.assert_allclose(np.linalg.norm(y.reshape(9, 3, 8), axis=2), np.linalg.norm(x.reshape(9, 3, 8), axis=2), rtol=1e-13)
    np.testing.assert_allclose(O.rope_rotate(y, pos, 3, 8, 100.0, sign=-1.0), x, atol=1e-13)
    np.testing.assert_array_equal(O.rope_rotate(x, np.zeros(9), 3, 8, 100.0), x)
    np.testing.assert_array_equal(O.rope_positions([0, 3, 4, 9]), [0, 1, 2, 0, 0, 1, 2, 3, 4])


def test_rope_scores_depend_on_relative_positions_only():
    # shifting every position by a constant changes neither the outputs nor any gradient
    cfg0 = _cfg(rope=True, causal=True)
    cfg1 = _cfg(rope=True, causal=True, rope_offset=37)
    rng = np.random.default_rng(6)
    T, cu = 10, [0, 6, 10]
    params = _rand_params(cfg0, rng)
    x = rng.standard_normal((T, cfg0.hidden)); dy = rng.standard_normal((T, cfg0.hidden))
    outs = []
    for cfg in (cfg0, cfg1):
        y, caches = O.stage_F(x, params, cu, cfg)
        dx, grads = O.stage_backward_unsplit(dy, caches, params, cfg)
        outs.append((y, dx, grads))
    np.testing.assert_allclose(outs[0][0], outs[1][0], rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(outs[0][1], outs[1][1], rtol=1e-9, atol=1e-10)
    for l in range(cfg0.n_layers):
        for k in outs[0][2][l]:
            np.testing.assert_allclose(outs[0][2][l][k], outs[1][2][l][k], rtol=1e-9, atol=1e-10)
    # and the variant is not a no-op: with several tokens per segment the output differs from no-rope
    y_plain, _ = O.stage_F(x, params, cu, _cfg(causal=True))
    assert np.abs(y_plain - outs[0][0]).max() > 1e-3
    # single-token segments sit at position 0: rope on == rope off, exactly
    cu1 = list(range(T + 1))
    ya, _ = O.stage_F(x, params, cu1, cfg0)
    yb, _ = O.stage_F(x, params, cu1, _cfg(causal=True))
    np.testing.assert_array_equal(ya, yb)


# ------------------------------------------------------------------ input generator sanity

def test_generator_is_counter_based_and_normal():
    a = SI.normal_f64(1, "t", (1000,))
    b = SI.normal_f64(1, "t", (1000,), chunk=77)
    np.testing.assert_array_equal(a, b)
    big = SI.normal_f64(2, "u", (200000,))
    assert abs(big.mean()) < 0.01 and abs(big.std() - 1.0) < 0.01
    t = SI.make_tensor(3, "w", (64, 64), 0.02, "bf16")
    assert np.array_equal(SI.bf16_bits_to_f64(t.storage), t.f64)
    assert np.all((t.f64.astype(np.float32).view(np.uint32) & 0xFFFF) == 0)
    order = SI.ready_order(8, 5)
    pos = {kj: i for i, kj in enumerate(order)}
    assert len(order) == 24 and all(pos[("F", j)] < pos[("B", j)] < pos[("W", j)] for j in range(8))
