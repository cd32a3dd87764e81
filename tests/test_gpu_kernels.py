"""Kernel-level GPU parity (through the C ABI of rrfp_kernels.h) against fp64 definitions."""
import sys

import numpy as np
import pytest

import stage_inputs as SI

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _gemm_case(M, N, K, ta, tb, out_fp32, with_r, family, in_dtype="bf16", seed=5):
    import torch
    import paper_2605_18750_amd as R
    from paper_2605_18750_amd import harness as Hn
    from tests.helpers import max_norm_rel_err
    name = f"gemm M{M} N{N} K{K} ta{ta} tb{tb} f32out{out_fp32} r{with_r} fam{family} {in_dtype}"
    _say(f"[kernel] {name}")
    A = SI.make_tensor(seed, name + "A", (K, M) if ta else (M, K), 1.0, in_dtype)
    B = SI.make_tensor(seed, name + "B", (N, K) if tb else (K, N), 1.0, in_dtype)
    Rr = SI.make_tensor(seed, name + "R", (M, N), 4.0, "fp32") if with_r else None     # the residual is always fp32
    ref = (A.f64.T if ta else A.f64) @ (B.f64.T if tb else B.f64)     # the definition, fp64
    if with_r:
        ref = ref + Rr.f64
    dA, dB = Hn.to_device(A.storage, in_dtype), Hn.to_device(B.storage, in_dtype)
    dR = Hn.to_device(Rr.storage, "fp32") if with_r else None
    odt = torch.float32 if (out_fp32 or in_dtype == "fp32") else torch.bfloat16
    dC = torch.full((M, N), float("nan"), dtype=odt, device="cuda:0")
    idt = R.STAGE_DTYPE_FP32 if in_dtype == "fp32" else R.STAGE_DTYPE_BF16
    R.rrfp_gemm(dA, dB, dC, dR, M, N, K, dA.shape[1], dB.shape[1], N, N, ta, tb, idt,
                R.STAGE_DTYPE_FP32 if odt == torch.float32 else R.STAGE_DTYPE_BF16, family)
    torch.cuda.synchronize()
    got = dC.cpu().to(torch.float64).numpy()
    assert np.all(np.isfinite(got)), name + ": unwritten or non-finite outputs"
    tol = 1e-4 if odt == torch.float32 and in_dtype == "fp32" else (2e-5 if odt == torch.float32 else 1e-2)
    # fp32 accumulation of exact bf16 products: error ~ sqrt(K) * 2^-24 relative to the max; bf16 output adds 2^-9
    err = max_norm_rel_err(got, ref)
    _say(f"[kernel] {name}: rel err {err:.3e} (tol {tol})")
    assert err <= tol, name


ORIENT = [(0, 0), (0, 1), (1, 0), (1, 1)]


@pytest.mark.parametrize("ta,tb", ORIENT)
def test_mfma_gemm_small_ragged(ta, tb):
    # several tiles in M and N with ragged tails, K with a ragged last step
    _gemm_case(264, 520, 200, ta, tb, out_fp32=False, with_r=False, family=2)
    _gemm_case(520, 264, 328, ta, tb, out_fp32=True, with_r=False, family=2)
    _gemm_case(40, 72, 64, ta, tb, out_fp32=False, with_r=True, family=2)


@pytest.mark.parametrize("K", [32, 96, 160, 416, 448, 480, 736, 768, 1056])
def test_mfma_gemm_k_steps_across_pipeline_boundaries(K):
    """K / 32 = 1, 3, 5, 13, 14, 15, 23, 24, 33 steps: shorter than the load pipeline, exactly at the point
    where the unguarded ten-step loop is first entered (14) and re-entered (24), odd and even counts
    (loads are issued for pairs of steps), for every operand orientation the direct-load kernel takes."""
    for ta, tb in ((0, 0), (0, 1), (1, 0)):
        _gemm_case(136, 264, K, ta, tb, out_fp32=(ta == 1), with_r=False, family=2, seed=K)
    # weight-gradient form with a ragged last step
    _gemm_case(264, 136, K + 8, 1, 0, out_fp32=True, with_r=False, family=2, seed=K + 1)


def test_mfma_gemm_ragged_token_counts():
    # forward / input-gradient forms with T not a multiple of anything; weight-gradient form with K = T odd
    _gemm_case(777, 512, 256, 0, 0, False, True, 2)
    _gemm_case(777, 256, 512, 0, 1, False, False, 2)
    _gemm_case(256, 512, 777, 1, 0, True, False, 2)
    _gemm_case(1, 8, 8, 0, 0, False, False, 2)


@pytest.mark.parametrize("ta,tb", ORIENT)
def test_simt_gemm(ta, tb):
    _gemm_case(70, 45, 33, ta, tb, out_fp32=True, with_r=True, family=1, in_dtype="fp32")
    _gemm_case(130, 65, 100, ta, tb, out_fp32=False, with_r=False, family=1)


def test_mfma_rejects_unsupported_shapes():
    import torch
    import paper_2605_18750_amd as R
    a = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(R.StageError):
        R.rrfp_gemm(a, a, a, None, 64, 60, 64, 64, 64, 64, 64, 0, 0, 1, 1, R.RRFP_GEMM_MFMA)   # N % 8
    with pytest.raises(R.StageError):
        R.rrfp_gemm(a, a, a, None, 64, 64, 60, 64, 64, 64, 64, 0, 0, 1, 1, R.RRFP_GEMM_MFMA)   # K % 8, A K-contiguous
    with pytest.raises(R.StageError):
        R.rrfp_gemm(a, a, a, None, 64, 64, 64, 32, 64, 64, 64, 0, 0, 1, 1, R.RRFP_GEMM_MFMA)   # lda < K


def test_mfma_gemm_full_size_sampled_rows():
    """Language-stage QKV projection at full size (4096 x 12288 x 4096): rows sampled across
    tiles are compared with the fp64 definition row by row."""
    import torch
    import paper_2605_18750_amd as R
    from paper_2605_18750_amd import harness as Hn
    from tests.helpers import max_norm_rel_err
    M, N, K = 4096, 12288, 4096
    _say("[kernel] full-size NN gemm, sampled rows")
    A = SI.make_tensor(1, "fullA", (M, K), 1.0, "bf16")
    B = SI.make_tensor(1, "fullB", (K, N), 0.02, "bf16")
    dA, dB = Hn.to_device(A.storage, "bf16"), Hn.to_device(B.storage, "bf16")
    dC = torch.empty((M, N), dtype=torch.bfloat16, device="cuda:0")
    R.rrfp_gemm(dA, dB, dC, None, M, N, K, K, N, N, N, 0, 0, 1, 1, R.RRFP_GEMM_MFMA)
    torch.cuda.synchronize()
    rows = [0, 1, 31, 32, 255, 256, 1000, 2047, 2048, 3333, 4095]
    got = dC[rows].cpu().to(torch.float64).numpy()
    ref = A.f64[rows] @ B.f64
    err = max_norm_rel_err(got, ref)
    _say(f"[kernel] full-size NN gemm: rel err {err:.3e}")
    assert err <= 1e-2


def test_mfma_gemm_short_tile_tail():
    """Shapes whose tile count leaves a small last round on 256 CUs (1000 x 17920: 4 x 70 = 280 tiles,
    24 left over = 6 tile columns) take 128-row tiles for those columns: every element is compared, so
    both launches, the seam between them and the ragged last row block are covered."""
    import torch
    import paper_2605_18750_amd as R
    from paper_2605_18750_amd import harness as Hn
    from tests.helpers import max_norm_rel_err
    M, N, K = 1000, 17920, 256
    _say("[kernel] NN gemm with short-tile tail")
    A = SI.make_tensor(2, "tailA", (M, K), 1.0, "bf16")
    B = SI.make_tensor(2, "tailB", (K, N), 0.05, "bf16")
    dA, dB = Hn.to_device(A.storage, "bf16"), Hn.to_device(B.storage, "bf16")
    dC = torch.full((M + 8, N), 7.0, dtype=torch.bfloat16, device="cuda:0")       # guard rows behind the output
    R.rrfp_gemm(dA, dB, dC, None, M, N, K, K, N, N, N, 0, 0, 1, 1, R.RRFP_GEMM_MFMA)
    torch.cuda.synchronize()
    got = dC[:M].cpu().to(torch.float64).numpy()
    ref = A.f64 @ B.f64
    for lo, hi in ((0, 16384), (16384, N)):        # main launch, tail launch
        err = max_norm_rel_err(got[:, lo:hi], ref[:, lo:hi])
        _say(f"[kernel] columns {lo}:{hi}: rel err {err:.3e}")
        assert err <= 1e-2
    assert torch.all(dC[M:] == 7.0), "rows past M were written"


@pytest.mark.parametrize("T,H,dtype", [(777, 512, "bf16"), (130, 256, "fp32"), (1030, 4096, "bf16"), (9, 1280, "bf16"),
                                       (65, 200, "fp32"), (300, 8192, "bf16"), (70, 2048, "fp32"), (33, 3000, "bf16"),
                                       (20, 4096, "fp32"), (12, 8192, "fp32"), (7, 1001, "fp32"), (5, 16384, "bf16")])
def test_rmsnorm_kernels_against_oracle(T, H, dtype):
    """RMSNorm forward and backward (rows + gain gradient) through their own entry points, against the fp64
    oracle on the same rounded inputs; T spans several row chunks with a ragged tail."""
    import torch
    import paper_2605_18750_amd as R
    from paper_2605_18750_amd import harness as Hn
    from oracle import stage_oracle as O
    from tests.helpers import max_norm_rel_err
    name = f"rmsnorm T{T} H{H} {dtype}"
    _say(f"[kernel] {name}")
    eps = 1e-5
    x = SI.make_tensor(3, name + "x", (T, H), 1.0, "fp32")
    g = SI.make_tensor(3, name + "g", (H,), 0.02, dtype, mean=1.0)
    dh = SI.make_tensor(3, name + "dh", (T, H), 1.0, "fp32")
    add = SI.make_tensor(3, name + "add", (T, H), 1.0, "fp32")
    h_ref, xhat, r_ref = O.rmsnorm_fwd(x.f64, g.f64, eps)
    dx_ref, dg_ref = O.rmsnorm_bwd(dh.f64, xhat, r_ref, g.f64)
    dx_ref = dx_ref + add.f64
    dt = R.STAGE_DTYPE_FP32 if dtype == "fp32" else R.STAGE_DTYPE_BF16
    tdt = torch.float32 if dtype == "fp32" else torch.bfloat16
    dx_, ddh, dadd = (Hn.to_device(t.storage, "fp32") for t in (x, dh, add))
    dgain = Hn.to_device(g.storage, dtype)
    h = torch.full((T, H), float("nan"), dtype=tdt, device="cuda:0")
    r = torch.full((T,), float("nan"), dtype=torch.float32, device="cuda:0")
    R.rrfp_rmsnorm_fwd(dx_, dgain, h, r, T, H, eps, dt)
    ws_bytes = R.rrfp_rmsnorm_bwd_workspace(T, H, dt)
    assert ws_bytes > 0
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0")
    out32 = torch.full((T, H), float("nan"), dtype=torch.float32, device="cuda:0")
    out_t = torch.full((T, H), float("nan"), dtype=tdt, device="cuda:0")
    dg = torch.full((H,), float("nan"), dtype=torch.float32, device="cuda:0")
    R.rrfp_rmsnorm_bwd(ddh, dx_, r, dgain, dadd, out32, out_t, dg, ws, ws_bytes, T, H, dt)
    torch.cuda.synchronize()
    tol_f32, tol_t = 2e-5, (2e-5 if dtype == "fp32" else 8e-3)     # fp32 arithmetic; bf16 storage rounds once (2^-9)
    errs = {"h": (max_norm_rel_err(Hn.to_f64(h), h_ref), tol_t),
            "r": (max_norm_rel_err(Hn.to_f64(r), r_ref.reshape(-1)), tol_f32),
            "dx fp32": (max_norm_rel_err(Hn.to_f64(out32), dx_ref), tol_f32),
            "dx storage": (max_norm_rel_err(Hn.to_f64(out_t), dx_ref), tol_t),
            "dg": (max_norm_rel_err(Hn.to_f64(dg), dg_ref), tol_f32)}
    for k, (e, tol) in errs.items():
        _say(f"[kernel] {name} {k}: {e:.3e} (tol {tol})")
        assert e <= tol, (name, k)
    with pytest.raises(R.StageError):
        R.rrfp_rmsnorm_bwd(ddh, dx_, r, dgain, dadd, out32, out_t, dg, ws, ws_bytes - 4, T, H, dt)


def test_grad_reduce_kernel_is_the_index_ordered_sum():
    """rrfp_grad_reduce against the oracle's grad_reduce (fp64: 1e-6 tolerance) and, bit for bit, against the
    fp32 sum in index order formed with torch on the device, including values that make the order matter."""
    import torch
    import paper_2605_18750_amd as R
    from oracle import stage_oracle as O
    M, n, stride = 5, 4 * 100003, 4 * 100010
    g = torch.Generator(device="cuda:0")
    g.manual_seed(3)
    slots = torch.empty(M * stride, dtype=torch.float32, device="cuda:0").normal_(0, 1, generator=g)
    slots[0:stride:7] *= 1e8                     # large first terms: ((a + b) + c) != (a + (b + c)) in fp32
    out = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda:0")
    R.rrfp_grad_reduce(slots, stride, M, out, n)
    torch.cuda.synchronize()
    acc = slots[0:n].clone()
    for j in range(1, M):
        acc += slots[j * stride: j * stride + n]
    assert torch.equal(acc.view(torch.int32), out.view(torch.int32))
    per_mb = [[{"w": slots[j * stride: j * stride + n].cpu().double().numpy()}] for j in range(M)]
    ref = O.grad_reduce(per_mb)[0]["w"]
    err = float(np.max(np.abs(out.cpu().double().numpy() - ref)) / np.max(np.abs(ref)))
    _say(f"[kernel] grad_reduce vs oracle: {err:.3e}")
    assert err <= 1e-6


@pytest.mark.parametrize("M,N,K", [(4096, 22016, 1024), (4096, 5640, 1056), (1280, 1280, 2080)])
def test_weight_gradient_gemm_with_workspace_split_forms(M, N, K):
    """The weight-gradient form with a workspace, every element against the fp64 definition: a grid whose last
    round is nearly empty (16 x 86 tiles, the up-projection shape: plain launch + tail launch split along K),
    the same with a ragged last tile column and a ragged K, and a small grid split along K as a whole."""
    import torch
    import paper_2605_18750_amd as R
    from paper_2605_18750_amd import harness as Hn
    from tests.helpers import max_norm_rel_err
    plan = R.rrfp_gemm_plan(M, N, K, 1, 0, R.STAGE_DTYPE_FP32, have_scratch=True)
    _say(f"[kernel] wgrad with workspace M{M} N{N} K{K}: plan {plan}")
    assert plan["split_k"] > 1
    A = SI.make_tensor(4, f"wsA{M}", (K, M), 1.0, "bf16")
    B = SI.make_tensor(4, f"wsB{N}", (K, N), 1.0, "bf16")
    dA, dB = Hn.to_device(A.storage, "bf16"), Hn.to_device(B.storage, "bf16")
    ws_bytes = 16 * M * N * 4 if plan["short_workgroups"] == 0 else 2 * M * 2048 * 4
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0")
    dC = torch.full((M + 8, N), float("nan"), dtype=torch.float32, device="cuda:0")
    dC[M:] = 7.0
    R.rrfp_gemm(dA, dB, dC, None, M, N, K, M, N, N, N, 1, 0, 1, 0, R.RRFP_GEMM_MFMA, workspace=ws, workspace_bytes=ws_bytes)
    torch.cuda.synchronize()
    got = dC[:M].cpu().to(torch.float64).numpy()
    assert np.all(np.isfinite(got))
    ref = A.f64.T @ B.f64
    err = max_norm_rel_err(got, ref)
    _say(f"[kernel] wgrad with workspace: rel err {err:.3e}")
    assert err <= 2e-5
    assert torch.all(dC[M:] == 7.0), "rows past M were written"
    # same call again: bit-identical (fixed summation order)
    dC2 = torch.empty((M, N), dtype=torch.float32, device="cuda:0")
    R.rrfp_gemm(dA, dB, dC2, None, M, N, K, M, N, N, N, 1, 0, 1, 0, R.RRFP_GEMM_MFMA, workspace=ws, workspace_bytes=ws_bytes)
    torch.cuda.synchronize()
    assert torch.equal(dC2.view(torch.int32), dC[:M].view(torch.int32))
