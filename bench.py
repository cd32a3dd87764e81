#!/usr/bin/env python3
"""bench.py -- throughput of the F/B/W stage tasks on one MI355X.

A "step" is one pass of the whole hot path over one batch: F, B and W of every microbatch of
the stage plus stage_grad_reduce, inputs resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload language|wide|vision|multimodal|tiny]

value     = algorithmic TFLOP of the step / wall time (GEMM 2*T*P per layer per task kind,
            attention forward 4*d*n_q*pairs with pairs = s^2/2 causal or s^2 bidirectional,
            attention backward counted as twice the forward, no recompute, no elementwise flops).
roofline  = the kernel with the largest share of the step time in the form the step launches it (the
            bf16 MFMA GEMM in its weight-gradient form on the up projection, fp32 output: one call of the
            W task), timed alone with HIP events on its stream, against the dense bf16 MFMA peak of
            2.5 PFLOP/s.
hbm_kernels = the HBM-bound kernels of the step timed alone through their own entry points (RMSNorm
            forward and backward at [T, hidden], the gradient reduction), algorithmic bytes per call
            against 8 TB/s, beside the rate of a plain device copy on the same box.
cpu_baseline = the fp64 oracle, as it stands, timed on this machine's host cores on a bounded
            sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA: 256 CUs x 4096 flop/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0


def task_flops(shape, cu):
    """Algorithmic flops of F, B, W for one microbatch with segment boundaries cu."""
    H, d, F = shape.hidden, shape.head_dim, shape.ffn
    nq, nkv = shape.n_q_heads, shape.n_kv_heads
    c = 3 if shape.mlp_kind == "swiglu" else 2
    P = H * nq * d + 2 * H * nkv * d + nq * d * H + c * H * F
    T = int(cu[-1])
    pairs = sum(((int(b) - int(a)) ** 2) / (2.0 if shape.causal else 1.0) for a, b in zip(cu[:-1], cu[1:]))
    A = 4.0 * d * nq * pairs
    L = shape.n_layers
    return {"F": L * (2.0 * T * P + A), "B": L * (2.0 * T * P + 2 * A), "W": L * 2.0 * T * P}


def cpu_baseline(shape, T_sample: int):
    """The oracle on one layer, one microbatch of T_sample tokens of the same shape."""
    import numpy as np
    import stage_inputs as SI
    from oracle import stage_oracle as O
    one = shape.replace(n_layers=1, name=shape.name + "/cpu_sample")
    cfg = O.OracleConfig(n_layers=1, hidden=one.hidden, n_q_heads=one.n_q_heads, n_kv_heads=one.n_kv_heads,
                         head_dim=one.head_dim, ffn=one.ffn, mlp_kind=one.mlp_kind, causal=one.causal,
                         norm_eps=one.norm_eps)
    if shape.name.startswith("vision"):
        cu = np.arange(0, T_sample + 1, SI.VISION_TOKENS_PER_IMAGE)
    else:
        cu = np.array([0, T_sample])
    T_sample = int(cu[-1])
    params = [{k: v.f64 for k, v in SI.make_layer_params(one, 0).items()}]
    x = SI.make_x(one, 0, T_sample).f64
    dy = SI.make_dy(one, 0, T_sample).f64
    t0 = time.perf_counter()
    _, caches = O.stage_F(x, params, cu, cfg)
    _, gains, wst = O.stage_B(dy, caches, params, cfg)
    O.stage_W(caches, wst, cfg)
    dt = time.perf_counter() - t0
    fl = task_flops(one, cu)
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    env = os.environ.get("OMP_NUM_THREADS")
    threads = min(cores, int(env)) if env and env.isdigit() else cores
    return {"value": (fl["F"] + fl["B"] + fl["W"]) / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"fp64 numpy oracle, F+B+W of 1 layer of the {shape.name} shape, 1 microbatch, T={T_sample}, "
                      f"{dt:.1f} s wall"}


def gemm_roofline(shape, T, Bw, s, gen, n_launch=40, form="nn"):
    """The bf16 MFMA GEMM of the up projection alone, HIP events on the launch stream.  form "nn": the
    forward [T, hidden] x [hidden, N_up] (the roofline kernel of the step bench); "nt": its input
    gradient [T, N_up] x [hidden, N_up]^T -> fp32 [T, hidden]; "tn": its weight gradient
    [T, hidden]^T x [T, N_up] -> fp32 [hidden, N_up] (for counter runs of the other operand orientations)."""
    import torch
    import paper_2605_18750_amd as R
    N_up = (2 if shape.mlp_kind == "swiglu" else 1) * shape.ffn
    H = shape.hidden
    A = torch.empty((T, H), dtype=torch.bfloat16, device=Bw.device).normal_(0.0, 1.0, generator=gen)
    if form == "nn":
        Cc = torch.empty((T, N_up), dtype=torch.bfloat16, device=Bw.device)
        dims = (T, N_up, H)

        def launch():
            R.rrfp_gemm(A, Bw, Cc, None, T, N_up, H, H, N_up, N_up, N_up, 0, 0, 1, 1, R.RRFP_GEMM_MFMA, s)
    else:
        G = torch.empty((T, N_up), dtype=torch.bfloat16, device=Bw.device).normal_(0.0, 1.0, generator=gen)
        if form == "nt":
            Cc = torch.empty((T, H), dtype=torch.float32, device=Bw.device)
            dims = (T, H, N_up)

            def launch():
                R.rrfp_gemm(G, Bw, Cc, None, T, H, N_up, N_up, N_up, H, H, 0, 1, 1, 0, R.RRFP_GEMM_MFMA, s)
        else:
            Cc = torch.empty((H, N_up), dtype=torch.float32, device=Bw.device)
            dims = (H, N_up, T)
            ws_bytes = T * shape.ffn * 4            # the scratch the W task hands to this call (B's idle fp32 temporary)
            ws = torch.empty(ws_bytes, dtype=torch.uint8, device=Bw.device)

            def launch():
                R.rrfp_gemm(A, G, Cc, None, H, N_up, T, H, N_up, N_up, N_up, 1, 0, 1, 0, R.RRFP_GEMM_MFMA, s,
                            workspace=ws, workspace_bytes=ws_bytes)
    with torch.cuda.stream(s):
        # the tensors above were just made: the chip has been idle, and its clock takes some tens of launches to
        # settle under the GEMM again (the step timed before ran with a settled clock)
        for _ in range(max(3, n_launch)):
            launch()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record(s)
        for _ in range(n_launch):
            launch()
        g1.record(s)
    torch.cuda.synchronize()
    g_ms = g0.elapsed_time(g1) / n_launch
    g_fl = 2.0 * dims[0] * dims[1] * dims[2]
    ach = g_fl / (g_ms * 1e-3) / 1e12
    # HBM traffic per call: a recorded rocprofv3 counter value (profiles/gemm_mfma_traffic.json names the
    # counter summary it comes from), not a measurement of this run.
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "gemm_mfma_traffic.json")
    if os.path.exists(tpath):
        try:
            rec = json.load(open(tpath))
            traffic = rec.get(f"{form}:{dims[0]}x{dims[1]}x{dims[2]}")
            traffic_source = rec.get("source") if traffic is not None else None
        except Exception:
            traffic = None
    label = {"nn": "(one call: 256-row tiles + 128-row tail launch)", "nt": "(fp32 out)",
             "tn": "(weight-gradient form of the W task, fp32 out; one call: plain launch + split-K tail launch + its reduce)"}[form]
    return {"bound": "mfma", "kernel": f"gemm_mfma_dl_kernel {form.upper()} {dims[0]}x{dims[1]}x{dims[2]} bf16 {label}", "achieved": round(ach, 1),
            "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / PEAK_BF16_TFLOPS, 4),
            "flops_per_launch": g_fl, "avg_launch_ms": round(g_ms, 4), "traffic": traffic,
            "traffic_source": traffic_source}


def gemm_sweep(s, n_launch=200):
    """One bf16 GEMM [M, K] x [K, 4096] per row, M = 4096 / 2048 / 1024 (256, 128, 64 tiles of 256 x 256) and
    K = 2048 / 4096 / 8192, in the weight-gradient (tn, fp32 out), input-gradient (nt, fp32 and bf16 out) and forward
    (nn, bf16 out) forms; HIP events over n_launch launches after n_launch warm-up launches.  The slope against K is
    the main-loop time of one tile, the intercept what a launch costs besides (launch, pipeline fill, the output
    burst).  With fewer tiles than CUs the forms with a K-contiguous A cut M into 128-row tiles."""
    import torch
    import paper_2605_18750_amd as R
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    BF, F32 = R.STAGE_DTYPE_BF16, R.STAGE_DTYPE_FP32
    N = 4096
    rows = []
    for form, out in (("tn", F32), ("nt", F32), ("nt", BF), ("nn", BF)):
        ta, tb = {"tn": (1, 0), "nt": (0, 1), "nn": (0, 0)}[form]
        for M in (4096, 2048, 1024):
            us = []
            for K in (2048, 4096, 8192):
                A = torch.empty((K, M) if ta else (M, K), dtype=torch.bfloat16, device=dev).normal_(0.0, 1.0, generator=gen)
                B = torch.empty((N, K) if tb else (K, N), dtype=torch.bfloat16, device=dev).normal_(0.0, 1.0 if form == "tn" else 0.02,
                                                                                                       generator=gen)
                C = torch.empty((M, N), dtype=torch.float32 if out == F32 else torch.bfloat16, device=dev)
                call = lambda: R.rrfp_gemm(A, B, C, None, M, N, K, A.shape[1], B.shape[1], N, 0, ta, tb, BF, out, stream=s)
                with torch.cuda.stream(s):
                    for _ in range(n_launch):
                        call()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(s)
                    for _ in range(n_launch):
                        call()
                    e1.record(s)
                torch.cuda.synchronize()
                us.append(e0.elapsed_time(e1) / n_launch * 1e3)
            slope = (us[2] - us[0]) / 6.0
            rows.append({"form": form, "out": "fp32" if out == F32 else "bf16", "M": M, "tiles_256": (M // 256) * (N // 256),
                         "us_at_K_2048_4096_8192": [round(u, 1) for u in us], "us_per_1024_K": round(slope, 2),
                         "intercept_us": round(us[0] - 2 * slope, 1)})
    return rows


def hbm_kernels(shape, T, M, grad_floats, s, gen, n_launch=20):
    """The HBM-bound kernels alone, HIP events on the launch stream.  Algorithmic bytes (storage type bf16):
    RMSNorm forward 2 * T * H * 2 B, RMSNorm backward 4 * T * H * 2 B (three reads, one write), gradient
    reduction (M + 1) * P * 4 B.  `moved` is what the kernel really reads and writes (the residual stream and
    the GEMM output it consumes are fp32 in this build)."""
    import torch
    import paper_2605_18750_amd as R
    H = shape.hidden
    dev = "cuda:0"
    dt = R.STAGE_DTYPE_BF16
    x = torch.empty((T, H), dtype=torch.float32, device=dev).normal_(0.0, 1.0, generator=gen)
    dh = torch.empty((T, H), dtype=torch.float32, device=dev).normal_(0.0, 1.0, generator=gen)
    add = torch.empty((T, H), dtype=torch.float32, device=dev).normal_(0.0, 1.0, generator=gen)
    g = torch.ones(H, dtype=torch.bfloat16, device=dev)
    h = torch.empty((T, H), dtype=torch.bfloat16, device=dev)
    r = torch.empty(T, dtype=torch.float32, device=dev)
    out32 = torch.empty((T, H), dtype=torch.float32, device=dev)
    out_t = torch.empty((T, H), dtype=torch.bfloat16, device=dev)
    dg = torch.empty(H, dtype=torch.float32, device=dev)
    nb = R.rrfp_rmsnorm_bwd_workspace(T, H, dt)
    ws = torch.empty(nb, dtype=torch.uint8, device=dev)
    n_red = min(grad_floats, 1 << 28) // 4 * 4
    slots = torch.empty(M * n_red, dtype=torch.float32, device=dev).normal_(0.0, 1.0, generator=gen)
    red = torch.empty(n_red, dtype=torch.float32, device=dev)
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    cases = [
        ("rmsnorm_fwd", lambda: R.rrfp_rmsnorm_fwd(x, g, h, r, T, H, 1e-5, dt, s), 2 * T * H * 2, T * H * (4 + 2)),
        ("rmsnorm_bwd (+ gain gradient)", lambda: R.rrfp_rmsnorm_bwd(dh, x, r, g, add, out32, out_t, dg, ws, nb, T, H, dt, s),
         4 * T * H * 2, T * H * (4 * 3 + 4 + 2)),
        ("grad_reduce", lambda: R.rrfp_grad_reduce(slots, n_red, M, red, n_red, s), (M + 1) * n_red * 4, (M + 1) * n_red * 4),
        ("device copy (torch, 1 GiB)", lambda: dst.copy_(src, non_blocking=True), 2 << 30, 2 << 30),
    ]
    out = []
    with torch.cuda.stream(s):
        for name, fn, alg, moved in cases:
            for _ in range(3):
                fn()
            # Six 1 GiB copies ahead of the timed launches keep the GPU busy for 2.6 ms while the host enqueues them:
            # a launch through the Python binding costs the host more than these kernels run, and an empty queue
            # would time the host.
            for _ in range(6):
                dst.copy_(src, non_blocking=True)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(s)
            for _ in range(n_launch):
                fn()
            e1.record(s)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / n_launch
            gbs = alg / (ms * 1e-3) / 1e9
            out.append({"kernel": name, "shape": f"T={T}, hidden={H}" if "rmsnorm" in name else
                        (f"{M} slots x {n_red} fp32" if name == "grad_reduce" else "1 GiB"),
                        "avg_launch_us": round(ms * 1e3, 2), "algorithmic_bytes": alg, "GB/s": round(gbs, 1),
                        "frac_of_hbm_peak": round(gbs / PEAK_HBM_GBS, 4), "moved_bytes": moved,
                        "moved_GB/s": round(moved / (ms * 1e-3) / 1e9, 1)})
    return out


def pipeline_study(shape, cus, per_mb, n_stages, with_oracle):
    """Replays measured per-microbatch task times (seconds) through the native simulator: N identical
    stages, fixed 1F1B against readiness-driven dispatch (BF hint with unsplit backward, BFW hint with
    the B/W split), under the jitter levels of the robustness table, 10 seeds each."""
    import numpy as np
    from paper_2605_18750_amd import arbiter as A
    M = len(cus)
    N = n_stages
    f = np.tile(np.array(per_mb["F"])[None, None, :], (N, 1, 1))
    b = np.tile(np.array(per_mb["B"])[None, None, :], (N, 1, 1))
    w = np.tile(np.array(per_mb["W"])[None, None, :], (N, 1, 1))
    levels = {"J0": (0.0, 0.0, 0.0), "J1": (0.1, 5e-3, 0.5), "J2": (0.2, 10e-3, 1.0), "J3": (0.3, 15e-3, 1.5)}
    methods = {"1f1b": (A.ARB_HINT_FIXED_1F1B, b + w, None), "rrfp_bf": (A.ARB_HINT_BF, b + w, None),
               "rrfp_bfw": (A.ARB_HINT_BFW, b, w)}
    table = {}
    for lv, (p, base, alpha) in levels.items():
        row = {}
        for name, (hint, bb, ww) in methods.items():
            ms, bub = [], []
            for seed in range(1 if p == 0.0 else 10):
                r = A.rrfp_sim_run(N, M, f, bb, ww, hint=hint, buffer_limit=32, jitter=(p, base, alpha, 1000 + seed),
                                   want_trace=False)
                assert not r["deadlock"]
                ms.append(r["makespan"] * 1e3)
                bub.append(1.0 - float(r["busy"].sum()) / (N * r["makespan"]))
            row[name] = {"iteration_ms": round(float(np.mean(ms)), 3), "bubble_frac": round(float(np.mean(bub)), 4)}
        for name in ("rrfp_bf", "rrfp_bfw"):
            row[name]["speedup_vs_1f1b"] = round(row["1f1b"]["iteration_ms"] / row[name]["iteration_ms"], 4)
        table[lv] = row
    # decision throughput of the native arbiter + event loop, and the oracle on a bounded sample
    rng = np.random.default_rng(7)
    Nb, Mb = 64, 2048
    fb, bb = rng.uniform(0.5, 2.0, (Nb, 1, Mb)), rng.uniform(1.0, 4.0, (Nb, 1, Mb))
    t0 = time.perf_counter()
    r = A.rrfp_sim_run(Nb, Mb, fb, bb, None, want_trace=False)
    native_rate = r["n_events"] / (time.perf_counter() - t0)
    out = {"only": "pipeline", "metric": "simulated iteration time of an N-stage pipeline built from measured task times",
           "workload": shape.name, "n_stages": N, "n_microbatches": M,
           "tokens_per_microbatch": [int(c[-1]) for c in cus],
           "task_ms": {k: [round(v * 1e3, 3) for v in per_mb[k]] for k in ("F", "B", "W")},
           "buffer_limit": 32, "levels": table,
           "simulator": {"tasks_per_s": round(native_rate), "n_stages": Nb, "n_microbatches": Mb}}
    if with_oracle:
        from oracle import arbiter_oracle as O
        No, Mo = 8, 256
        t0 = time.perf_counter()
        ro = O.simulate(No, Mo, lambda d, s, c, j: float(fb[s, 0, j] if d == O.F else bb[s, 0, j]))
        out["cpu_baseline"] = {"value": round(2 * No * Mo / (time.perf_counter() - t0)), "unit": "tasks/s", "cores": 1,
                               "kind": "oracle", "sample": f"python oracle simulator, {No} stages x {Mo} microbatches"}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="language")
    ap.add_argument("--streams", type=int, default=1, help="streams the tasks are dealt to (B/F/W order)")
    ap.add_argument("--gemm-form", default=None, choices=["nn", "nt", "tn"],
                    help="operand orientation of the roofline GEMM (forward, input-gradient or weight-gradient form of the "
                         "up projection); default: tn, the form with the largest share of the step")
    ap.add_argument("--only", default="step", choices=["step", "gemm", "gemm_sweep", "copy", "pipeline"],
                    help="gemm: launch only the roofline GEMM (for counter runs); gemm_sweep: time of the GEMM forms against "
                         "K with a full, a half and a quarter round of 256 x 256 tiles (main-loop rate and fixed cost per "
                         "launch, with and without every CU busy); copy: a 2 GiB device copy, the "
                         "calibration of the FETCH_SIZE / WRITE_SIZE counters; pipeline: measure the per-microbatch "
                         "task times of the workload and replay them through the native pipeline simulator "
                         "(fixed 1F1B against readiness-driven dispatch, jitter levels J0-J3)")
    ap.add_argument("--sweep-launches", type=int, default=200, help="timed (and warm-up) launches per row of --only gemm_sweep")
    ap.add_argument("--pipeline-stages", type=int, default=8)
    ap.add_argument("--rope", action="store_true", help="turn on the rotary-embedding variant of the layer (off in the headline workload)")
    ap.add_argument("--qk-norm", action="store_true", help="turn on the QK-norm variant of the layer (off in the headline workload)")
    ap.add_argument("--layernorm-bias", action="store_true",
                    help="turn on the LayerNorm + projection-bias variant of the layer (off in the five workloads)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=4096)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2605_18750_amd as R
    from paper_2605_18750_amd import harness as Hn
    import stage_inputs as SI

    R.lib()   # fails loudly if the HIP library is not built
    if args.only == "pipeline" and args.workload == "language":
        args.workload = "multimodal"      # the workload whose microbatches differ in cost
    shape = {"language": SI.LANGUAGE, "wide": SI.WIDE_GQA, "vision": SI.VISION, "multimodal": SI.MULTIMODAL,
             "tiny": SI.TINY}[args.workload]
    if args.rope:
        shape = shape.replace(rope=True, name=shape.name + "+rope")
    if args.qk_norm:
        shape = shape.replace(qk_norm=True, name=shape.name + "+qknorm")
    if args.layernorm_bias:
        shape = shape.replace(norm_kind="layer", bias=True, name=shape.name + "+layernorm+bias")
    if args.only == "gemm_sweep":
        torch.cuda.set_device(0)
        print(json.dumps({"only": "gemm_sweep", "rows": gemm_sweep(torch.cuda.Stream(), n_launch=args.sweep_launches)}))
        return
    if args.only in ("gemm", "copy"):
        torch.cuda.set_device(0)
        gen = torch.Generator(device="cuda:0")
        gen.manual_seed(SI.BASE_SEED)
        if args.only == "copy":
            src = torch.empty(1 << 31, dtype=torch.uint8, device="cuda:0")
            dst = torch.empty_like(src)
            for _ in range(3):
                dst.copy_(src)
            torch.cuda.synchronize()
            print(json.dumps({"only": "copy", "bytes_read": 1 << 31, "bytes_written": 1 << 31, "launches": 3}))
            return
        T = max(int(SI.default_cu_seqlens(shape, j)[-1]) for j in range(shape.n_microbatches))
        N_up = (2 if shape.mlp_kind == "swiglu" else 1) * shape.ffn
        Bw = torch.empty((shape.hidden, N_up), dtype=torch.bfloat16, device="cuda:0").normal_(0.0, shape.w_std, generator=gen)
        print(json.dumps({"only": "gemm", "roofline": gemm_roofline(shape, T, Bw, torch.cuda.Stream(), gen, n_launch=args.steps,
                                                                    form=args.gemm_form or "tn")}))
        return
    M = shape.n_microbatches
    cus = [SI.default_cu_seqlens(shape, j) for j in range(M)]
    T_max = max(int(c[-1]) for c in cus)
    cfg = Hn.make_config(shape, T_max, max(len(c) - 1 for c in cus))
    dev = "cuda:0"
    torch.cuda.set_device(0)
    tdt = torch.float32 if shape.dtype == "fp32" else torch.bfloat16

    # Synthetic inputs, generated on the device from a fixed seed: weights N(0, w_std), gains
    # 1 + N(0, w_std), x N(0, x_std), dy N(0, dy_std).
    gen = torch.Generator(device=dev)
    gen.manual_seed(SI.BASE_SEED)
    pb, gb, ab = R.stage_query(cfg)
    esz = 4 if shape.dtype == "fp32" else 2
    params = torch.empty(pb // esz, dtype=tdt, device=dev)
    params.normal_(0.0, shape.w_std, generator=gen)
    for l in range(cfg.n_layers):
        for which in (R.STAGE_P_G1, R.STAGE_P_G2):
            off, (r, _) = R.stage_param_layout(cfg, l, which)
            params[off:off + r] += 1.0
    arena = torch.empty(ab, dtype=torch.uint8, device=dev)
    grad_out = torch.empty(gb // 4, dtype=torch.float32, device=dev)
    st = R.stage_create(cfg, params, arena, ab)
    xs = [torch.empty((int(c[-1]), shape.hidden), dtype=tdt, device=dev).normal_(0.0, shape.x_std, generator=gen) for c in cus]
    dys = [torch.empty((int(c[-1]), shape.hidden), dtype=tdt, device=dev).normal_(0.0, shape.dy_std, generator=gen) for c in cus]
    ys = [torch.empty_like(x) for x in xs]
    dxs = [torch.empty_like(x) for x in xs]
    streams = [torch.cuda.Stream() for _ in range(max(1, args.streams))]

    fl = [task_flops(shape, c) for c in cus]
    step_flops = sum(f["F"] + f["B"] + f["W"] for f in fl)

    # Issue order: all F, then for each microbatch B then W (a B/F/W-style drain), dealt to streams.
    order = [("F", j) for j in range(M)]
    for j in range(M):
        order += [("B", j), ("W", j)]

    def step(events=None):
        for i, (kind, j) in enumerate(order):
            s = streams[i % len(streams)]
            if events is not None:
                e0 = torch.cuda.Event(enable_timing=True)
                e0.record(s)
            if kind == "F":
                R.stage_F(st, j, xs[j], cus[j], ys[j], s)
            elif kind == "B":
                R.stage_B(st, j, dys[j], dxs[j], s)
            else:
                R.stage_W(st, j, s)
            if events is not None:
                e1 = torch.cuda.Event(enable_timing=True)
                e1.record(s)
                events.append((kind, j, e0, e1))
        if events is not None:
            e0 = torch.cuda.Event(enable_timing=True)
            e0.record(streams[0])
        R.stage_grad_reduce(st, grad_out, streams[0])
        if events is not None:
            e1 = torch.cuda.Event(enable_timing=True)
            e1.record(streams[0])
            events.append(("R", -1, e0, e1))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3

    # Per-task times (one stream, events around every task), outside the timed region.
    saved = streams
    streams = streams[:1]
    per_kind = {"F": [], "B": [], "W": [], "R": []}
    for _ in range(3):
        ev = []
        step(ev)
        torch.cuda.synchronize()
        for kind, j, e0, e1 in ev:
            per_kind[kind].append((j, e0.elapsed_time(e1)))
    streams = saved
    tasks = {}
    red_ms = float(np.median([t for _, t in per_kind.pop("R")]))
    if args.only == "pipeline":
        per_mb = {k: [float(np.median([t for jj, t in lst if jj == j])) * 1e-3 for j in range(M)] for k, lst in per_kind.items()}
        torch.cuda.synchronize()
        R.stage_destroy(st)
        del arena
        print(json.dumps(pipeline_study(shape, cus, per_mb, args.pipeline_stages, not args.no_cpu_baseline)))
        return
    for kind, lst in per_kind.items():
        ms = float(np.median([t for _, t in lst]))
        tf = float(np.median([fl[j][kind] / (t * 1e-3) / 1e12 for j, t in lst]))
        p5, p95 = (float(v) for v in np.percentile([t for _, t in lst], [5, 95]))
        tasks[kind] = {"ms_per_microbatch": round(ms, 4), "p5_ms": round(p5, 4), "p95_ms": round(p95, 4),
                       "samples": len(lst), "tflops": round(tf, 1),
                       "frac_of_bf16_mfma_peak": round(tf / PEAK_BF16_TFLOPS, 4)}
    # stage_grad_reduce alone (HBM-bound): (M + 1) gradient buffers move per call.
    red_gbs = (M + 1) * gb / (red_ms * 1e-3) / 1e9
    grad_reduce = {"ms": round(red_ms, 4), "GB/s": round(red_gbs, 1), "frac_of_hbm_peak": round(red_gbs / PEAK_HBM_GBS, 4),
                   "bytes": (M + 1) * gb}
    # Roofline of the dominant kernel: the weight-gradient GEMM of the up projection ([hidden, N_up] with
    # K = tokens, fp32 out), the single launch with the largest share of the step and the form (both operands
    # K-strided) that takes the largest share of the step overall; timed alone with HIP events on its stream.
    roof, hbm = None, None
    if shape.dtype == "bf16":
        off, (r, c) = R.stage_param_layout(cfg, 0, R.STAGE_P_WUP)
        roof = gemm_roofline(shape, T_max, params[off:off + r * c].view(r, c), streams[0], gen, form=args.gemm_form or "tn")

    torch.cuda.synchronize()
    R.stage_destroy(st)
    del arena
    if shape.dtype == "bf16":
        hbm = hbm_kernels(shape, T_max, M, gb // 4, streams[0], gen)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(shape, args.cpu_sample_tokens)

    value = step_flops / wall * args.steps / 1e12
    out = {
        "metric": "F/B/W task TFLOP/s per stage (bf16), % of MFMA peak; ms per microbatch",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"{shape.name}: {shape.n_layers} layers, hidden {shape.hidden}, {shape.n_q_heads} q heads / "
                               f"{shape.n_kv_heads} kv heads x {shape.head_dim}, ffn {shape.ffn} {shape.mlp_kind}, "
                               f"{'causal' if shape.causal else 'bidirectional'}, T per microbatch "
                               f"{sorted(set(int(c[-1]) for c in cus))}, {M} microbatches",
                   "step": "F, B, W of every microbatch + stage_grad_reduce", "streams": len(streams),
                   "step_tflop": round(step_flops / 1e12, 3)},
        "frac_of_bf16_mfma_peak": round(value / PEAK_BF16_TFLOPS, 4),
        "tasks": tasks,
        "grad_reduce": grad_reduce,
        "roofline": roof,
        "hbm_kernels": hbm,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
