"""Host-side checks that need no GPU: the library loads and exports every symbol the header
declares; configuration validation; parameter layout; the per-microbatch dependency state
machine (paper Section 3.1 / 4.1 / 7.1 ordering rules) through stage_create_dry."""
import os
import re
import ctypes

import pytest

import paper_2605_18750_amd as R
from paper_2605_18750_amd import harness as Hn
import stage_inputs as SI

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(**kw):
    base = dict(n_layers=2, hidden=128, n_q_heads=4, n_kv_heads=2, head_dim=32, ffn=192, max_tokens=64,
                n_microbatches=3, max_segments=2, dtype=0, mlp_kind=0, causal=1, norm_kind=0, norm_eps=1e-5,
                rope=0, rope_base=10000.0, bias=0, qk_norm=0)
    base.update(kw)
    return R.stage_config(**base)


def test_library_exports_every_declared_symbol():
    inc = os.path.join(ROOT, "include")
    hdr = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b((?:stage|rrfp|arbiter)_[A-Za-z_0-9]+)\s*\(", hdr))
    assert {"stage_create", "stage_F", "stage_B", "stage_W", "stage_grad_reduce", "arbiter_next", "rrfp_sim_run"} <= names
    L = ctypes.CDLL(R.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n


def test_config_validation():
    R.stage_query(_cfg())
    bad = [dict(n_kv_heads=3), dict(hidden=0), dict(head_dim=24), dict(head_dim=144), dict(dtype=2),
           dict(mlp_kind=5), dict(causal=2), dict(norm_kind=2), dict(bias=2), dict(qk_norm=3), dict(norm_eps=-1.0), dict(rope=2), dict(rope=1, rope_base=1.0), dict(ffn=190),
           dict(dtype=1, head_dim=32), dict(dtype=1, head_dim=64, hidden=96), dict(n_layers=65)]
    for kw in bad:
        with pytest.raises(R.StageError) as e:
            R.stage_query(_cfg(**kw))
        assert e.value.code == R.STAGE_EINVAL, kw
        assert len(str(e.value)) > 20


def test_layout_is_disjoint_aligned_and_sized():
    for shape, T in ((SI.TINY, 128), (SI.LANGUAGE, 4096), (SI.WIDE_GQA, 4096), (SI.VISION, 6272)):
        cfg = Hn.make_config(shape, T, 8)
        pb, gb, ab = R.stage_query(cfg)
        esz = 4 if shape.dtype == "fp32" else 2
        spans = []
        for l in range(cfg.n_layers):
            for w in range(R.STAGE_P_COUNT):
                off, (r, c) = R.stage_param_layout(cfg, l, w)
                assert off % 128 == 0
                spans.append((off, off + r * c))
        spans.sort()
        assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
        assert spans[-1][1] * esz <= pb and gb == pb // esz * 4 and ab > 0
    cfg = Hn.make_config(SI.WIDE_GQA, 4096)
    assert R.stage_param_layout(cfg, 0, R.STAGE_P_WQKV)[1] == (8192, (64 + 16) * 128)
    assert R.stage_param_layout(cfg, 1, R.STAGE_P_WUP)[1] == (8192, 2 * 28672)
    assert R.stage_param_layout(Hn.make_config(SI.VISION, 6272, 8), 0, R.STAGE_P_WUP)[1] == (1280, 5120)
    with pytest.raises(R.StageError):
        R.stage_param_layout(cfg, 2, 0)
    with pytest.raises(R.StageError):
        R.stage_param_layout(cfg, 0, R.STAGE_P_COUNT)
    # vectors of the variants: zero-sized when off, [n, 1] when on, still disjoint and aligned
    assert R.stage_param_layout(cfg, 0, R.STAGE_P_BQKV)[1] == (0, 1)
    on = Hn.make_config(SI.VISION.replace(norm_kind="layer", bias=True), 6272, 8)
    assert R.stage_param_layout(on, 0, R.STAGE_P_B1)[1] == (1280, 1)
    assert R.stage_param_layout(on, 3, R.STAGE_P_BQKV)[1] == (3 * 1280, 1)
    assert R.stage_param_layout(on, 3, R.STAGE_P_BUP)[1] == (5120, 1)
    spans = sorted((lambda o, rc: (o, o + rc[0] * rc[1]))(*R.stage_param_layout(on, l, w))
                   for l in range(on.n_layers) for w in range(R.STAGE_P_COUNT))
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))


def test_language_arena_fits_one_gpu():
    for shape, T, nseg in ((SI.LANGUAGE, 4096, 1), (SI.WIDE_GQA, 4096, 1), (SI.MULTIMODAL, 6144, 2), (SI.VISION, 6272, 8)):
        pb, gb, ab = R.stage_query(Hn.make_config(shape, T, nseg))
        assert pb + gb + ab < 250 * 2 ** 30, (shape.name, (pb + gb + ab) / 2 ** 30)


def _expect(code, fn, *a):
    with pytest.raises(R.StageError) as e:
        fn(*a)
    assert e.value.code == code, str(e.value)


def test_dependency_state_machine():
    st = R.stage_create_dry(_cfg())
    cu = [0, 40, 64]
    _expect(R.STAGE_ENOTREADY, R.stage_B, st, 0, None, None)          # B before F
    _expect(R.STAGE_ENOTREADY, R.stage_W, st, 0)                      # W before B
    _expect(R.STAGE_ENOTREADY, R.stage_grad_reduce, st, None)         # reduce before all W
    R.stage_F(st, 0, None, cu, None)
    _expect(R.STAGE_ENOTREADY, R.stage_F, st, 0, None, cu, None)      # slot busy
    _expect(R.STAGE_ENOTREADY, R.stage_W, st, 0)
    R.stage_F(st, 2, None, [0, 10], None)                             # any ready order
    R.stage_B(st, 2, None, None)
    _expect(R.STAGE_ENOTREADY, R.stage_B, st, 2, None, None)          # double issue
    R.stage_B(st, 0, None, None)
    R.stage_F(st, 1, None, cu, None)
    R.stage_W(st, 0)
    _expect(R.STAGE_ENOTREADY, R.stage_W, st, 0)
    _expect(R.STAGE_ENOTREADY, R.stage_F, st, 0, None, cu, None)      # busy until the reduce
    R.stage_B(st, 1, None, None)
    R.stage_W(st, 1)                                                  # W may trail other microbatches' work
    _expect(R.STAGE_ENOTREADY, R.stage_grad_reduce, st, None)
    R.stage_W(st, 2)
    R.stage_grad_reduce(st, None)
    R.stage_F(st, 0, None, cu, None)                                  # slots are free again
    R.stage_destroy(st)


def test_argument_validation_has_no_side_effect():
    st = R.stage_create_dry(_cfg())
    _expect(R.STAGE_EINVAL, R.stage_F, st, 3, None, [0, 8], None)     # mb out of range
    _expect(R.STAGE_EINVAL, R.stage_F, st, -1, None, [0, 8], None)
    _expect(R.STAGE_EINVAL, R.stage_F, st, 0, None, [1, 8], None)     # cu[0] != 0
    _expect(R.STAGE_EINVAL, R.stage_F, st, 0, None, [0, 8, 8], None)  # empty segment
    _expect(R.STAGE_EINVAL, R.stage_F, st, 0, None, [0, 9, 5], None)  # not monotone
    _expect(R.STAGE_EINVAL, R.stage_F, st, 0, None, [0, 65], None)    # T > max_tokens
    _expect(R.STAGE_EINVAL, R.stage_F, st, 0, None, [0, 1, 2, 3], None)  # too many segments
    _expect(R.STAGE_EINVAL, R.stage_F, st, 0, None, [0], None)        # no segment
    assert "max_tokens" in R.stage_last_error(st) or len(R.stage_last_error(st)) > 0
    R.stage_F(st, 0, None, [0, 64], None)                             # still free after the failures
    _expect(R.STAGE_EINVAL, R.stage_B, st, 7, None, None)
    _expect(R.STAGE_EINVAL, R.stage_W, st, 7)
    R.stage_destroy(st)


def test_real_create_rejects_bad_buffers_before_any_hip_call():
    cfg = _cfg()
    _, _, ab = R.stage_query(cfg)
    _expect(R.STAGE_EINVAL, R.stage_create, cfg, None, None, ab)
    _expect(R.STAGE_EINVAL, R.stage_create, cfg, 256 + 8, 4096, ab)     # misaligned
    _expect(R.STAGE_ENOMEM, R.stage_create, cfg, 256, 4096, ab - 1)     # arena too small


def test_gemm_launch_plan_is_a_pure_function_of_shape_and_cu_count():
    """The cut of a GEMM into launches (tile rows, tail launch, split-K ranges) decides the order in which
    every output element is summed; it may depend on the shape and the device's CU count only.  Language-stage
    shapes on 256 CUs: the forward up projection is 1280 workgroups of 256-row tiles (exactly 5 rounds) plus 192
    of 128-row tiles for the 6 trailing tile columns; the one-round input-gradient shape is untouched; the
    weight-gradient form runs 2 x 2 wavefronts and is only split along K when its grid leaves CUs idle."""
    import paper_2605_18750_amd as R
    BF, F32 = R.STAGE_DTYPE_BF16, R.STAGE_DTYPE_FP32
    T, H, F2, Q = 4096, 4096, 22016, 12288
    up = R.rrfp_gemm_plan(T, F2, H, 0, 0, BF)
    assert up == dict(kernel=1, wavefronts=8, main_workgroups=1280, short_workgroups=192, split_k=1)
    assert R.rrfp_gemm_plan(T, F2, H, 0, 0, BF) == up                      # same answer every time
    assert R.rrfp_gemm_plan(T, H, F2, 0, 1, F32) == dict(kernel=1, wavefronts=8, main_workgroups=256, short_workgroups=0, split_k=1)
    assert R.rrfp_gemm_plan(T, Q, H, 0, 0, BF)["main_workgroups"] == 768   # 3 full rounds: no tail launch
    assert R.rrfp_gemm_plan(T, Q, H, 0, 0, BF)["short_workgroups"] == 0
    # weight gradient of the up projection: 16 x 86 = 1376 tiles = 5.4 rounds; the 6 trailing tile columns (96
    # tiles) become a tail launch split along K into 2 ranges (192 workgroups, half a round) when scratch exists
    wg = R.rrfp_gemm_plan(H, F2, T, 1, 0, F32, have_scratch=True)
    assert wg == dict(kernel=1, wavefronts=4, main_workgroups=1280, short_workgroups=192, split_k=2)
    assert R.rrfp_gemm_plan(H, F2, T, 1, 0, F32, have_scratch=False) == dict(kernel=1, wavefronts=4, main_workgroups=1376,
                                                                            short_workgroups=0, split_k=1)
    # down projection (43 x 16 = 688 tiles): the 176 left-over tiles do not fit a split tail: one plain launch
    assert R.rrfp_gemm_plan(11008, H, T, 1, 0, F32, have_scratch=True) == dict(kernel=1, wavefronts=4, main_workgroups=688,
                                                                              short_workgroups=0, split_k=1)
    # whole rounds (QKV: 768 tiles) are left alone
    assert R.rrfp_gemm_plan(H, Q, T, 1, 0, F32, have_scratch=True)["short_workgroups"] == 0
    # vision stage: dW of the output projection, 1280 x 1280 with K = 6272 tokens: 25 tiles -> split along K
    small = R.rrfp_gemm_plan(1280, 1280, 6272, 1, 0, F32, have_scratch=True)
    assert small["main_workgroups"] == 25 and 1 < small["split_k"] <= 16
    assert R.rrfp_gemm_plan(1280, 1280, 6272, 1, 0, F32, have_scratch=False)["split_k"] == 1
    # a grid that fills at most half the CUs goes entirely to 128-row tiles
    assert R.rrfp_gemm_plan(1000, 2048, 1280, 0, 0, BF) == dict(kernel=1, wavefronts=8, main_workgroups=0, short_workgroups=64, split_k=1)
    # the CU count is an input: with 32 CUs the same 32 tiles are one full round of 256-row tiles
    assert R.rrfp_gemm_plan(1000, 2048, 1280, 0, 0, BF, n_cu=32) == dict(kernel=1, wavefronts=8, main_workgroups=32, short_workgroups=0, split_k=1)
    # K not a multiple of 32 with a K-contiguous operand: register-staged kernel; N not a multiple of 8: refused
    assert R.rrfp_gemm_plan(264, 520, 200, 0, 0, BF)["kernel"] == 2
    assert R.rrfp_gemm_plan(264, 516, 256, 0, 0, BF)["kernel"] == 0


def test_dkv_head_subsets_are_a_pure_function_of_shape():
    # one query head per KV head: never split (the language stage)
    assert R.rrfp_attn_dkv_subsets(32, 32, 32) == 1
    # wide-GQA stage: 8 KV heads x 32 key tiles = one workgroup per CU -> two subsets give two per CU
    assert R.rrfp_attn_dkv_subsets(64, 8, 32) == 2
    # enough key tiles already: no split; very few: the largest divisor of the group size up to 4
    assert R.rrfp_attn_dkv_subsets(64, 8, 64) == 1
    assert R.rrfp_attn_dkv_subsets(64, 8, 4) == 4
    assert R.rrfp_attn_dkv_subsets(4, 2, 3) == 2
    assert R.rrfp_attn_dkv_subsets(4, 1, 2) == 4
    assert R.rrfp_attn_dkv_subsets(6, 2, 1) == 3 and R.rrfp_attn_dkv_subsets(16, 2, 1) == 4 and R.rrfp_attn_dkv_subsets(10, 2, 1) == 1
    assert R.rrfp_attn_dkv_subsets(64, 8, 32, n_cu=128) == 1
    _expect(R.STAGE_EINVAL, R.rrfp_attn_dkv_subsets, 6, 4, 1)
