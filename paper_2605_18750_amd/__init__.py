"""Thin ctypes binding of librrfp_stage.so: the same names as include/rrfp_stage.h and
argument marshalling only.  Every step of the F/B/W path runs in the library's HIP kernels;
this module fails loudly if the library is missing."""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "librrfp_stage.so")

STAGE_OK, STAGE_EINVAL, STAGE_ENOTREADY, STAGE_ENOMEM, STAGE_EHIP = 0, -1, -2, -3, -4
STAGE_DTYPE_FP32, STAGE_DTYPE_BF16 = 0, 1
STAGE_MLP_SWIGLU, STAGE_MLP_GELU = 0, 1
(STAGE_P_G1, STAGE_P_WQKV, STAGE_P_WO, STAGE_P_G2, STAGE_P_WUP, STAGE_P_WD, STAGE_P_B1, STAGE_P_BQKV, STAGE_P_BO,
 STAGE_P_B2, STAGE_P_BUP, STAGE_P_BD, STAGE_P_GQ, STAGE_P_GK, STAGE_P_COUNT) = range(15)


class stage_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "max_tokens",
        "n_microbatches", "max_segments", "dtype", "mlp_kind", "causal", "norm_kind")] + [
        ("norm_eps", C.c_float), ("rope", C.c_int32), ("rope_base", C.c_float), ("bias", C.c_int32), ("qk_norm", C.c_int32)]


class StageError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"stage error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Loads the library (built by `python -m paper_2605_18750_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2605_18750_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, sz = C.c_void_p, C.c_size_t
        cfgp = C.POINTER(stage_config)
        L.stage_query.argtypes = [cfgp, C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
        L.stage_param_layout.argtypes = [cfgp, C.c_int, C.c_int, C.POINTER(sz), C.POINTER(C.c_int64)]
        L.stage_create.argtypes = [cfgp, vp, vp, sz, C.POINTER(vp)]
        L.stage_create_dry.argtypes = [cfgp, C.POINTER(vp)]
        L.stage_F.argtypes = [vp, C.c_int, vp, C.POINTER(C.c_int32), C.c_int, vp, vp]
        L.stage_B.argtypes = [vp, C.c_int, vp, vp, vp]
        L.stage_W.argtypes = [vp, C.c_int, vp]
        L.stage_grad_reduce.argtypes = [vp, vp, vp]
        L.stage_grad_slot.argtypes = [vp, C.c_int, C.POINTER(vp)]
        L.stage_intermediate.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.POINTER(vp)]
        L.stage_intermediate.restype = C.c_int
        L.stage_destroy.argtypes = [vp]
        L.stage_last_error.argtypes = [vp]
        L.stage_last_error.restype = C.c_char_p
        L.rrfp_gemm.argtypes = [vp, vp, vp, vp] + [C.c_int] * 12 + [vp]
        L.rrfp_gemm.restype = C.c_int
        L.rrfp_gemm_ws.argtypes = [vp, vp, vp, vp] + [C.c_int] * 12 + [vp, sz, vp]
        L.rrfp_gemm_ws.restype = C.c_int
        L.rrfp_gemm_plan.argtypes = [C.c_int] * 11 + [C.POINTER(C.c_int32)]
        L.rrfp_gemm_plan.restype = C.c_int
        L.rrfp_attn_dkv_subsets.argtypes = [C.c_int] * 4
        L.rrfp_attn_dkv_subsets.restype = C.c_int
        L.rrfp_rmsnorm_fwd.argtypes = [vp, vp, vp, vp, C.c_int, C.c_int, C.c_float, C.c_int, vp]
        L.rrfp_rmsnorm_fwd.restype = C.c_int
        L.rrfp_rmsnorm_bwd_workspace.argtypes = [C.c_int, C.c_int, C.c_int]
        L.rrfp_rmsnorm_bwd_workspace.restype = sz
        L.rrfp_rmsnorm_bwd.argtypes = [vp] * 9 + [sz, C.c_int, C.c_int, C.c_int, vp]
        L.rrfp_rmsnorm_bwd.restype = C.c_int
        L.rrfp_rmsnorm_bwd_static_limit.argtypes = []
        L.rrfp_rmsnorm_bwd_static_limit.restype = sz
        L.rrfp_rmsnorm_bwd_static.argtypes = [vp] * 8 + [C.c_int, C.c_int, C.c_int, vp]
        L.rrfp_rmsnorm_bwd_static.restype = C.c_int
        L.rrfp_grad_reduce.argtypes = [vp, sz, C.c_int, vp, sz, vp]
        L.rrfp_grad_reduce.restype = C.c_int
        for f in ("stage_query", "stage_param_layout", "stage_create", "stage_create_dry", "stage_F",
                  "stage_B", "stage_W", "stage_grad_reduce", "stage_grad_slot", "stage_destroy"):
            getattr(L, f).restype = C.c_int
        _lib = L
    return _lib


def _ptr(t) -> int:
    """Device/host address of a torch tensor, or an int address, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(s) -> int:
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream


def _check(rc: int, st=None):
    if rc != STAGE_OK:
        raise StageError(rc, stage_last_error(st))


def stage_last_error(st=None) -> str:
    return lib().stage_last_error(st).decode()


def stage_query(cfg: stage_config):
    """-> (param_bytes, grad_bytes, arena_bytes)"""
    a, b, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().stage_query(C.byref(cfg), C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def stage_param_layout(cfg: stage_config, layer: int, which: int):
    """-> (offset_elems, (rows, cols))"""
    off = C.c_size_t()
    shape = (C.c_int64 * 2)()
    _check(lib().stage_param_layout(C.byref(cfg), layer, which, C.byref(off), shape))
    return off.value, (shape[0], shape[1])


def stage_create(cfg: stage_config, params_dev, arena_dev, arena_bytes: int):
    h = C.c_void_p()
    _check(lib().stage_create(C.byref(cfg), _ptr(params_dev), _ptr(arena_dev), arena_bytes, C.byref(h)))
    return h


def stage_create_dry(cfg: stage_config):
    h = C.c_void_p()
    _check(lib().stage_create_dry(C.byref(cfg), C.byref(h)))
    return h


def stage_F(st, mb: int, x_dev, cu_seqlens, y_dev, stream=None):
    n = len(cu_seqlens) - 1
    cu = (C.c_int32 * (n + 1))(*[int(v) for v in cu_seqlens])
    _check(lib().stage_F(st, mb, _ptr(x_dev), cu, n, _ptr(y_dev), _stream(stream)), st)


def stage_B(st, mb: int, dy_dev, dx_dev, stream=None):
    _check(lib().stage_B(st, mb, _ptr(dy_dev), _ptr(dx_dev), _stream(stream)), st)


def stage_W(st, mb: int, stream=None):
    _check(lib().stage_W(st, mb, _stream(stream)), st)


def stage_grad_reduce(st, grad_out_dev, stream=None):
    _check(lib().stage_grad_reduce(st, _ptr(grad_out_dev), _stream(stream)), st)


def stage_grad_slot(st, mb: int) -> int:
    p = C.c_void_p()
    _check(lib().stage_grad_slot(st, mb, C.byref(p)), st)
    return p.value


(STAGE_T_X, STAGE_T_H1, STAGE_T_QKV, STAGE_T_O, STAGE_T_X1, STAGE_T_H2, STAGE_T_UP, STAGE_T_M, STAGE_T_DY,
 STAGE_T_DUP, STAGE_T_DX1, STAGE_T_DQKV, STAGE_T_LSE, STAGE_T_H1_HALF, STAGE_T_COUNT) = range(15)


def stage_intermediate(st, mb: int, layer: int, which: int) -> int:
    p = C.c_void_p()
    _check(lib().stage_intermediate(st, mb, layer, which, C.byref(p)), st)
    return p.value


RRFP_GEMM_AUTO, RRFP_GEMM_SIMT, RRFP_GEMM_MFMA = 0, 1, 2


def rrfp_gemm(A, B, Cout, R, M, N, K, lda, ldb, ldc, ldr, trans_a, trans_b, in_dtype, out_dtype,
              family=RRFP_GEMM_AUTO, stream=None, workspace=None, workspace_bytes=0):
    """workspace given: rrfp_gemm_ws (the weight-gradient form may then split along K)."""
    if workspace is not None:
        rc = lib().rrfp_gemm_ws(_ptr(A), _ptr(B), _ptr(Cout), _ptr(R), M, N, K, lda, ldb, ldc, ldr, int(trans_a), int(trans_b),
                                in_dtype, out_dtype, family, _ptr(workspace), workspace_bytes, _stream(stream))
    else:
        rc = lib().rrfp_gemm(_ptr(A), _ptr(B), _ptr(Cout), _ptr(R), M, N, K, lda, ldb, ldc, ldr,
                             int(trans_a), int(trans_b), in_dtype, out_dtype, family, _stream(stream))
    if rc != STAGE_OK:
        raise StageError(rc, "rrfp_gemm rejected its arguments" if rc == STAGE_EINVAL else "HIP launch failed")


def rrfp_attn_dkv_subsets(n_q_heads, n_kv_heads, n_kv_tiles, n_cu=256):
    """Workgroups that share the query heads of one KV head in the dK/dV kernel (pure host logic)."""
    rc = lib().rrfp_attn_dkv_subsets(n_q_heads, n_kv_heads, n_kv_tiles, n_cu)
    if rc < 1:
        raise StageError(rc, "rrfp_attn_dkv_subsets rejected its arguments")
    return rc


def rrfp_gemm_plan(M, N, K, trans_a, trans_b, out_dtype, n_cu=256, have_scratch=False, lda=None, ldb=None, ldc=None):
    """Launch plan of the bf16 MFMA GEMM for a shape (host logic only, no GPU): dict with kernel
    (0 refused, 1 direct-to-LDS, 2 register-staged), wavefronts, main_workgroups, short_workgroups, split_k."""
    lda = (M if trans_a else K) if lda is None else lda
    ldb = (K if trans_b else N) if ldb is None else ldb
    ldc = N if ldc is None else ldc
    out = (C.c_int32 * 5)()
    rc = lib().rrfp_gemm_plan(M, N, K, lda, ldb, ldc, int(trans_a), int(trans_b), out_dtype, int(have_scratch), n_cu, out)
    if rc != STAGE_OK:
        raise StageError(rc, "rrfp_gemm_plan rejected its arguments")
    return dict(zip(("kernel", "wavefronts", "main_workgroups", "short_workgroups", "split_k"), (int(v) for v in out)))


def _kcheck(rc: int, name: str):
    if rc != STAGE_OK:
        raise StageError(rc, f"{name} rejected its arguments" if rc == STAGE_EINVAL else f"{name}: HIP launch failed")


def rrfp_rmsnorm_fwd(x, g, h, r_out, T: int, H: int, eps: float, dtype: int, stream=None):
    _kcheck(lib().rrfp_rmsnorm_fwd(_ptr(x), _ptr(g), _ptr(h), _ptr(r_out), T, H, eps, dtype, _stream(stream)), "rrfp_rmsnorm_fwd")


def rrfp_rmsnorm_bwd_workspace(T: int, H: int, dtype: int) -> int:
    return lib().rrfp_rmsnorm_bwd_workspace(T, H, dtype)


def rrfp_rmsnorm_bwd(dh, x, r, g, add_in, out32, out_t, dg, workspace, workspace_bytes: int, T: int, H: int, dtype: int,
                     stream=None):
    _kcheck(lib().rrfp_rmsnorm_bwd(_ptr(dh), _ptr(x), _ptr(r), _ptr(g), _ptr(add_in), _ptr(out32), _ptr(out_t), _ptr(dg),
                                   _ptr(workspace), workspace_bytes, T, H, dtype, _stream(stream)), "rrfp_rmsnorm_bwd")


def rrfp_rmsnorm_bwd_static_limit() -> int:
    return lib().rrfp_rmsnorm_bwd_static_limit()


def rrfp_rmsnorm_bwd_static(dh, x, r, g, add_in, out32, out_t, dg, T: int, H: int, dtype: int, stream=None):
    rc = lib().rrfp_rmsnorm_bwd_static(_ptr(dh), _ptr(x), _ptr(r), _ptr(g), _ptr(add_in), _ptr(out32), _ptr(out_t), _ptr(dg),
                                       T, H, dtype, _stream(stream))
    if rc == STAGE_ENOMEM:
        raise StageError(rc, "rrfp_rmsnorm_bwd_static: shape needs more than the library's static scratch")
    _kcheck(rc, "rrfp_rmsnorm_bwd_static")


def rrfp_grad_reduce(slots, slot_stride: int, M: int, out, n: int, stream=None):
    _kcheck(lib().rrfp_grad_reduce(_ptr(slots), slot_stride, M, _ptr(out), n, _stream(stream)), "rrfp_grad_reduce")


def stage_destroy(st):
    _check(lib().stage_destroy(st))
