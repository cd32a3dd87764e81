"""Seeded synthetic inputs for the F/B/W stage-task path.

This module is input plumbing only: stage shapes, a counter-based normal
generator, and rounding of generated values to the storage dtype.  It holds
none of the layer arithmetic, so both the CPU oracle's tests and the GPU
harness draw their inputs from here and receive the SAME already-rounded values.

Generator: element i of tensor `name` under `seed` is a pure function of
(seed, name, i): two splitmix64-style 64-bit mixes give two uniforms, Box-Muller
turns them into one standard normal.  Values are produced in fp64, scaled, then
rounded (round-to-nearest-even) to fp32 or bf16; the rounded value is what both
sides consume.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field, asdict

import numpy as np

BASE_SEED = 2026

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


@dataclass(frozen=True)
class StageShape:
    """Shape of one pipeline stage (the stage_config fields that describe the model)."""
    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    n_microbatches: int
    dtype: str = "bf16"          # "fp32" | "bf16"
    mlp_kind: str = "swiglu"     # "swiglu" | "gelu"
    causal: bool = True
    norm_eps: float = 1e-5
    rope: bool = False            # rotary position embedding on q and k (model-fidelity variant)
    norm_kind: str = "rms"        # "rms" | "layer" (model-fidelity variant)
    bias: bool = False            # biases on the four projections (model-fidelity variant)
    qk_norm: bool = False         # RMSNorm over head_dim on q and k heads (model-fidelity variant)
    rope_base: float = 10000.0
    w_std: float = 0.02
    x_std: float = 1.0
    dy_std: float = 1.0

    def replace(self, **kw) -> "StageShape":
        d = asdict(self)
        d.update(kw)
        return StageShape(**d)


# The five workload configurations (shapes only).
TINY = StageShape("tiny_fp32", 1, 256, 4, 4, 64, 688, 4, dtype="fp32",
                  x_std=0.02, dy_std=0.02)
LANGUAGE = StageShape("language_bf16", 4, 4096, 32, 32, 128, 11008, 8)
WIDE_GQA = StageShape("wide_gqa_bf16", 2, 8192, 64, 8, 128, 28672, 4)
MULTIMODAL = StageShape("multimodal_varlen_bf16", 4, 4096, 32, 32, 128, 11008, 16)
VISION = StageShape("vision_bf16", 8, 1280, 16, 16, 80, 5120, 8,
                    mlp_kind="gelu", causal=False)

TINY_SEQ = 128
LANGUAGE_SEQ = 4096
WIDE_SEQ = 4096
VISION_TOKENS_PER_IMAGE = 784
VISION_IMAGES_PER_MB = 8
MULTIMODAL_IMAGE_TOKENS = (256, 1024, 2304, 4096)
MULTIMODAL_TEXT_RANGE = (512, 2048)


def _tensor_key(seed: int, name: str) -> np.uint64:
    h = hashlib.sha256(f"{seed}:{name}".encode()).digest()
    return np.uint64(int.from_bytes(h[:8], "little"))


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on a uint64 array (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def _uniform_bits(key: np.uint64, idx: np.ndarray, stream: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        ctr = idx * np.uint64(2) + np.uint64(stream)
        z = key + (ctr + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15)
    return _mix(z)


def uniform_ints(seed: int, name: str, n: int, lo: int, hi: int) -> np.ndarray:
    """n integers uniform on [lo, hi] inclusive (modulo draw; bias < 2^-50)."""
    key = _tensor_key(seed, name)
    bits = _uniform_bits(key, np.arange(n, dtype=np.uint64), 0)
    return (lo + (bits % np.uint64(hi - lo + 1)).astype(np.int64)).astype(np.int64)


def normal_f64(seed: int, name: str, shape, std: float = 1.0, mean: float = 0.0,
               chunk: int = 1 << 22) -> np.ndarray:
    """Standard normals scaled to N(mean, std^2), fp64, element i a function of (seed,name,i)."""
    n = int(np.prod(shape))
    key = _tensor_key(seed, name)
    out = np.empty(n, dtype=np.float64)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        idx = np.arange(s, e, dtype=np.uint64)
        b1 = _uniform_bits(key, idx, 0)
        b2 = _uniform_bits(key, idx, 1)
        # 53-bit uniforms; u1 in (0,1], u2 in [0,1)
        u1 = ((b1 >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
        u2 = (b2 >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
        out[s:e] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    out *= std
    if mean != 0.0:
        out += mean
    return out.reshape(shape)


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp64/fp32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    f32 = np.ascontiguousarray(x, dtype=np.float32)
    bits = f32.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = bits + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


@dataclass
class Tensor:
    """One generated tensor: the rounded values (fp64 view) and their storage bits."""
    f64: np.ndarray            # exactly-representable values, fp64
    storage: np.ndarray        # float32 array (fp32) or uint16 bf16 bit patterns (bf16)
    dtype: str


def make_tensor(seed: int, name: str, shape, std: float, dtype: str, mean: float = 0.0) -> Tensor:
    raw = normal_f64(seed, name, shape, std=std, mean=mean)
    if dtype == "fp32":
        st = raw.astype(np.float32)
        return Tensor(st.astype(np.float64), st, dtype)
    if dtype == "bf16":
        bits = round_to_bf16_bits(raw)
        return Tensor(bf16_bits_to_f64(bits), bits, dtype)
    raise ValueError(dtype)


# Logical parameter tensors of one layer: name -> (rows, cols) with y = x @ W, W [in, out].
def layer_param_shapes(s: StageShape) -> dict:
    H, d, F = s.hidden, s.head_dim, s.ffn
    nq, nkv = s.n_q_heads, s.n_kv_heads
    shapes = {
        "g1": (H,),
        "Wq": (H, nq * d), "Wk": (H, nkv * d), "Wv": (H, nkv * d),
        "Wo": (nq * d, H),
        "g2": (H,),
    }
    if s.mlp_kind == "swiglu":
        shapes.update({"Wg": (H, F), "Wu": (H, F), "Wd": (F, H)})
    else:
        shapes.update({"W1": (H, F), "Wd": (F, H)})
    if s.norm_kind == "layer":
        shapes.update({"b1": (H,), "b2": (H,)})
    if s.qk_norm:
        shapes.update({"gq": (d,), "gk": (d,)})
    if s.bias:
        shapes.update({"bq": (nq * d,), "bk": (nkv * d,), "bv": (nkv * d,), "bo": (H,), "bd": (H,)})
        shapes.update({"bg": (F,), "bu": (F,)} if s.mlp_kind == "swiglu" else {"bf": (F,)})
    return shapes


def make_layer_params(s: StageShape, layer: int, seed: int = BASE_SEED) -> dict:
    """Logical parameters of one layer.  Weights N(0, w_std); norm gains 1 + N(0, w_std)."""
    out = {}
    for nm, shp in layer_param_shapes(s).items():
        is_gain = nm in ("g1", "g2", "gq", "gk")
        out[nm] = make_tensor(seed, f"{s.name}/L{layer}/{nm}", shp, s.w_std, s.dtype,
                              mean=1.0 if is_gain else 0.0)
    return out


def make_stage_params(s: StageShape, seed: int = BASE_SEED) -> list:
    return [make_layer_params(s, l, seed) for l in range(s.n_layers)]


def make_x(s: StageShape, mb: int, T: int, seed: int = BASE_SEED) -> Tensor:
    return make_tensor(seed, f"{s.name}/x/mb{mb}", (T, s.hidden), s.x_std, s.dtype)


def make_dy(s: StageShape, mb: int, T: int, seed: int = BASE_SEED) -> Tensor:
    return make_tensor(seed, f"{s.name}/dy/mb{mb}", (T, s.hidden), s.dy_std, s.dtype)


def multimodal_lengths(s: StageShape = MULTIMODAL, seed: int = BASE_SEED):
    """Per-microbatch (text_len, image_tokens): text uniform on [512, 2048], image
    tokens uniform on the four-value set.  One packed causal sample per microbatch."""
    M = s.n_microbatches
    lo, hi = MULTIMODAL_TEXT_RANGE
    text = uniform_ints(seed, f"{s.name}/text_len", M, lo, hi)
    pick = uniform_ints(seed, f"{s.name}/image_pick", M, 0, len(MULTIMODAL_IMAGE_TOKENS) - 1)
    img = np.array([MULTIMODAL_IMAGE_TOKENS[int(p)] for p in pick], dtype=np.int64)
    return text, img


def default_cu_seqlens(s: StageShape, mb: int = 0, seed: int = BASE_SEED) -> np.ndarray:
    """cu_seqlens (int32, n_seg+1) of microbatch mb for the named workloads."""
    if s.name.startswith("tiny"):
        return np.array([0, TINY_SEQ], dtype=np.int32)
    if s.name.startswith("language"):
        return np.array([0, LANGUAGE_SEQ], dtype=np.int32)
    if s.name.startswith("wide"):
        return np.array([0, WIDE_SEQ], dtype=np.int32)
    if s.name.startswith("multimodal"):
        text, img = multimodal_lengths(s, seed)
        return np.array([0, int(text[mb] + img[mb])], dtype=np.int32)
    if s.name.startswith("vision"):
        return (np.arange(VISION_IMAGES_PER_MB + 1) * VISION_TOKENS_PER_IMAGE).astype(np.int32)
    raise ValueError(s.name)


def ready_order(M: int, seed: int, name: str = "ready_order") -> list:
    """A seeded random topological order of the tasks {F_j < B_j < W_j : j < M}.

    Returns a list of (kind, j).  At every step one of the currently issuable tasks is
    drawn uniformly, so every legal interleaving has non-zero probability."""
    nxt = [0] * M                      # 0: F pending, 1: B pending, 2: W pending, 3: done
    draws = uniform_ints(seed, name, 3 * M, 0, (1 << 30))
    order = []
    for step in range(3 * M):
        cand = [j for j in range(M) if nxt[j] < 3]
        j = cand[int(draws[step]) % len(cand)]
        order.append(("FBW"[nxt[j]], j))
        nxt[j] += 1
    return order
