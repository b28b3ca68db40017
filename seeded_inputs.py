"""Seeded synthetic inputs for the split-backward stage (shared by the CPU oracle's tests and the HIP path's tests).

This module holds no arithmetic of the method itself: it only names the workload shapes and draws
random tensors.  Every tensor is a pure function of (seed, tensor name, element index), so any
slice of any tensor can be regenerated anywhere, in any order, without state.

Generator: a 64-bit counter hash (splitmix64 finaliser) gives two uniforms per element, which a
Box-Muller transform turns into one standard normal in fp64.  Storage rounding (fp32 or bf16,
round-to-nearest-even) is applied exactly once, here, so that both consumers see identical values.

Workload recipe (the paper trains on randomly generated data, Section 3.2): weights ~ N(0, 0.02),
RMSNorm gains ~ 1 + N(0, 0.02), stage input x ~ N(0, 1), upstream gradient dY ~ N(0, 1).
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLDEN = 0x9E3779B97F4A7C15


@dataclasses.dataclass(frozen=True)
class StageShape:
    """Shape of one pipeline stage.  n_heads == 0 means MLP-only blocks (no attention half)."""
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    seq: int
    micro_batch: int
    n_microbatches: int
    dtype: str            # "f32" or "bf16": storage type of weights / activations / stashes
    seed: int
    rms_eps: float = 1e-6
    rope_base: float = 10000.0
    causal: bool = True

    @property
    def tokens(self) -> int:
        return self.seq * self.micro_batch

    def replace(self, **kw) -> "StageShape":
        return dataclasses.replace(self, **kw)


# The five workloads of the benchmark definition; the seed is 20240518 + index.
CONFIGS = {
    "tiny_f32": StageShape("tiny_f32", 1, 256, 4, 64, 688, 128, 2, 4, "f32", 20240519),
    "mlp_bf16": StageShape("mlp_bf16", 4, 2048, 0, 0, 5504, 2048, 1, 8, "bf16", 20240520),
    "llama7b_s1024": StageShape("llama7b_s1024", 8, 4096, 32, 128, 11008, 1024, 1, 4, "bf16", 20240521),
    "llama7b_s2048": StageShape("llama7b_s2048", 8, 4096, 32, 128, 11008, 2048, 2, 8, "bf16", 20240522),
    "llama13b_s2048": StageShape("llama13b_s2048", 10, 5120, 40, 128, 13824, 2048, 1, 16, "bf16", 20240523),
}


def _fnv1a64(text: str) -> int:
    h = 0xCBF29CE484222325
    for ch in text.encode("utf-8"):
        h ^= ch
        h = (h * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return h


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on a uint64 array (wrap-around arithmetic)."""
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def _normal_chunk(key: int, start: int, count: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        idx = np.arange(start, start + count, dtype=np.uint64)
        base = np.uint64(key) + (idx * np.uint64(2)) * np.uint64(_GOLDEN)
        h1 = _mix64(base)
        h2 = _mix64(base + np.uint64(_GOLDEN))
    # 53-bit uniforms in (0, 1): never exactly 0, so the log is finite
    u1 = ((h1 >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)
    u2 = ((h2 >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * np.pi) * u2)


def standard_normal(seed: int, name: str, shape, *, threads: int = 8) -> np.ndarray:
    """fp64 N(0,1) tensor, a pure function of (seed, name, flat element index)."""
    n = int(np.prod(shape, dtype=np.int64)) if len(tuple(shape)) else 1
    key = (_fnv1a64(name) ^ ((seed * _GOLDEN) & 0xFFFFFFFFFFFFFFFF)) & 0xFFFFFFFFFFFFFFFF
    key = int(_mix64(np.array([key], dtype=np.uint64))[0])
    chunk = 1 << 22
    if n <= chunk:
        return _normal_chunk(key, 0, n).reshape(shape)
    out = np.empty(n, dtype=np.float64)

    def work(s):
        c = min(chunk, n - s)
        out[s:s + c] = _normal_chunk(key, s, c)

    with ThreadPoolExecutor(max_workers=threads) as pool:
        list(pool.map(work, range(0, n, chunk)))
    return out.reshape(shape)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even); returns float32 holding bf16-representable values."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(f.shape)


def bf16_bits(x_rounded: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of an array that already holds bf16-representable float32 values."""
    u = np.ascontiguousarray(x_rounded, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_from_bits(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def store_round(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values once to the storage type; result is float32 (exactly representable in dtype)."""
    if dtype == "bf16":
        return round_bf16(x)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(f"unknown dtype {dtype!r}")


def stage_params(shape: StageShape) -> dict:
    """Per-layer parameter lists, rounded to the storage dtype, as float32 arrays.

    Layout: every weight is [in, out] row-major so that Y = X @ W.  q/k/v are fused as [d, 3d]
    (column blocks q, k, v), gate/up as [d, 2f] (column blocks gate, up).
    """
    d, f, s = shape.d_model, shape.d_ffn, shape.seed
    attn = shape.n_heads > 0
    p = {k: [] for k in ("w_qkv", "w_o", "g1", "w_gu", "w_d", "g2")}
    for l in range(shape.n_layers):
        if attn:
            p["w_qkv"].append(store_round(0.02 * standard_normal(s, f"L{l}.w_qkv", (d, 3 * d)), shape.dtype))
            p["w_o"].append(store_round(0.02 * standard_normal(s, f"L{l}.w_o", (d, d)), shape.dtype))
            p["g1"].append(store_round(1.0 + 0.02 * standard_normal(s, f"L{l}.g1", (d,)), shape.dtype))
        p["w_gu"].append(store_round(0.02 * standard_normal(s, f"L{l}.w_gu", (d, 2 * f)), shape.dtype))
        p["w_d"].append(store_round(0.02 * standard_normal(s, f"L{l}.w_d", (f, d)), shape.dtype))
        p["g2"].append(store_round(1.0 + 0.02 * standard_normal(s, f"L{l}.g2", (d,)), shape.dtype))
    return p


def stage_input(shape: StageShape, mb: int) -> np.ndarray:
    """Stage input activations of micro-batch mb: [tokens, d_model], token-major (sequence b = rows b*seq..)."""
    return store_round(standard_normal(shape.seed, f"x.mb{mb}", (shape.tokens, shape.d_model)), shape.dtype)


def stage_upstream_grad(shape: StageShape, mb: int) -> np.ndarray:
    """Gradient of the loss w.r.t. the stage output for micro-batch mb: [tokens, d_model]."""
    return store_round(standard_normal(shape.seed, f"dy.mb{mb}", (shape.tokens, shape.d_model)), shape.dtype)
