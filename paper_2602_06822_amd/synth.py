"""Seeded synthetic inputs for the POP pruned-FFN path.

This module is shared by the CPU oracle's tests and by the HIP path's tests and
benchmark.  It holds none of the method's arithmetic: it only draws random
tensors with the shapes, dtypes and value distributions of the workloads and
casts them to their storage dtype.  Everything is generated on the host with a
counter-based generator (Philox), keyed by (base seed, config, layer/expert,
tensor name), so any tensor can be regenerated independently of the others.

Workload recipe (stand-in for the trained Llama / Mixtral checkpoints and the
benchmark prompts the paper evaluates on, none of which are available here):

* weights  W_gate[m][d], W_up[m][d], W_down[d][m]  ~ N(0, 0.02^2)
* activations  X[T][d] ~ N(0, 1); a few fixed hidden "outlier" channels are
  scaled by 20.  For the bf16 Llama/Mixtral-shaped layers the outlier channels
  (round(0.001*d) of them) are heavy tailed: Student-t(nu=4) * 20.
* decode vectors follow the same law and reuse the same outlier channels.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20260206

F32 = 0
BF16 = 1


def _key(*parts) -> int:
    h = hashlib.sha256(("|".join(str(p) for p in parts)).encode()).digest()
    return int.from_bytes(h[:8], "little")


def rng(*parts) -> np.random.Generator:
    """Counter-based generator keyed by BASE_SEED and the given name parts."""
    return np.random.Generator(np.random.Philox(key=_key(BASE_SEED, *parts)))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even cast of finite float32 values to bf16 bit patterns (uint16)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a: np.ndarray, dtype: int) -> np.ndarray:
    """float32 array -> storage array: float32 (F32) or uint16 bf16 bits (BF16)."""
    if dtype == F32:
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == BF16:
        return f32_to_bf16_bits(a)
    raise ValueError(f"unknown dtype code {dtype}")


def storage_to_f64(a: np.ndarray, dtype: int) -> np.ndarray:
    """Exact widening of a storage array to float64."""
    if dtype == F32:
        return a.astype(np.float64)
    return bf16_bits_to_f32(a).astype(np.float64)


@dataclass
class LayerConfig:
    name: str
    d: int
    m: int
    dtype: int
    n_outlier: int
    heavy_tail: bool
    w_std: float = 0.02
    outlier_scale: float = 20.0


@dataclass
class Layer:
    cfg: LayerConfig
    w_gate: np.ndarray  # [m][d] storage
    w_up: np.ndarray    # [m][d] storage
    w_down: np.ndarray  # [d][m] storage
    outlier_channels: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))


# The five benchmark workloads' layer shapes.
CFG1 = LayerConfig("cfg1_small_fp32", d=512, m=1376, dtype=F32, n_outlier=4, heavy_tail=False)
CFG2 = LayerConfig("cfg2_llama2_7b", d=4096, m=11008, dtype=BF16, n_outlier=4, heavy_tail=True)
CFG3 = LayerConfig("cfg3_llama2_7b_stack", d=4096, m=11008, dtype=BF16, n_outlier=4, heavy_tail=True)
CFG4 = LayerConfig("cfg4_llama2_13b_stack", d=5120, m=13824, dtype=BF16, n_outlier=5, heavy_tail=True)
CFG5 = LayerConfig("cfg5_mixtral_expert", d=4096, m=14336, dtype=BF16, n_outlier=4, heavy_tail=True)


def small_config(name: str, d: int, m: int, dtype: int, n_outlier: int = 2,
                 heavy_tail: bool = False) -> LayerConfig:
    return LayerConfig(name, d=d, m=m, dtype=dtype, n_outlier=n_outlier, heavy_tail=heavy_tail)


def make_layer(cfg: LayerConfig, layer_id: int = 0) -> Layer:
    def w(name, shape):
        g = rng(cfg.name, layer_id, name)
        a = g.standard_normal(shape, dtype=np.float32)
        a *= np.float32(cfg.w_std)
        return to_storage(a, cfg.dtype)

    outl = np.sort(rng(cfg.name, layer_id, "outlier_channels").choice(cfg.d, size=cfg.n_outlier,
                                                                        replace=False))
    return Layer(cfg, w("w_gate", (cfg.m, cfg.d)), w("w_up", (cfg.m, cfg.d)),
                 w("w_down", (cfg.d, cfg.m)), outl)


def make_layers(cfg: LayerConfig, layer_ids, workers: int = 8):
    """Several layers of one shape, drawn in parallel threads (each tensor has its own counter-based stream, so
    the result does not depend on the order or the number of workers)."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=max(1, workers)) as ex:
        return list(ex.map(lambda i: make_layer(cfg, i), layer_ids))


def make_activations(layer: Layer, T: int, tag: str, layer_id: int = 0) -> np.ndarray:
    """X[T][d] in the layer's storage dtype; `tag` names the tensor ("prompt", "decode", ...)."""
    cfg = layer.cfg
    g = rng(cfg.name, layer_id, tag, T)
    x = g.standard_normal((T, cfg.d), dtype=np.float32)
    if len(layer.outlier_channels):
        if cfg.heavy_tail:
            t = g.standard_t(4.0, size=(T, len(layer.outlier_channels))).astype(np.float32)
            x[:, layer.outlier_channels] = t * np.float32(cfg.outlier_scale)
        else:
            x[:, layer.outlier_channels] *= np.float32(cfg.outlier_scale)
    return to_storage(x, cfg.dtype)


def make_router_logits(cfg: LayerConfig, T: int, n_experts: int, tag: str) -> np.ndarray:
    """Router logits [T][n_experts] ~ N(0,1), float32 (MoE workload)."""
    return rng(cfg.name, "router", tag, T).standard_normal((T, n_experts), dtype=np.float32)


def make_scores(n: int, tag: str, ties: str = "none") -> np.ndarray:
    """Non-negative float32 score vectors for the selection tests.

    ties = "none": distinct values; "some": values drawn from a small set so many
    are equal; "all": one repeated value; "zeros": mix of +0.0, -0.0 and a few values.
    """
    g = rng("scores", tag, n, ties)
    if ties == "none":
        s = np.abs(g.standard_normal(n, dtype=np.float32)) + np.float32(1e-3)
        # make the values distinct without changing their law materially
        s = np.unique(s)
        while len(s) < n:
            extra = np.abs(g.standard_normal(n - len(s), dtype=np.float32)) + np.float32(1e-3)
            s = np.unique(np.concatenate([s, extra]))
        s = s[:n]
        g.shuffle(s)
        return s.astype(np.float32)
    if ties == "some":
        vals = np.abs(g.standard_normal(max(2, n // 8), dtype=np.float32))
        return vals[g.integers(0, len(vals), size=n)].astype(np.float32)
    if ties == "all":
        return np.full(n, np.float32(0.75), dtype=np.float32)
    if ties == "zeros":
        s = np.zeros(n, dtype=np.float32)
        neg = g.random(n) < 0.3
        s[neg] = np.float32(-0.0)
        some = g.random(n) < 0.2
        s[some] = np.abs(g.standard_normal(int(some.sum()), dtype=np.float32))
        return s
    raise ValueError(ties)


SCORE_SHAPES = ("low_byte", "two_bytes", "crowded", "three_values", "narrow_band", "wide_signed")


def make_scores_shaped(n: int, tag: str, shape: str) -> np.ndarray:
    """float32 score vectors whose bit patterns are laid out to reach the corners of a digit-wise rank selection.

    "low_byte": values that differ in their lowest 8 bits only (many ties); "two_bytes": in their lowest 16 bits;
    "crowded": 70 % one value, the rest log-normal (one digit bucket holds most keys); "three_values": three distinct
    values; "narrow_band": uniform in [1, 1 + 2^-10) (the ranks of interest share their leading digits);
    "wide_signed": heavy-tailed with both signs over many binades.
    """
    g = rng("scores_shaped", tag, n, shape)
    one = np.float32(1.0).view(np.uint32)
    if shape == "low_byte":
        return (one + g.integers(0, 200, size=n).astype(np.uint32)).view(np.float32)
    if shape == "two_bytes":
        return (one + g.integers(0, 60000, size=n).astype(np.uint32)).view(np.float32)
    if shape == "crowded":
        s = np.exp(g.standard_normal(n)).astype(np.float32)
        s[g.random(n) < 0.7] = np.float32(3.0)
        return s
    if shape == "three_values":
        return np.array([0.5, 1.0, 2.0], dtype=np.float32)[g.integers(0, 3, size=n)]
    if shape == "narrow_band":
        return (np.float32(1.0) + g.random(n, dtype=np.float32) * np.float32(2.0 ** -10)).astype(np.float32)
    if shape == "wide_signed":
        return (np.exp(6.0 * g.standard_normal(n)) * np.where(g.random(n) < 0.3, -1.0, 1.0)).astype(np.float32)
    raise ValueError(shape)
