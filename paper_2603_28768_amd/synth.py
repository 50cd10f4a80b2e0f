"""Seeded synthetic inputs for one MoE layer under expert-parallel serving.

This module only draws random numbers and rounds them to a storage type.  It
holds none of the method's arithmetic (no routing, no counting, no planning, no
FFN), so both the CPU checker and the HIP path can be fed from it without
sharing any code of the method itself.

The workloads stand in for the paper's profiled expert-load traces (Sec. 3.1:
3000 inference batches of FinePDFs / Lambada / RedPajama requests on
DeepSeek-R1 and Kimi-K2), which are not redistributable here.  What is kept is
their shape: top-8 routing over 128..384 experts, a Zipf-like popularity per
layer whose exponent decides whether the layer is low-skew (peak about 2.5x the
mean) or high-skew (hottest expert more than 10x the mean), and separate
profiling and evaluation batches (Sec. 5.1).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 28768


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    """Shape of one synthetic MoE layer and of the simulated deployment."""

    name: str
    index: int            # added to the base seed so configs draw different numbers
    dtype: str            # "f32" or "bf16": storage type of activations and weights
    T: int                # tokens in one evaluation batch
    H: int                # hidden size
    E: int                # logical experts in the layer
    k: int                # experts activated per token
    I: int                # SwiGLU intermediate size
    D: int                # simulated expert-parallel ranks
    gpus_per_node: int
    replica_slots: int    # replication budget, counted in expert slots over all ranks
    zipf_s: float         # popularity exponent
    hot_experts: int = 0  # this many seeded experts get their popularity multiplied ...
    hot_factor: float = 1.0  # ... by this factor
    profile_batches: int = 8


CONFIGS = {
    "tiny": LayerConfig("tiny", 1, "f32", 256, 128, 16, 2, 256, 4, 2, 4, 1.2),
    "qwen3": LayerConfig("qwen3", 2, "bf16", 4096, 4096, 128, 8, 1536, 8, 8, 8, 1.0),
    "dsv3": LayerConfig("dsv3", 3, "bf16", 8192, 7168, 256, 8, 2048, 32, 8, 32, 1.2),
    "kimi": LayerConfig("kimi", 4, "bf16", 16384, 7168, 384, 8, 2048, 64, 8, 128, 1.4,
                        hot_experts=4, hot_factor=5.0),
    # one layer of the multi-layer stack: DeepSeek-V3 shape at a long prefill batch
    "dsv3_long": LayerConfig("dsv3_long", 5, "bf16", 32768, 7168, 256, 8, 2048, 32, 8, 256, 1.0),
}


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of `cfg` with some fields replaced (used for reduced test sizes)."""
    return dataclasses.replace(cfg, **kw)


def _stream_id(tag: str) -> int:
    v = 0
    for ch in tag.encode():
        v = (v * 131 + ch) % (1 << 31)
    return v


def rng(cfg_index: int, tag: str, *ids: int) -> np.random.Generator:
    """Counter-based generator for the stream named by (config, tag, ids...)."""
    ss = np.random.SeedSequence([BASE_SEED + cfg_index, _stream_id(tag), *[int(i) for i in ids]])
    return np.random.Generator(np.random.Philox(ss))


# ---------------------------------------------------------------- storage types

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))
    return ((bits + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """float32 values that are exactly representable in the storage type."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    if dtype == "f32":
        return a
    raise ValueError(dtype)


# ------------------------------------------------------------------- popularity

def popularity(E: int, zipf_s: float, cfg_index: int, layer: int = 0,
               hot_experts: int = 0, hot_factor: float = 1.0) -> np.ndarray:
    """Zipf popularity over a seeded permutation of the experts, normalised to sum 1."""
    g = rng(cfg_index, "popularity", layer)
    perm = g.permutation(E)                 # perm[r] = expert holding popularity rank r
    pop = np.empty(E, dtype=np.float64)
    pop[perm] = (np.arange(E, dtype=np.float64) + 1.0) ** (-float(zipf_s))
    if hot_experts:
        hot = g.choice(E, size=hot_experts, replace=False)
        pop[hot] *= hot_factor
    return pop / pop.sum()


def layer_popularity(cfg: LayerConfig, layer: int = 0) -> np.ndarray:
    return popularity(cfg.E, cfg.zipf_s, cfg.index, layer, cfg.hot_experts, cfg.hot_factor)


def router_logits(cfg: LayerConfig, pop: np.ndarray, tag: str, batch: int = 0,
                  T: Optional[int] = None, layer: int = 0) -> np.ndarray:
    """fp32 router scores: unit Gaussian noise plus the log-popularity bias."""
    T = cfg.T if T is None else T
    g = rng(cfg.index, "logits/" + tag, layer, batch)
    z = g.standard_normal((T, cfg.E), dtype=np.float32)
    return (z + np.log(pop).astype(np.float32)[None, :]).astype(np.float32)


def gate_weights(cfg: LayerConfig, layer: int = 0) -> np.ndarray:
    """W_router [E][H] of a linear gating network: N(0, 1/sqrt(H)), storage-rounded (scores of
    unit-variance activations then have unit variance, like `router_logits` without its bias)."""
    g = rng(cfg.index, "gate", layer)
    w = g.standard_normal((cfg.E, cfg.H), dtype=np.float32) * np.float32(1.0 / math.sqrt(cfg.H))
    return round_to_storage(w, cfg.dtype)


def activations(cfg: LayerConfig, T: Optional[int] = None, layer: int = 0) -> np.ndarray:
    T = cfg.T if T is None else T
    g = rng(cfg.index, "x", layer)
    return round_to_storage(g.standard_normal((T, cfg.H), dtype=np.float32), cfg.dtype)


def expert_weights(cfg: LayerConfig, expert: int, layer: int = 0
                   ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(W_gate [I][H], W_up [I][H], W_down [H][I]); N(0, 1/sqrt(fan_in)), storage-rounded.

    A function of (config, layer, expert) only, so every copy of a replicated
    expert holds the same numbers whatever rank it is placed on.
    """
    out = []
    for which, (rows, cols) in enumerate(((cfg.I, cfg.H), (cfg.I, cfg.H), (cfg.H, cfg.I))):
        g = rng(cfg.index, "w", layer, expert, which)
        w = g.standard_normal((rows, cols), dtype=np.float32)
        w *= np.float32(1.0 / math.sqrt(cols))
        out.append(round_to_storage(w, cfg.dtype))
    return tuple(out)


# ------------------------------------------------------------- routing traces

def trace_layer_exponents(L: int, cfg_index: int, lo: float = 0.6, hi: float = 1.6) -> np.ndarray:
    """Per-layer Zipf exponents drawn uniformly from [lo, hi]."""
    return rng(cfg_index, "trace_s").uniform(lo, hi, size=L)


def routing_trace_layer(E: int, k: int, T: int, zipf_s: float, cfg_index: int,
                        layer: int) -> np.ndarray:
    """int32 [T][k]: per token, k distinct experts drawn one after another from the
    layer's popularity, a repeat being rejected and drawn again (sampling without
    replacement, proportional to popularity)."""
    pop = popularity(E, zipf_s, cfg_index, layer)
    cdf = np.cumsum(pop)
    cdf[-1] = 1.0
    g = rng(cfg_index, "trace", layer)
    out = np.empty((T, k), dtype=np.int32)
    for j in range(k):
        todo = np.arange(T)
        while todo.size:
            cand = np.searchsorted(cdf, g.random(todo.size), side="right").astype(np.int32)
            np.minimum(cand, E - 1, out=cand)
            clash = np.zeros(todo.size, dtype=bool)
            for jj in range(j):
                clash |= out[todo, jj] == cand
            ok = ~clash
            out[todo[ok], j] = cand[ok]
            todo = todo[clash]
    return out
