"""Seeded synthetic W4A16 mixture-of-experts workloads.

This module only draws inputs.  It serves the CPU oracle and the HIP path alike
and contains none of the layer's arithmetic: no nibble unpack, no
dequantisation, no GEMM, no activation, no combine, no bucketing.  The packed
weight words are drawn directly as uniform 32-bit integers (eight independent
uniform nibbles each), so nothing here even needs a packing routine.

What it does hold is input preparation that happens before the layer's
boundary: casting the drawn activations / scales to the 16-bit storage format
and turning router logits into (expert id, weight) pairs per token.  Both
consumers receive exactly the same arrays.

The synthetic recipe stands in for the 256-expert FP16xINT4 layer of the
paper's mixed-type MoE evaluation (Section VII-B, "Mixed-type MoE"), whose
real checkpoint weights are not available.

All 16-bit floating tensors travel as raw uint16 bit patterns so that fp16 and
bf16 are handled the same way by every consumer.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

__all__ = ["MoEConfig", "MoEInputs", "CONFIGS", "make_inputs", "route_topk",
           "to_bits", "skew_bias"]


@dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int          # tokens
    K: int          # hidden size
    N: int          # expert intermediate size
    E: int          # experts
    topk: int
    group: int      # quantisation group length along the reduction dim
    dtype: str      # "f16" | "bf16"
    skew: bool = False
    seed: int = 0

    @property
    def S(self) -> int:
        return self.T * self.topk


# The five seeded configurations of the benchmark statement.
CONFIGS: Dict[str, MoEConfig] = {
    "tiny": MoEConfig("tiny", T=16, K=256, N=512, E=8, topk=2, group=128, dtype="f16"),
    "mixtral_decode": MoEConfig("mixtral_decode", T=64, K=4096, N=14336, E=8, topk=2,
                                group=128, dtype="f16"),
    "deepseek_decode": MoEConfig("deepseek_decode", T=128, K=7168, N=2048, E=256, topk=8,
                                 group=128, dtype="f16"),
    "deepseek_prefill": MoEConfig("deepseek_prefill", T=4096, K=7168, N=2048, E=256, topk=8,
                                  group=128, dtype="f16"),
    "skewed_bf16": MoEConfig("skewed_bf16", T=1024, K=2048, N=1408, E=64, topk=6,
                             group=64, dtype="bf16", skew=True),
}
CONFIG_ORDER = ["tiny", "mixtral_decode", "deepseek_decode", "deepseek_prefill", "skewed_bf16"]


@dataclass
class MoEInputs:
    cfg: MoEConfig
    x_bits: np.ndarray        # [T, K] uint16 bit patterns of dtype
    logits: np.ndarray        # [T, E] float32
    topk_ids: np.ndarray      # [T, topk] int32
    topk_weights: np.ndarray  # [T, topk] float32
    qw1: np.ndarray           # [E, 2N, K/8] int32, 8 nibbles per word
    s1_bits: np.ndarray       # [E, 2N, K/group] uint16
    z1: np.ndarray            # [E, 2N, K/group] uint8 in 0..15
    qw2: np.ndarray           # [E, K, N/8] int32
    s2_bits: np.ndarray       # [E, K, N/group] uint16
    z2: np.ndarray            # [E, K, N/group] uint8
    extra: dict = field(default_factory=dict)


def to_bits(values: np.ndarray, dtype: str) -> np.ndarray:
    """Cast float32 values to the 16-bit storage format (round to nearest even)
    and return the raw bit patterns as uint16."""
    v = np.ascontiguousarray(values, dtype=np.float32)
    if dtype == "f16":
        return v.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        b = v.view(np.uint32)
        lsb = (b >> np.uint32(16)) & np.uint32(1)
        r = (b + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
        return r.astype(np.uint16)
    raise ValueError(f"unknown dtype {dtype!r}")


def skew_bias(E: int) -> np.ndarray:
    """Per-expert logit bias 2*ln(1/rank^1.2) with rank = e + 1 (expert 0 hottest)."""
    rank = np.arange(1, E + 1, dtype=np.float64)
    return (-2.4 * np.log(rank)).astype(np.float32)


def route_topk(logits: np.ndarray, topk: int):
    """Router used to prepare the layer's inputs.

    Picks the top-k logits per token (descending, ties to the lower expert
    index) and returns the softmax over the selected logits, i.e. the full
    softmax renormalised over the chosen experts.  ids int32, weights float32.
    """
    logits = np.asarray(logits, dtype=np.float32)
    order = np.argsort(-logits, axis=1, kind="stable")[:, :topk]
    sel = np.take_along_axis(logits, order, axis=1).astype(np.float64)
    sel = sel - sel.max(axis=1, keepdims=True)
    p = np.exp(sel)
    p /= p.sum(axis=1, keepdims=True)
    return order.astype(np.int32), p.astype(np.float32)


def _draw_weight(rng: np.random.Generator, E: int, rows: int, red: int, group: int, dtype: str):
    """One quantised weight tensor [E, rows, red]: packed words, scales, zero points."""
    qw = np.empty((E, rows, red // 8), dtype=np.int32)
    for e in range(E):  # per expert to bound temporaries
        qw[e] = rng.integers(0, 2 ** 32, size=(rows, red // 8), dtype=np.uint32).view(np.int32)
    s = rng.uniform(0.002, 0.02, size=(E, rows, red // group)).astype(np.float32)
    z = rng.integers(0, 16, size=(E, rows, red // group), dtype=np.uint8)
    return qw, to_bits(s, dtype), z


def make_inputs(cfg: MoEConfig, logits_override: Optional[np.ndarray] = None) -> MoEInputs:
    """Draw one workload.  Draw order is fixed: X, logits, W1 (words, scales,
    zeros), W2 (words, scales, zeros), all from numpy's PCG64 seeded with cfg.seed."""
    assert cfg.K % cfg.group == 0 and cfg.N % cfg.group == 0 and cfg.group % 8 == 0
    rng = np.random.default_rng(cfg.seed)
    x = (0.5 * rng.standard_normal((cfg.T, cfg.K))).astype(np.float32)
    logits = rng.standard_normal((cfg.T, cfg.E)).astype(np.float32)
    if cfg.skew:
        logits = (logits + skew_bias(cfg.E)[None, :]).astype(np.float32)
    if logits_override is not None:
        logits = np.asarray(logits_override, dtype=np.float32)
    ids, w = route_topk(logits, cfg.topk)
    qw1, s1, z1 = _draw_weight(rng, cfg.E, 2 * cfg.N, cfg.K, cfg.group, cfg.dtype)
    qw2, s2, z2 = _draw_weight(rng, cfg.E, cfg.K, cfg.N, cfg.group, cfg.dtype)
    return MoEInputs(cfg, to_bits(x, cfg.dtype), logits, ids, w, qw1, s1, z1, qw2, s2, z2)
