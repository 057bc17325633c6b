"""Seeded synthetic inputs for the blockwise-scaled FP8 GEMM.

Input preparation only: Gaussian activations and weights are drawn, scaled per 1 x 128 tile
(activations) / 128 x 128 block (weights) so that the largest magnitude of a tile maps to 448, and
cast to 8-bit e4m3 codes with a library cast (PyTorch's float8_e4m3fn).  None of the GEMM's
arithmetic lives here: no decode, no product, no accumulation.  The oracle and the HIP path read
the same code bytes and float32 scales.

The shapes stand in for the linear layers of the FP8 serving workload the paper evaluates
(Section VII-D; per-layer results in the appendix figure on blockwise scaled FP8 GEMM layers):
fused QKV, attention output, fused gate/up and down projections of a 32-billion-parameter dense
transformer (hidden 5120, intermediate 25600, 64 + 8 heads of 128), at decode and prefill row counts.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict

import numpy as np
import torch

BLOCK = 128


@dataclass(frozen=True)
class Fp8GemmConfig:
    name: str
    M: int
    N: int
    K: int
    seed: int = 0


@dataclass
class Fp8GemmInputs:
    cfg: Fp8GemmConfig
    a_codes: np.ndarray      # [M, K] uint8
    a_scale: np.ndarray      # [M, K/128] float32
    b_codes: np.ndarray      # [N, K] uint8
    b_scale: np.ndarray      # [ceil(N/128), K/128] float32


FP8_CONFIGS: Dict[str, Fp8GemmConfig] = {c.name: c for c in [
    Fp8GemmConfig("fp8_tiny", M=37, N=192, K=384),
    Fp8GemmConfig("fp8_qkv_decode", M=64, N=10240, K=5120),
    Fp8GemmConfig("fp8_down_decode", M=16, N=5120, K=25600),
    Fp8GemmConfig("fp8_gateup_decode", M=32, N=51200, K=5120),
    Fp8GemmConfig("fp8_gateup_prefill", M=4096, N=51200, K=5120),
    Fp8GemmConfig("fp8_qkv_prefill", M=4096, N=10240, K=5120),
    Fp8GemmConfig("fp8_down_prefill", M=4096, N=5120, K=25600),
]}


def _cast_e4m3(x: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).clamp_(-448.0, 448.0)
    return t.to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def make_fp8_inputs(cfg: Fp8GemmConfig) -> Fp8GemmInputs:
    assert cfg.K % BLOCK == 0
    rng = np.random.default_rng(cfg.seed)
    M, N, K = cfg.M, cfg.N, cfg.K
    KB, NB = K // BLOCK, -(-N // BLOCK)
    x = rng.standard_normal((M, K), dtype=np.float32)
    amax = np.abs(x.reshape(M, KB, BLOCK)).max(axis=2)
    a_scale = (np.maximum(amax, 1e-12) / np.float32(448.0)).astype(np.float32)
    a_codes = _cast_e4m3(x / np.repeat(a_scale, BLOCK, axis=1))
    w = (np.float32(0.02) * rng.standard_normal((N, K), dtype=np.float32))
    wp = np.zeros((NB * BLOCK, K), dtype=np.float32)
    wp[:N] = w
    bmax = np.abs(wp.reshape(NB, BLOCK, KB, BLOCK)).max(axis=(1, 3))
    b_scale = (np.maximum(bmax, 1e-12) / np.float32(448.0)).astype(np.float32)
    b_codes = _cast_e4m3(w / np.repeat(np.repeat(b_scale, BLOCK, axis=0)[:N], BLOCK, axis=1))
    return Fp8GemmInputs(cfg, a_codes, a_scale, b_codes, b_scale)


# --------------------------------------------------------------------------
# FP8 mixture-of-experts layer workloads
# --------------------------------------------------------------------------
# Activations, routing and sizes as in the 16-bit MoE workloads (moe_workloads.make_inputs);
# expert weights are e4m3 codes with one float32 scale per 128 x 128 block.  Drawing Gaussian
# weights and casting them would need tens of GB of float32 temporaries at 256 experts, so the
# codes are drawn directly: a byte u uniform in 0..255 is mapped through a 256-entry table to the
# e4m3 code of the ((u + 0.5) / 256)-quantile of a Gaussian whose 4.5-sigma point sits at 448 (what
# scaling a 128 x 128 Gaussian block by its maximum gives, to within the block-to-block spread);
# block scales are uniform in [0.5, 1.5] * sigma_w * 4.5 / 448 with sigma_w = 0.02.  The table is
# built with a library cast: input preparation, none of the layer's arithmetic.
@dataclass(frozen=True)
class Fp8MoEConfig:
    name: str
    T: int
    K: int
    N: int
    E: int
    topk: int
    dtype: str = "bf16"
    seed: int = 0

    @property
    def S(self) -> int:
        return self.T * self.topk


@dataclass
class Fp8MoEInputs:
    cfg: Fp8MoEConfig
    x_bits: np.ndarray        # [T, K] uint16 patterns of cfg.dtype
    topk_ids: np.ndarray      # [T, topk] int32
    topk_weights: np.ndarray  # [T, topk] float32
    w1_codes: np.ndarray      # [E, 2N, K] uint8
    w1_scale: np.ndarray      # [E, 2N/128, K/128] float32
    w2_codes: np.ndarray      # [E, K, N] uint8
    w2_scale: np.ndarray      # [E, K/128, N/128] float32


FP8_MOE_CONFIGS: Dict[str, Fp8MoEConfig] = {c.name: c for c in [
    Fp8MoEConfig("fp8_moe_tiny", T=16, K=256, N=256, E=8, topk=2),
    Fp8MoEConfig("fp8_moe_decode", T=128, K=7168, N=2048, E=256, topk=8),
    Fp8MoEConfig("fp8_moe_prefill", T=4096, K=7168, N=2048, E=256, topk=8),
]}

SIGMA_W = 0.02


def _gaussian_code_table() -> np.ndarray:
    from scipy.special import ndtri
    z = ndtri((np.arange(256) + 0.5) / 256.0)
    return _cast_e4m3((z / 4.5 * 448.0).astype(np.float32))


def _draw_fp8_weight(rng: np.random.Generator, table: np.ndarray, E: int, rows: int, red: int, seed_key=None):
    """Codes: one generator per expert when seed_key is given (seed sequence seed_key + [e]), so the
    experts can be drawn by several threads with the same result for any thread count; otherwise
    from rng, expert after expert.  Scales: from rng."""
    codes = np.empty((E, rows, red), dtype=np.uint8)

    def draw(e, g):
        u = g.integers(0, 256, size=(rows, red), dtype=np.uint8)
        np.take(table, u, out=codes[e], mode="wrap")       # (wrap: no bounds pass; the indices are bytes)

    if seed_key is None:
        for e in range(E):      # per expert to bound temporaries
            draw(e, rng)
    else:
        import os
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=max(1, min(16, os.cpu_count() or 1))) as pool:
            list(pool.map(lambda e: draw(e, np.random.default_rng(list(seed_key) + [e])), range(E)))
    scale = (rng.uniform(0.5, 1.5, size=(E, -(-rows // BLOCK), red // BLOCK)) * (SIGMA_W * 4.5 / 448.0))
    return codes, scale.astype(np.float32)


_WEIGHT_CACHE: dict = {}      # the last weight set drawn, keyed by (E, K, N, seed)


def _fp8_moe_weights(cfg: Fp8MoEConfig):
    """The layer's weights come from generators of their own, so configurations that differ only in
    the token number share them: the codes of expert e of W1 / W2 from the seed sequence
    [cfg.seed, 1, 1 or 2, e], the block scales (W1 then W2) from [cfg.seed, 1].  The last set is
    kept and handed out again (11 GB at 256 experts): callers must not write into the arrays."""
    key = (cfg.E, cfg.K, cfg.N, cfg.seed)
    if key not in _WEIGHT_CACHE:
        _WEIGHT_CACHE.clear()
        rng = np.random.default_rng([cfg.seed, 1])
        table = _gaussian_code_table()
        w1c, w1s = _draw_fp8_weight(rng, table, cfg.E, 2 * cfg.N, cfg.K, seed_key=(cfg.seed, 1, 1))
        w2c, w2s = _draw_fp8_weight(rng, table, cfg.E, cfg.K, cfg.N, seed_key=(cfg.seed, 1, 2))
        _WEIGHT_CACHE[key] = (w1c, w1s, w2c, w2s)
    return _WEIGHT_CACHE[key]


def make_fp8_moe_inputs(cfg: Fp8MoEConfig) -> Fp8MoEInputs:
    """Activations and routing: numpy PCG64 seeded with the sequence [cfg.seed, 0], draw order X,
    logits.  Weights: _fp8_moe_weights."""
    from . import route_topk, to_bits
    assert cfg.K % BLOCK == 0 and cfg.N % BLOCK == 0
    rng = np.random.default_rng([cfg.seed, 0])
    x = (0.5 * rng.standard_normal((cfg.T, cfg.K))).astype(np.float32)
    logits = rng.standard_normal((cfg.T, cfg.E)).astype(np.float32)
    ids, w = route_topk(logits, cfg.topk)
    w1c, w1s, w2c, w2s = _fp8_moe_weights(cfg)
    return Fp8MoEInputs(cfg, to_bits(x, cfg.dtype), ids, w, w1c, w1s, w2c, w2s)
