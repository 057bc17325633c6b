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
