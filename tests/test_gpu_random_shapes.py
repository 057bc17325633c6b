"""GPU parity of moe_w4a16_layer on seeded random shapes (the grouped mixed-type GEMM of Section
VII-B around the FP16 x INT4 semantics of Section II-C): token numbers from 1 to 1500, group sizes
32 to 256, 1 to 40 experts, both 16-bit types, skewed routing, expert ids out of range, and shapes
the eight-wave 128-slot tile accepts; whole output, element by element, against the CPU oracle.
The fixed shape lists of the other modules pin the corners; this one walks the space between."""
from __future__ import annotations

import sys

import numpy as np
import pytest
import torch

from moe_workloads import MoEConfig, make_inputs
from oracle import moe_oracle as O

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2504_16214_amd as M
    import gpu_util as U


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def draw_case(rng, case):
    g = int(rng.choice([32, 64, 128, 128, 128, 256]))
    K = g * int(rng.integers(1, max(2, 2048 // g) + 1))
    N = g * int(rng.integers(1, max(2, 1536 // g) + 1))
    if rng.random() < 0.3:      # shapes the eight-wave tile accepts
        g, K, N = 128, 1024 * int(rng.integers(1, 3)), 1024 * int(rng.integers(1, 3))
    E = int(rng.integers(1, 41))
    topk = int(rng.integers(1, min(E, 8) + 1))
    T = int(rng.choice([1, 2, 7, 16, 33, 64, 100, 257, 700, 1500]))
    dt = "f16" if rng.random() < 0.5 else "bf16"
    cfg = MoEConfig(f"random{case}", T=T, K=K, N=N, E=E, topk=topk, group=g, dtype=dt,
                    skew=bool(rng.random() < 0.3), seed=1000 + case)
    return cfg, bool(rng.random() < 0.3)


@pytest.mark.parametrize("stream_seed", [11, 12])
def test_layer_on_random_shapes(stream_seed):
    rng = np.random.default_rng(stream_seed)
    wide = 0
    for case in range(40):
        cfg, spoil = draw_case(rng, case)
        inp = make_inputs(cfg)
        if spoil:                  # a tenth of the expert ids out of range: those slots contribute nothing
            ids = inp.topk_ids.copy()
            m = rng.random(ids.shape) < 0.1
            ids[m] = rng.choice([-1, cfg.E, cfg.E + 5], size=int(m.sum()))
            inp.topk_ids = ids
        say(f"random shape {case}: {cfg} invalid_ids={spoil}")
        got = U.dev_to_f64(U.run_layer(U.DevInputs(inp)))
        wide += M.moe_last_gemm_plan()["waves"] == 8
        want = O.layer(O.decode_bits(inp.x_bits, cfg.dtype), inp.topk_ids, inp.topk_weights, inp.qw1,
                       O.decode_bits(inp.s1_bits, cfg.dtype), inp.z1, inp.qw2,
                       O.decode_bits(inp.s2_bits, cfg.dtype), inp.z2, cfg.group, cfg.dtype)
        U.assert_close(got, want, f"random shape {case} {cfg}")
    say(f"  {wide} of 40 cases ran the eight-wave tile")
    assert wide >= 2
