"""GPU parity of moe_w4a16_layer on seeded random shapes (the grouped mixed-type GEMM of Section
VII-B around the FP16 x INT4 semantics of Section II-C): token numbers from 1 to 1500, group sizes
32 to 256, 1 to 40 experts, both 16-bit types, skewed routing, expert ids out of range, and shapes
the eight-wave 128-slot tile accepts; whole output, element by element, against the CPU oracle.
The fixed shape lists of the other modules pin the corners; this one walks the space between.
fp16 cases meet |gpu - oracle| <= 0.02 + 0.01 |oracle| on every output; bf16 cases get the term
derived in bf16_flip_allowance on top (both sides round the gate/up product and the activation to
8 significant bits, and a differently rounded LARGE activation moves a token's outputs by more
than the plain bound; the three cases that showed it are kept as tests of their own)."""
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


def bf16_flip_allowance(inp, mid):
    """What ONE differently rounded activation may move every output of its token by.

    bf16 keeps 8 significant bits.  The gate/up product H is rounded to bf16 on both sides; the
    float32 and the float64 sum land on different sides of a rounding boundary for about one
    element in a thousand, and such an H moves act = silu(g) * u by up to two bf16 steps.  For a
    large activation that is not small: 2 * 2^-7 * 11 = 0.17 at |act| = 11, times a down-projection
    weight of 0.3 = 0.05 on an output, against 0.02 + 0.01 |out| (fp16 has three more bits, so the
    same event stays eight times smaller).  Both results are correct roundings of the operator, so
    for bf16 the comparison adds, per output, two steps of the activation at the worst of the eight
    largest activations of each of the token's slots, times that weight."""
    c = inp.cfg
    act = mid["act"]                                   # [S, N] values of bf16
    S, N = act.shape
    extra = np.zeros((S, c.K))
    se = inp.topk_ids.reshape(-1)
    s2 = O.decode_bits(inp.s2_bits, c.dtype)
    for e in np.unique(se[(se >= 0) & (se < c.E)]):
        W = np.abs(O.dequant(inp.qw2[e], s2[e], inp.z2[e], c.group))        # [K, N]
        for s in np.nonzero(se == e)[0]:
            top = np.argsort(np.abs(act[s]))[-8:]
            a = np.abs(act[s, top])
            step = np.where(a > 0, 2.0 ** (np.floor(np.log2(np.maximum(a, 1e-300))) - 7), 0.0)
            extra[s] = (W[:, top] * (2.0 * step)[None, :]).max(axis=1)
    w = inp.topk_weights.astype(np.float64).reshape(-1)
    return (extra * w[:, None]).reshape(c.T, c.topk, c.K).sum(axis=1)


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


def check_case(inp, what):
    cfg = inp.cfg
    got = U.dev_to_f64(U.run_layer(U.DevInputs(inp)))
    want, mid = O.layer(O.decode_bits(inp.x_bits, cfg.dtype), inp.topk_ids, inp.topk_weights, inp.qw1,
                        O.decode_bits(inp.s1_bits, cfg.dtype), inp.z1, inp.qw2,
                        O.decode_bits(inp.s2_bits, cfg.dtype), inp.z2, cfg.group, cfg.dtype,
                        return_intermediates=True)
    if cfg.dtype == "f16":
        U.assert_close(got, want, what)
        return 0
    assert np.all(np.isfinite(got))
    err = np.abs(got - want)
    plain = U.ATOL + U.RTOL * np.abs(want)
    bad = err > plain + bf16_flip_allowance(inp, mid)
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} outside the bf16 bound"
    return int((err > plain).sum())


# Three bf16 shapes on which a differently rounded large activation moves a dozen outputs of one
# token past 0.02 + 0.01 |out| (found by longer runs of the walk below).
FLIP_CASES = [
    MoEConfig("flip_a", T=700, K=2048, N=2048, E=1, topk=1, group=128, dtype="bf16", seed=1081),
    MoEConfig("flip_b", T=1500, K=1920, N=384, E=35, topk=1, group=128, dtype="bf16", skew=True, seed=1015),
    MoEConfig("flip_c", T=100, K=2048, N=1536, E=22, topk=4, group=256, dtype="bf16", skew=True, seed=1146),
]


@pytest.mark.parametrize("cfg", FLIP_CASES, ids=lambda c: c.name)
def test_bf16_outputs_moved_by_one_rounding_of_a_large_activation(cfg):
    say(f"bf16 rounding-flip case {cfg}")
    inp = make_inputs(cfg)
    beyond_plain = check_case(inp, cfg.name)
    say(f"  outputs beyond the plain bound: {beyond_plain} of {cfg.T * cfg.K}")
    assert beyond_plain <= 1e-4 * cfg.T * cfg.K


@pytest.mark.parametrize("stream_seed,n_cases", [(11, 40), (12, 40)])
def test_layer_on_random_shapes(stream_seed, n_cases):
    rng = np.random.default_rng(stream_seed)
    wide = 0
    for case in range(n_cases):
        cfg, spoil = draw_case(rng, case)
        inp = make_inputs(cfg)
        if spoil:                  # a tenth of the expert ids out of range: those slots contribute nothing
            ids = inp.topk_ids.copy()
            m = rng.random(ids.shape) < 0.1
            ids[m] = rng.choice([-1, cfg.E, cfg.E + 5], size=int(m.sum()))
            inp.topk_ids = ids
        say(f"random shape {case}: {cfg} invalid_ids={spoil}")
        check_case(inp, f"random shape {case} {cfg}")
        wide += M.moe_last_gemm_plan()["waves"] == 8
    say(f"  {wide} of {n_cases} cases ran the eight-wave tile")
    assert wide >= 2
