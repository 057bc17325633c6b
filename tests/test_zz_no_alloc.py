"""The layer entry point that allocates nothing (moe_w4a16_layer_noalloc: built-in scratch array
instead of a caller workspace) against moe_w4a16_layer, through the C ABI: two calls in a row on
the same GPU, the second with a smaller input, so that the second call runs on whatever the
first one left in the shared array."""
from __future__ import annotations

import sys

import numpy as np
import pytest
import torch

from moe_workloads import CONFIGS, MoEConfig, make_inputs
from oracle import moe_oracle as O

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2504_16214_amd as M
    import gpu_util as U


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def run_noalloc(d):
    c = d.cfg
    out = torch.full((c.T, c.K), float("nan"), dtype=U.TORCH_DT[c.dtype], device="cuda")
    M.moe_w4a16_layer_noalloc(d.X, d.ids, d.w, d.qw1, d.s1, d.z1, d.qw2, d.s2, d.z2, out, c.group)
    torch.cuda.synchronize()
    return out


def test_noalloc_layer_matches_workspace_layer_twice():
    big = MoEConfig("noalloc_big", T=96, K=1024, N=2048, E=12, topk=4, group=128, dtype="f16", seed=41)
    small = MoEConfig("noalloc_small", T=7, K=512, N=384, E=5, topk=2, group=128, dtype="bf16", seed=42)
    for cfg in (big, small):
        say(f"noalloc layer {cfg}")
        inp = make_inputs(cfg)
        if cfg is small:
            inp.topk_ids[3, 1] = cfg.E + 2          # an ignored slot: its rows of the shared array stay stale
        d = U.DevInputs(inp)
        want = U.dev_to_f64(U.run_layer(d))
        got = U.dev_to_f64(run_noalloc(d))
        U.assert_close(got, want, f"{cfg.name}: noalloc vs workspace entry point")
        assert np.array_equal(got, want), "same kernels, same plan: expected identical bits"
        c = inp.cfg
        ref = O.layer(O.decode_bits(inp.x_bits, c.dtype), inp.topk_ids, inp.topk_weights, inp.qw1,
                      O.decode_bits(inp.s1_bits, c.dtype), inp.z1, inp.qw2, O.decode_bits(inp.s2_bits, c.dtype),
                      inp.z2, c.group, c.dtype)
        U.assert_close(got, ref, f"{cfg.name}: noalloc vs oracle")


def test_noalloc_layer_rejects_sizes_beyond_the_array():
    say("noalloc layer size limit")
    d = U.DevInputs(make_inputs(CONFIGS["tiny"]))
    c = d.cfg
    T_big = 4096                                   # S*K*4 alone is 8 MiB * 16 here: far beyond 64 MiB with K = 7168
    X = torch.zeros((T_big, 7168), dtype=torch.float16, device="cuda")
    ids = torch.zeros((T_big, 8), dtype=torch.int32, device="cuda")
    w = torch.zeros((T_big, 8), dtype=torch.float32, device="cuda")
    out = torch.empty((T_big, 7168), dtype=torch.float16, device="cuda")
    # shapes are validated on the host before any launch: the (too small) weight tensors are never read
    qw1 = torch.zeros((1, 2 * 2048, 7168 // 8), dtype=torch.int32, device="cuda")
    s1 = torch.zeros((1, 2 * 2048, 56), dtype=torch.float16, device="cuda")
    z1 = torch.zeros((1, 2 * 2048, 56), dtype=torch.uint8, device="cuda")
    qw2 = torch.zeros((1, 7168, 2048 // 8), dtype=torch.int32, device="cuda")
    s2 = torch.zeros((1, 7168, 16), dtype=torch.float16, device="cuda")
    z2 = torch.zeros((1, 7168, 16), dtype=torch.uint8, device="cuda")
    with pytest.raises(M.MoEError) as e:
        M.moe_w4a16_layer_noalloc(X, ids, w, qw1, s1, z1, qw2, s2, z2, out, 128)
    assert e.value.status == 3 and "scratch" in str(e.value)
    # and a call that fits still works afterwards
    got = U.dev_to_f64(run_noalloc(d))
    assert np.array_equal(got, U.dev_to_f64(U.run_layer(d)))
