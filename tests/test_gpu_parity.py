"""GPU parity: every HIP entry point against the CPU oracle, through the C ABI.

Integer outputs bit-exact; floating outputs within |gpu - oracle| <= 2e-2 + 1e-2*|oracle|
(the acceptance bound of the benchmark statement, fp32 accumulation on the GPU, fp64 in the
oracle).  Small and medium shapes are compared element by element; the full-size seeded
configurations are compared on sampled outputs the oracle computes one by one."""
from __future__ import annotations

import json
import os
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


def oracle_slot_expert(inp):
    return inp.topk_ids.reshape(-1)


# ------------------------------------------------------------------ bucketing
@pytest.mark.parametrize("T,topk,E,block_m,mode", [
    (16, 2, 8, 16, "uniform"), (1, 1, 1, 16, "uniform"), (1, 8, 256, 16, "uniform"),
    (128, 8, 256, 16, "uniform"), (128, 8, 256, 64, "uniform"), (64, 2, 8, 32, "uniform"),
    (777, 3, 5, 16, "uniform"), (1024, 6, 64, 128, "skew"), (4096, 8, 256, 128, "uniform"),
    (4096, 8, 256, 16, "uniform"), (300, 4, 7, 256, "one_expert"), (200, 2, 1000, 16, "invalid"),
    (33, 1, 1024, 32, "uniform"), (5000, 2, 3, 64, "invalid"),
])
def test_align_bit_exact(T, topk, E, block_m, mode):
    say(f"align T={T} topk={topk} E={E} block_m={block_m} mode={mode}")
    rng = np.random.default_rng(T * 131 + topk * 17 + E)
    if mode == "uniform":
        ids = rng.integers(0, E, (T, topk))
    elif mode == "skew":
        p = 1.0 / np.arange(1, E + 1) ** 1.5
        ids = rng.choice(E, size=(T, topk), p=p / p.sum())
    elif mode == "one_expert":
        ids = np.full((T, topk), E - 1)
    else:
        ids = rng.integers(-2, E + 3, (T, topk))
    ids = ids.astype(np.int32)
    got = U.run_align(U.i32(ids), E, block_m)
    U.assert_align_equal(got, O.align_by_expert(ids, E, block_m), block_m)


def test_align_empty_input():
    say("align T=0")
    ids = torch.zeros((0, 2), dtype=torch.int32, device="cuda")
    got = U.run_align(ids, 4, 16)
    assert got["capacity"] == 0
    assert got["num_padded"].item() == 0
    np.testing.assert_array_equal(got["expert_counts"].cpu().numpy(), [0, 0, 0, 0])
    np.testing.assert_array_equal(got["expert_offsets"].cpu().numpy(), [0] * 5)


# ------------------------------------------------------------------ staged GEMM
def staged_gemm_case(cfg, block_m, which="w1", corrupt_ids=False, tile=None):
    inp = make_inputs(cfg)
    c = inp.cfg
    ids = inp.topk_ids.copy()
    if corrupt_ids:
        ids.reshape(-1)[::5] = c.E + 1
        ids.reshape(-1)[3::11] = -1
    d = U.DevInputs(inp)
    ids_dev = U.i32(ids)
    al = U.run_align(ids_dev, c.E, block_m)
    S = c.S
    if which == "w1":
        A_dev, row_div, qw, s, z, s_bits, N_out = d.X, c.topk, d.qw1, d.s1, d.z1, inp.s1_bits, 2 * c.N
        A64 = O.decode_bits(inp.x_bits, c.dtype)
        qw_h, z_h = inp.qw1, inp.z1
    else:
        rng = np.random.default_rng(99)
        A64 = O.rnd(rng.standard_normal((S, c.N)) * 2.0, c.dtype)
        A_dev, row_div, qw, s, z, s_bits, N_out = U.vals_to_dev(A64, c.dtype), 1, d.qw2, d.s2, d.z2, inp.s2_bits, c.K
        qw_h, z_h = inp.qw2, inp.z2
    C = torch.full((S, N_out), 777.0, dtype=U.TORCH_DT[c.dtype], device="cuda")
    if tile:
        M.moe_set_tile_override(*tile)
    try:
        M.moe_w4a16_grouped_gemm(A_dev, row_div, qw, s, z, al["sorted_slot_ids"], al["block_expert_ids"],
                                 al["num_padded"], S, c.group, block_m, C)
        torch.cuda.synchronize()
    finally:
        M.moe_set_tile_override(0, 0)
    want = O.grouped_gemm(A64, row_div, qw_h, O.decode_bits(s_bits, c.dtype), z_h, ids.reshape(-1),
                          c.group, c.dtype, fill=777.0)
    return U.assert_close(U.dev_to_f64(C), want, f"gemm {which} {cfg} bm={block_m} tile={tile}")


GEMM_SHAPES = [
    dict(T=16, K=256, N=512, E=8, topk=2, group=128, dtype="f16"),
    # ragged feature tail (N_out % 64 != 0) and a single partial K stage
    dict(T=40, K=224, N=96, E=5, topk=3, group=32, dtype="f16"),
    # K tail (2.5 stages of 256), bf16, group 64
    dict(T=70, K=640, N=192, E=4, topk=2, group=64, dtype="bf16"),
    dict(T=9, K=96, N=96, E=3, topk=2, group=32, dtype="f16"),
    # group sizes that are not powers of two / span two chunk-steps
    dict(T=50, K=288, N=96, E=6, topk=2, group=96, dtype="bf16"),
    dict(T=33, K=512, N=256, E=2, topk=1, group=256, dtype="f16"),
]


@pytest.mark.parametrize("shape", GEMM_SHAPES)
@pytest.mark.parametrize("block_m", [16, 64, 256])
@pytest.mark.parametrize("which", ["w1", "w2"])
def test_grouped_gemm_matches_oracle(shape, block_m, which):
    cfg = MoEConfig(name="g", seed=5, **shape)
    say(f"gemm {which} {shape} block_m={block_m}")
    staged_gemm_case(cfg, block_m, which)


@pytest.mark.parametrize("tile", [(1, 1), (1, 2), (1, 4), (2, 1), (2, 2), (2, 4), (4, 2), (4, 4), (8, 2), (8, 4)])
@pytest.mark.parametrize("dtype,group", [("f16", 128), ("bf16", 64), ("f16", 32)])
def test_every_gemm_tile_variant(tile, dtype, group):
    cfg = MoEConfig(name="v", T=150, K=640, N=384, E=3, topk=2, group=group, dtype=dtype, seed=8)
    say(f"gemm variant tile={tile} dtype={dtype} group={group}")
    staged_gemm_case(cfg, 128, "w1", tile=tile)


@pytest.mark.parametrize("tile", [(1, 1), (1, 2), (1, 4), (2, 1), (2, 2)])
@pytest.mark.parametrize("dtype,K", [("f16", 1024), ("bf16", 3072)])
@pytest.mark.parametrize("which", ["w1", "w2"])
def test_register_resident_scale_variants(tile, dtype, K, which):
    """group 128 with 16-byte aligned scale rows: scales / zero points live in registers."""
    cfg = MoEConfig(name="szr", T=90, K=K, N=1024, E=4, topk=2, group=128, dtype=dtype, seed=12)
    say(f"gemm register-scale variant tile={tile} dtype={dtype} K={K} {which}")
    M.moe_set_scale_path(2)
    try:
        staged_gemm_case(cfg, 32, which, tile=tile)
    finally:
        M.moe_set_scale_path(0)


@pytest.mark.parametrize("tpw", [1, 2, 3, 8])
@pytest.mark.parametrize("which", ["w1", "w2"])
def test_multi_tile_workgroups(tpw, which):
    """Several feature tiles per workgroup (continuous pipeline across tiles), including a
    ragged last group of tiles."""
    cfg = MoEConfig(name="tpw", T=70, K=1024, N=2048, E=5, topk=2, group=128, dtype="f16", seed=14)
    say(f"gemm tiles_per_workgroup={tpw} {which}")
    M.moe_set_scale_path(2)
    M.moe_set_tiles_per_workgroup(tpw)
    try:
        staged_gemm_case(cfg, 16, which, tile=(1, 2))
    finally:
        M.moe_set_tiles_per_workgroup(0)
        M.moe_set_scale_path(0)


def test_scale_paths_agree_bitwise():
    cfg = MoEConfig(name="szr_eq", T=64, K=2048, N=1024, E=6, topk=2, group=128, dtype="f16", seed=13)
    say("layer with LDS-table scales vs register scales")
    d = U.DevInputs(make_inputs(cfg))
    outs = []
    for mode in (1, 2):
        M.moe_set_scale_path(mode)
        try:
            outs.append(U.dev_to_f64(U.run_layer(d)))
        finally:
            M.moe_set_scale_path(0)
    assert np.array_equal(outs[0], outs[1])


@pytest.mark.parametrize("dtype,group,K", [("f16", 128, 1024), ("bf16", 64, 512), ("f16", 32, 256)])
@pytest.mark.parametrize("block_m", [16, 64, 128])
def test_zero_and_negative_scales(dtype, group, K, block_m):
    """A zero scale silences its group, a negative one flips it: both are legal inputs (the
    large-tile kernels keep the accumulator in units of the group scale and must not divide by
    zero)."""
    cfg = MoEConfig(name="zs", T=100, K=K, N=256, E=3, topk=2, group=group, dtype=dtype, seed=15)
    say(f"gemm zero/negative scales dtype={dtype} group={group} block_m={block_m}")
    inp = make_inputs(cfg)
    rng = np.random.default_rng(3)
    s = O.decode_bits(inp.s1_bits, dtype)
    s[rng.random(s.shape) < 0.25] = 0.0
    s[rng.random(s.shape) < 0.15] *= -1.0
    s[:, :, 0] = 0.0                       # first group of every row
    s[0, :8, :] = 0.0                      # whole rows
    inp.s1_bits = O.encode_bits(s, dtype)
    d = U.DevInputs(inp)
    al = U.run_align(d.ids, cfg.E, block_m)
    C = torch.full((cfg.S, 2 * cfg.N), 777.0, dtype=U.TORCH_DT[dtype], device="cuda")
    M.moe_w4a16_grouped_gemm(d.X, cfg.topk, d.qw1, d.s1, d.z1, al["sorted_slot_ids"], al["block_expert_ids"],
                             al["num_padded"], cfg.S, cfg.group, block_m, C)
    torch.cuda.synchronize()
    want = O.grouped_gemm(O.decode_bits(inp.x_bits, dtype), cfg.topk, inp.qw1, s, inp.z1,
                          inp.topk_ids.reshape(-1), cfg.group, dtype)
    U.assert_close(U.dev_to_f64(C), want, "zero/negative scales")


def test_grouped_gemm_ignores_invalid_slots_and_leaves_rows_untouched():
    cfg = MoEConfig(name="inv", T=30, K=256, N=128, E=4, topk=2, group=128, dtype="f16", seed=6)
    say("gemm with out-of-range expert ids")
    staged_gemm_case(cfg, 16, "w1", corrupt_ids=True)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("which", ["w1", "w2"])
def test_grouped_gemm_block_256_register_scales(dtype, which):
    """256-row bucketing blocks (walked as two 128-row tiles) on the register-scale kernels; each
    expert owns two blocks, the second one ragged."""
    cfg = MoEConfig(name="bm256", T=700, K=1024, N=1024, E=3, topk=2, group=128, dtype=dtype, seed=31)
    say(f"gemm block_m=256 register scales dtype={dtype} {which}")
    staged_gemm_case(cfg, 256, which)
    assert M.moe_last_gemm_plan()["mt"] == 8


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("block_m", [128, 256])
def test_wide_tile_every_live_sub_tile_count(dtype, block_m):
    """The eight-wave 128-token tile runs a main loop compiled per number of live 16-row
    sub-tiles: experts sized so that tiles with 1, 2, ... 8 live sub-tiles all occur (full and
    ragged last sub-tiles, a 129-row expert, an empty expert), staged GEMMs and the layer."""
    counts = [5, 16, 17, 40, 0, 64, 70, 96, 100, 113, 128, 129, 260]
    E, T = len(counts), sum(counts)
    cfg = MoEConfig(name="live", T=T, K=1024, N=1024, E=E, topk=1, group=128, dtype=dtype, seed=33)
    say(f"wide tile live sub-tile counts dtype={dtype} block_m={block_m}")
    inp = make_inputs(cfg)
    ids = np.repeat(np.arange(E), counts).astype(np.int32)
    np.random.default_rng(5).shuffle(ids)
    inp.topk_ids = ids.reshape(T, 1)
    inp.topk_weights = np.full((T, 1), 0.75, np.float32)
    d = U.DevInputs(inp)
    al = U.run_align(d.ids, E, block_m)
    tables = (al["sorted_slot_ids"], al["block_expert_ids"], al["num_padded"])
    H = torch.full((T, 2 * cfg.N), 777.0, dtype=U.TORCH_DT[dtype], device="cuda")
    M.moe_w4a16_grouped_gemm(d.X, 1, d.qw1, d.s1, d.z1, *tables, T, cfg.group, block_m, H)
    torch.cuda.synchronize()
    assert M.moe_last_gemm_plan()["waves"] == 8
    want = O.grouped_gemm(O.decode_bits(inp.x_bits, dtype), 1, inp.qw1, O.decode_bits(inp.s1_bits, dtype), inp.z1,
                          ids, cfg.group, dtype, fill=777.0)
    U.assert_close(U.dev_to_f64(H), want, "wide tile gate/up GEMM")
    M.moe_set_block_m_override(block_m)
    try:
        out = U.run_layer(d)
    finally:
        M.moe_set_block_m_override(0)
    U.assert_close(U.dev_to_f64(out), oracle_layer(inp), "wide tile layer")
    # the four-wave tiles on the same blocks give the same numbers up to fp32 summation order
    M.moe_set_wide_tiles(1)
    try:
        H4 = torch.full((T, 2 * cfg.N), 777.0, dtype=U.TORCH_DT[dtype], device="cuda")
        M.moe_w4a16_grouped_gemm(d.X, 1, d.qw1, d.s1, d.z1, *tables, T, cfg.group, block_m, H4)
        torch.cuda.synchronize()
        assert M.moe_last_gemm_plan()["waves"] == 4
    finally:
        M.moe_set_wide_tiles(0)
    U.assert_close(U.dev_to_f64(H4), want, "four-wave tile on 128-slot blocks")


@pytest.mark.parametrize("dtype,group", [("f16", 128), ("bf16", 64)])
def test_layer_forced_to_block_256(dtype, group):
    cfg = MoEConfig("bm256_layer", T=400, K=1024, N=1024, E=3, topk=2, group=group, dtype=dtype, seed=32)
    say(f"layer forced to block_m=256 {cfg}")
    inp = make_inputs(cfg)
    M.moe_set_block_m_override(256)
    try:
        out = U.run_layer(U.DevInputs(inp))
    finally:
        M.moe_set_block_m_override(0)
    U.assert_close(U.dev_to_f64(out), oracle_layer(inp), "layer block_m 256")


# ------------------------------------------------------------------ elementwise steps
@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("S,N", [(37, 64), (5, 7), (300, 1408)])
def test_silu_mul_matches_oracle(dt, S, N):
    say(f"silu_mul dt={dt} S={S} N={N}")
    rng = np.random.default_rng(S + N)
    H = O.rnd(rng.standard_normal((S, 2 * N)) * 4.0, dt)
    if N >= 4:
        H[0, :4] = [-30.0, 30.0, 0.0, -0.0]
    act = torch.empty((S, N), dtype=U.TORCH_DT[dt], device="cuda")
    M.moe_silu_mul(U.vals_to_dev(H, dt), act)
    torch.cuda.synchronize()
    U.assert_close(U.dev_to_f64(act), O.silu_mul(H, dt), "silu_mul")


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("T,topk,K", [(16, 2, 256), (3, 5, 9), (200, 8, 7168)])
def test_combine_matches_oracle(dt, T, topk, K):
    say(f"combine dt={dt} T={T} topk={topk} K={K}")
    rng = np.random.default_rng(T + K)
    Y = O.rnd(rng.standard_normal((T * topk, K)) * 20.0, dt)
    w = rng.dirichlet(np.ones(topk), T).astype(np.float32)
    out = torch.empty((T, K), dtype=U.TORCH_DT[dt], device="cuda")
    M.moe_combine(U.vals_to_dev(Y, dt), torch.from_numpy(w).cuda(), out)
    torch.cuda.synchronize()
    U.assert_close(U.dev_to_f64(out), O.combine(Y, w, dt), "combine")


def test_staged_chain_with_invalid_ids_uses_the_masked_combine():
    """align -> GEMM -> SiLU-and-multiply -> GEMM -> combine through the staged entry points with
    expert ids outside [0, E): the GEMMs leave the rows of such slots untouched (NaN here), the
    masked combine lets them contribute zero, as the oracle's combine(slot_valid=...) does."""
    cfg = MoEConfig("staged_inv", T=40, K=256, N=128, E=5, topk=3, group=128, dtype="f16", seed=44)
    say(f"staged chain with invalid ids {cfg}")
    inp = make_inputs(cfg)
    inp.topk_ids[1, 0] = cfg.E
    inp.topk_ids[6, 2] = -3
    inp.topk_ids[9, :] = 77
    d = U.DevInputs(inp)
    block_m = 16
    al = U.run_align(d.ids, cfg.E, block_m)
    tables = (al["sorted_slot_ids"], al["block_expert_ids"], al["num_padded"])
    nan = float("nan")
    H = torch.full((cfg.S, 2 * cfg.N), nan, dtype=torch.float16, device="cuda")
    M.moe_w4a16_grouped_gemm(d.X, cfg.topk, d.qw1, d.s1, d.z1, *tables, cfg.S, cfg.group, block_m, H)
    act = torch.empty((cfg.S, cfg.N), dtype=torch.float16, device="cuda")
    M.moe_silu_mul(H, act)
    Y = torch.full((cfg.S, cfg.K), nan, dtype=torch.float16, device="cuda")
    M.moe_w4a16_grouped_gemm(act, 1, d.qw2, d.s2, d.z2, *tables, cfg.S, cfg.group, block_m, Y)
    out = torch.empty((cfg.T, cfg.K), dtype=torch.float16, device="cuda")
    M.moe_combine_masked(Y, d.w, d.ids, cfg.E, out)
    torch.cuda.synchronize()
    got = U.dev_to_f64(out)
    assert np.all(got[9] == 0)
    # the staged chain rounds Y to 16 bits (the fused layer does not): build the reference from the staged oracles
    X64 = O.decode_bits(inp.x_bits, "f16")
    se = inp.topk_ids.reshape(-1)
    Ho = O.grouped_gemm(X64, cfg.topk, inp.qw1, O.decode_bits(inp.s1_bits, "f16"), inp.z1, se, cfg.group, "f16", fill=0.0)
    Yo = O.grouped_gemm(O.silu_mul(Ho, "f16"), 1, inp.qw2, O.decode_bits(inp.s2_bits, "f16"), inp.z2, se, cfg.group,
                        "f16", fill=0.0)
    want = O.combine(Yo, inp.topk_weights, "f16", slot_valid=(se >= 0) & (se < cfg.E))
    U.assert_close(got, want, "staged chain, masked combine")


# ------------------------------------------------------------------ whole layer, element by element
def oracle_layer(inp, **kw):
    c = inp.cfg
    return O.layer(O.decode_bits(inp.x_bits, c.dtype), inp.topk_ids, inp.topk_weights, inp.qw1,
                   O.decode_bits(inp.s1_bits, c.dtype), inp.z1, inp.qw2,
                   O.decode_bits(inp.s2_bits, c.dtype), inp.z2, c.group, c.dtype, **kw)


LAYER_SHAPES = [
    CONFIGS["tiny"],
    MoEConfig("mid_f16", T=70, K=512, N=384, E=12, topk=3, group=128, dtype="f16", seed=3),
    MoEConfig("mid_bf16_skew", T=200, K=256, N=192, E=16, topk=4, group=64, dtype="bf16", skew=True, seed=4),
    MoEConfig("one_token", T=1, K=256, N=128, E=8, topk=2, group=128, dtype="f16", seed=5),
    MoEConfig("dense_e1", T=20, K=128, N=128, E=1, topk=1, group=32, dtype="bf16", seed=6),
    MoEConfig("big_blocks", T=600, K=256, N=128, E=4, topk=2, group=128, dtype="f16", seed=7),
]


@pytest.mark.parametrize("cfg", LAYER_SHAPES, ids=lambda c: c.name)
def test_layer_matches_oracle_elementwise(cfg):
    say(f"layer {cfg}")
    inp = make_inputs(cfg)
    out = U.run_layer(U.DevInputs(inp))
    U.assert_close(U.dev_to_f64(out), oracle_layer(inp), f"layer {cfg.name}")


@pytest.mark.parametrize("N,splits", [(2048, 2), (3072, 2), (3072, 3), (3072, 8), (5120, 0), (5120, 3)])
@pytest.mark.parametrize("tile", [(1, 2), (2, 2), (4, 2)])
def test_layer_with_split_reduction(N, splits, tile):
    """The down projection's reduction cut into ranges (partial float32 planes added by the
    combine): even and ragged ranges, more splits than scale panels, the automatic choice."""
    cfg = MoEConfig("ksplit", T=20, K=256, N=N, E=3, topk=2, group=128, dtype="f16", seed=21)
    say(f"layer reduction splits={splits} tile={tile} {cfg}")
    inp = make_inputs(cfg)
    M.moe_set_reduction_splits(splits)
    M.moe_set_tile_override(*tile)
    try:
        out = U.run_layer(U.DevInputs(inp))
    finally:
        M.moe_set_reduction_splits(0)
        M.moe_set_tile_override(0, 0)
    U.assert_close(U.dev_to_f64(out), oracle_layer(inp), f"layer split {N}/{splits}")


def test_layer_split_reduction_limited_by_workspace():
    """More splits requested than partial planes fit in the workspace (large token tiles reserve
    one plane): the layer uses what fits and the result is unchanged."""
    cfg = MoEConfig("ksplit_ws", T=200, K=256, N=3072, E=2, topk=1, group=128, dtype="f16", seed=22)
    say(f"layer reduction splits vs workspace {cfg}")
    inp = make_inputs(cfg)
    M.moe_set_reduction_splits(3)
    try:
        out = U.run_layer(U.DevInputs(inp))
    finally:
        M.moe_set_reduction_splits(0)
    U.assert_close(U.dev_to_f64(out), oracle_layer(inp), "layer split vs workspace")


def test_layer_with_invalid_expert_ids_contributes_zero():
    cfg = MoEConfig("inv_layer", T=24, K=256, N=128, E=6, topk=3, group=128, dtype="f16", seed=9)
    say(f"layer invalid ids {cfg}")
    inp = make_inputs(cfg)
    inp.topk_ids[2, 0] = 6
    inp.topk_ids[5, 2] = -1
    inp.topk_ids[7, :] = 100
    out = U.run_layer(U.DevInputs(inp))
    want = oracle_layer(inp)
    assert np.all(want[7] == 0)
    U.assert_close(U.dev_to_f64(out), want, "layer invalid ids")


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_layer_matches_golden_fixture(dt):
    with open(os.path.join(os.path.dirname(__file__), "golden", f"small_layer_{dt}.json")) as f:
        doc = json.load(f)
    c = doc["config"]
    cfg = MoEConfig("golden_small", T=c["T"], K=c["K"], N=c["N"], E=c["E"], topk=c["topk"],
                    group=c["group"], dtype=dt, seed=c["seed"])
    say(f"layer golden {dt}")
    inp = make_inputs(cfg)
    d = U.DevInputs(inp)
    out = U.run_layer(d)
    U.assert_close(U.dev_to_f64(out), O.decode_bits(np.array(doc["out_bits"], np.uint16), dt), "golden out")
    al = U.run_align(d.ids, cfg.E, c["block_m"])
    U.assert_align_equal(al, {k: np.array(v, np.int32) for k, v in doc["align"].items()}, c["block_m"])


def test_layer_token_permutation_permutes_output():
    cfg = MoEConfig("perm", T=48, K=256, N=128, E=8, topk=2, group=128, dtype="f16", seed=10)
    say(f"layer permutation {cfg}")
    inp = make_inputs(cfg)
    base = U.dev_to_f64(U.run_layer(U.DevInputs(inp)))
    perm = np.random.default_rng(1).permutation(cfg.T)
    inp.x_bits, inp.topk_ids, inp.topk_weights = inp.x_bits[perm], inp.topk_ids[perm], inp.topk_weights[perm]
    got = U.dev_to_f64(U.run_layer(U.DevInputs(inp)))
    # each token's result does not depend on its position: equal up to the tolerance at worst,
    # and in fact bitwise here because the per-token summation order does not change
    U.assert_close(got, base[perm], "permutation")
    assert np.array_equal(got, base[perm])


def test_layer_empty_batch_is_a_noop():
    say("layer T=0")
    cfg = MoEConfig("empty", T=0, K=256, N=128, E=4, topk=2, group=128, dtype="f16", seed=1)
    inp = make_inputs(MoEConfig("e1", T=1, K=256, N=128, E=4, topk=2, group=128, dtype="f16", seed=1))
    d = U.DevInputs(inp)
    d.cfg = cfg
    d.X, d.ids, d.w = d.X[:0].contiguous(), d.ids[:0].contiguous(), d.w[:0].contiguous()
    out = torch.empty((0, 256), dtype=torch.float16, device="cuda")
    U.run_layer(d, out)


def test_error_paths_report_status():
    say("error paths")
    inp = make_inputs(CONFIGS["tiny"])
    d = U.DevInputs(inp)
    out = torch.empty((16, 256), dtype=torch.float16, device="cuda")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(M.MoEError) as e:
        M.moe_w4a16_layer(d.X, d.ids, d.w, d.qw1, d.s1, d.z1, d.qw2, d.s2, d.z2, out, 128, small)
    assert e.value.status == 3 and "workspace" in str(e.value)
    with pytest.raises(M.MoEError) as e:
        M.moe_w4a16_layer(d.X, d.ids, d.w, d.qw1, d.s1, d.z1, d.qw2, d.s2, d.z2, out, 48, small)
    assert e.value.status == 2
    al = U.run_align(d.ids, 8, 16)
    H = torch.empty((32, d.qw1.shape[1]), dtype=torch.float16, device="cuda")
    with pytest.raises(M.MoEError) as e:
        M.moe_w4a16_grouped_gemm(d.X, 2, d.qw1, d.s1, d.z1, al["sorted_slot_ids"], al["block_expert_ids"],
                                 al["num_padded"], 32, 128, 24, H)
    assert e.value.status == 1
    # a buffer of the wrong shape never reaches the library: the binding refuses it
    with pytest.raises(ValueError):
        M.moe_w4a16_grouped_gemm(d.X, 2, d.qw1, d.s1, d.z1, al["sorted_slot_ids"], al["block_expert_ids"],
                                 al["num_padded"], 32, 128, 16, out)


# ------------------------------------------------------------------ full-size seeded configurations
def stratified_samples(slot_expert, E, block_m, N_out, plan, rng, per_expert=8):
    """(slot, feature) samples aimed at the borders of the launch's decomposition: for every active
    expert the first and last row of each of its row blocks (and of each 16*mt-row tile inside a
    block), paired with features taken in rotation from: column 0, column N_out - 1, and the first
    and last column of the first and last feature tile of every workgroup's tile group; plus two
    uniformly random entries per expert."""
    tile_w = 16 * plan["nt"] * plan["waves"]
    group_w = tile_w * plan["tiles_per_workgroup"]
    cols = {0, N_out - 1}
    for g0 in range(0, N_out, group_w):
        g1 = min(g0 + group_w, N_out)
        last_tile0 = g0 + ((g1 - g0 - 1) // tile_w) * tile_w
        cols.update({g0, min(g0 + tile_w, g1) - 1, last_tile0, g1 - 1})
    cols = sorted(cols)
    rows_per_tile = 16 * plan["mt"]
    ss, nn = [], []
    cursor = 0
    for e in range(E):
        slots = np.nonzero(slot_expert == e)[0]          # ascending = the order inside the expert's segment
        if slots.size == 0:
            continue
        picks = set()
        for r0 in range(0, slots.size, min(block_m, rows_per_tile)):
            picks.update({r0, min(r0 + min(block_m, rows_per_tile), slots.size) - 1})
        picks = sorted(picks)
        n_here = max(per_expert - 2, len(picks))
        for i in range(n_here):
            ss.append(int(slots[picks[i % len(picks)]]))
            nn.append(cols[cursor % len(cols)])
            cursor += 1
        for _ in range(2):
            ss.append(int(slots[rng.integers(0, slots.size)]))
            nn.append(int(rng.integers(0, N_out)))
    return np.array(ss), np.array(nn), len(cols)


def sampled_gemm_check(inp, d, which, block_m, rng):
    """Staged GEMM at full size, in the tile plan the library picks for it: stratified (slot, feature)
    outputs against the oracle's single-entry evaluation of the definition."""
    c = inp.cfg
    S = c.S
    al = U.run_align(d.ids, c.E, block_m)
    U.assert_align_equal(al, O.align_by_expert(inp.topk_ids, c.E, block_m), block_m)
    if which == "w1":
        A64, A_dev, row_div = O.decode_bits(inp.x_bits, c.dtype), d.X, c.topk
        qw, s, z, qw_h, s_h, z_h, N_out = d.qw1, d.s1, d.z1, inp.qw1, inp.s1_bits, inp.z1, 2 * c.N
    else:
        A64 = O.rnd(np.random.default_rng(17).standard_normal((S, c.N)) * 2.0, c.dtype)
        A_dev, row_div = U.vals_to_dev(A64, c.dtype), 1
        qw, s, z, qw_h, s_h, z_h, N_out = d.qw2, d.s2, d.z2, inp.qw2, inp.s2_bits, inp.z2, c.K
    C = torch.empty((S, N_out), dtype=U.TORCH_DT[c.dtype], device="cuda")
    M.moe_w4a16_grouped_gemm(A_dev, row_div, qw, s, z, al["sorted_slot_ids"], al["block_expert_ids"],
                             al["num_padded"], S, c.group, block_m, C)
    torch.cuda.synchronize()
    plan = M.moe_last_gemm_plan()
    se = inp.topk_ids.reshape(-1)
    ss, nn, ncols = stratified_samples(se, c.E, block_m, N_out, plan, rng)
    say(f"  staged {which}: plan {plan}, {ss.size} samples over {np.unique(se[ss]).size} experts, "
        f"{ncols} border columns")
    got = U.dev_to_f64(C[torch.from_numpy(ss).cuda(), torch.from_numpy(nn).cuda()])
    want = np.empty(ss.size)
    for i, (si, ni) in enumerate(zip(ss, nn)):
        e = int(se[si])
        want[i] = O.gemm_entry(A64, row_div, qw_h[e, ni][None, None], O.decode_bits(s_h[e, ni], c.dtype)[None, None],
                               z_h[e, ni][None, None], np.zeros(S, np.int64), c.group, int(si), 0)
    U.assert_close(got, O.rnd(want, c.dtype), f"{c.name} staged {which} samples")
    del C


def tokens_covering_experts(topk_ids, n_tokens, always=()):
    """Greedy choice of n_tokens tokens whose routed experts are as many distinct ones as possible."""
    chosen = list(dict.fromkeys(int(t) for t in always))
    seen = set(int(e) for t in chosen for e in topk_ids[t])
    while len(chosen) < n_tokens:
        gain = np.array([len(set(row.tolist()) - seen) for row in topk_ids])
        gain[chosen] = -1
        t = int(np.argmax(gain))
        chosen.append(t)
        seen.update(int(e) for e in topk_ids[t])
    return sorted(chosen), len(seen)


def prepacked_layer(d):
    c = d.cfg
    dtc = M.MOE_F16 if c.dtype == "f16" else M.MOE_BF16
    p1, p2 = torch.empty_like(d.qw1), torch.empty_like(d.qw2)
    M.moe_repack_qweight(d.qw1, False, p1)
    M.moe_repack_qweight(d.qw2, True, p2)
    ws = torch.empty(M.moe_w4a16_layer_workspace_bytes(c.T, c.K, c.N, c.E, c.topk, dtc), dtype=torch.uint8, device="cuda")
    out = torch.full((c.T, c.K), float("nan"), dtype=U.TORCH_DT[c.dtype], device="cuda")
    M.moe_w4a16_layer_prepacked(d.X, d.ids, d.w, p1, d.s1, d.z1, p2, d.s2, d.z2, out, c.group, ws)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("name", ["mixtral_decode", "skewed_bf16"])
def test_full_size_config_elementwise(name):
    """Configurations whose oracle finishes in about a minute: the whole layer output and both staged
    GEMMs, every element, in the launch configuration the benchmark times."""
    cfg = CONFIGS[name]
    say(f"full-size elementwise {cfg}: generating")
    inp = make_inputs(cfg)
    d = U.DevInputs(inp)
    say(f"full-size elementwise {name}: oracle (whole layer with intermediates)")
    want, mid = oracle_layer(inp, return_intermediates=True)
    block_m = M.moe_layer_block_m_for(cfg.T, cfg.K, cfg.N, cfg.E, cfg.topk, cfg.group)
    al = U.run_align(d.ids, cfg.E, block_m)
    U.assert_align_equal(al, O.align_by_expert(inp.topk_ids, cfg.E, block_m), block_m)
    tables = (al["sorted_slot_ids"], al["block_expert_ids"], al["num_padded"])
    say(f"full-size elementwise {name}: staged gate/up GEMM (block_m={block_m})")
    H = torch.empty((cfg.S, 2 * cfg.N), dtype=U.TORCH_DT[cfg.dtype], device="cuda")
    M.moe_w4a16_grouped_gemm(d.X, cfg.topk, d.qw1, d.s1, d.z1, *tables, cfg.S, cfg.group, block_m, H)
    torch.cuda.synchronize()
    say(f"  plan {M.moe_last_gemm_plan()}")
    U.assert_close(U.dev_to_f64(H), mid["H"], f"{name} staged gate/up GEMM, all {H.numel()} outputs")
    say(f"full-size elementwise {name}: staged SiLU-and-multiply and down GEMM on the oracle's act")
    act = torch.empty((cfg.S, cfg.N), dtype=U.TORCH_DT[cfg.dtype], device="cuda")
    M.moe_silu_mul(U.vals_to_dev(mid["H"], cfg.dtype), act)
    torch.cuda.synchronize()
    U.assert_close(U.dev_to_f64(act), mid["act"], f"{name} staged silu_mul")
    Y = torch.empty((cfg.S, cfg.K), dtype=U.TORCH_DT[cfg.dtype], device="cuda")
    M.moe_w4a16_grouped_gemm(U.vals_to_dev(mid["act"], cfg.dtype), 1, d.qw2, d.s2, d.z2, *tables, cfg.S, cfg.group,
                             block_m, Y)
    torch.cuda.synchronize()
    say(f"  plan {M.moe_last_gemm_plan()}")
    U.assert_close(U.dev_to_f64(Y), O.rnd(mid["Y"], cfg.dtype), f"{name} staged down GEMM, all {Y.numel()} outputs")
    say(f"full-size elementwise {name}: layer")
    got = U.dev_to_f64(U.run_layer(d))
    say(f"  down-projection plan {M.moe_last_gemm_plan()}")
    worst = U.assert_close(got, want, f"{name} layer, all {got.size} outputs")
    say(f"  layer worst error / bound = {worst:.4f}")
    assert np.array_equal(got, U.dev_to_f64(U.run_layer(d))), "layer is not run-to-run deterministic"
    if cfg.group == 128 and cfg.K % 1024 == 0 and cfg.N % 1024 == 0:
        say(f"full-size elementwise {name}: layer on operand-order weights")
        U.assert_close(U.dev_to_f64(prepacked_layer(d)), want, f"{name} prepacked layer, all outputs")


@pytest.mark.parametrize("name,n_tokens", [("deepseek_decode", 16), ("deepseek_prefill", 8)])
def test_full_size_config_stratified(name, n_tokens):
    """The two 256-expert configurations (5.9 GB of weights: a full oracle pass is out of reach):
    staged GEMMs on stratified samples -- every active expert, every row block, the border tiles
    of every tile group -- and the layer on tokens chosen to cover as many experts as possible."""
    cfg = CONFIGS[name]
    say(f"full-size stratified {cfg}: generating")
    inp = make_inputs(cfg)
    d = U.DevInputs(inp)
    rng = np.random.default_rng(123)
    block_m = M.moe_layer_block_m_for(cfg.T, cfg.K, cfg.N, cfg.E, cfg.topk, cfg.group)
    say(f"full-size stratified {name}: staged GEMM samples (block_m={block_m})")
    sampled_gemm_check(inp, d, "w1", block_m, rng)
    sampled_gemm_check(inp, d, "w2", block_m, rng)
    say(f"full-size stratified {name}: layer")
    got = U.dev_to_f64(U.run_layer(d))
    assert np.all(np.isfinite(got))
    loads = np.bincount(inp.topk_ids.reshape(-1), minlength=cfg.E)
    hot_expert = int(np.argmax(loads))
    tok_hot = int(np.nonzero((inp.topk_ids == hot_expert).any(axis=1))[0][0])
    tokens, n_experts = tokens_covering_experts(inp.topk_ids, n_tokens, always=(0, cfg.T - 1, tok_hot))
    say(f"full-size stratified {name}: oracle for tokens {tokens} ({n_experts} distinct experts)")
    assert n_experts >= (100 if n_tokens >= 16 else 48)
    want = oracle_layer(inp, tokens=tokens)
    worst = U.assert_close(got[tokens], want, f"{name} layer tokens {tokens}")
    say(f"  layer worst error / bound = {worst:.4f}")
    assert np.array_equal(got, U.dev_to_f64(U.run_layer(d))), "layer is not run-to-run deterministic"
    say(f"full-size stratified {name}: layer on operand-order weights, same tokens")
    U.assert_close(U.dev_to_f64(prepacked_layer(d))[tokens], want, f"{name} prepacked layer tokens {tokens}")


def test_layer_large_batch_byte_offsets_beyond_4_gib():
    """T = 16384 on the 256-expert layer shape: 131072 slots, a float32 down-projection plane of
    3.76 GB, i.e. byte offsets past 2^32 in the workspace.  The first token, one in the middle and
    the last two (whose slots sit at the far end of every intermediate) against the oracle."""
    import dataclasses
    cfg = dataclasses.replace(CONFIGS["deepseek_prefill"], T=16384)
    say(f"large batch {cfg}: generating")
    inp = make_inputs(cfg)
    d = U.DevInputs(inp)
    got = U.dev_to_f64(U.run_layer(d))
    tokens = [0, cfg.T // 2 + 1, cfg.T - 2, cfg.T - 1]
    say(f"large batch: oracle for tokens {tokens}")
    want = oracle_layer(inp, tokens=tokens)
    worst = U.assert_close(got[tokens], want, f"T={cfg.T} layer tokens {tokens}")
    say(f"  layer worst error / bound = {worst:.4f}")
