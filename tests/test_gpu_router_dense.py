"""GPU parity of the router and of the plain (one weight matrix, no routing) W4A16 GEMM.

Router: expert ids bit-exact against the oracle's selection; weights within 2e-6 absolute
(float32 exp / divide / k-term sum against float64: a few float32 ulps of values <= 1).
Dense GEMM: the floating-point bound of the benchmark statement."""
from __future__ import annotations

import sys

import numpy as np
import pytest
import torch

from moe_workloads import CONFIGS, MoEConfig, make_inputs, skew_bias
from oracle import moe_oracle as O

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2504_16214_amd as M
    import gpu_util as U

W_ATOL = 2e-6


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def run_router(logits: np.ndarray, bias, topk: int):
    T, E = logits.shape
    ld = torch.from_numpy(np.ascontiguousarray(logits, dtype=np.float32)).cuda()
    bd = None if bias is None else torch.from_numpy(np.ascontiguousarray(bias, dtype=np.float32)).cuda()
    ids = torch.full((T, topk), -7, dtype=torch.int32, device="cuda")
    w = torch.full((T, topk), float("nan"), dtype=torch.float32, device="cuda")
    M.moe_route_topk(ld, bd, ids, w)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), w.cpu().numpy()


@pytest.mark.parametrize("T,E,topk,with_bias", [
    (16, 8, 2, False), (64, 8, 2, False), (128, 256, 8, False), (1024, 64, 6, True), (37, 100, 5, True),
    (5, 1024, 64, False), (9, 1, 1, False), (3, 70, 70 - 6, True), (4096, 256, 8, False), (1, 65, 3, False),
])
def test_router_matches_oracle(T, E, topk, with_bias):
    say(f"router T={T} E={E} topk={topk} bias={with_bias}")
    rng = np.random.default_rng(1000 + T + 7 * E + topk)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    bias = skew_bias(E) if with_bias else None
    ids, w = run_router(logits, bias, topk)
    ids_o, w_o = O.route_topk(logits, topk, bias=bias)
    np.testing.assert_array_equal(ids, ids_o)
    assert np.max(np.abs(w.astype(np.float64) - w_o)) <= W_ATOL
    assert np.all(np.abs(w.astype(np.float64).sum(axis=1) - 1.0) <= 1e-5)


def test_router_ties_signed_zeros_and_infinities():
    say("router ties")
    E, topk = 40, 4
    logits = np.random.default_rng(3).standard_normal((6, E)).astype(np.float32)
    logits[0, :] = 1.5                                     # all equal: ids 0..3
    logits[1, [30, 2, 17]] = 8.0                           # three-way tie for the top
    logits[2, :] = -1.0; logits[2, 11] = -0.0; logits[2, 12] = 0.0
    logits[3, :] = -np.inf; logits[3, [5, 9, 33, 34]] = [0.5, 0.25, 0.125, 1.0]   # -inf never beats a finite value
    logits[4, 39] = logits[4, 0] = 3.0                     # first and last index
    ids, w = run_router(logits, None, topk)
    ids_o, w_o = O.route_topk(logits, topk)
    np.testing.assert_array_equal(ids, ids_o)
    assert list(ids[0]) == [0, 1, 2, 3] and list(ids[1][:3]) == [2, 17, 30] and list(ids[2][:2]) == [11, 12]
    assert list(ids[3]) == [34, 5, 9, 33] and list(ids[4][:2]) == [0, 39]
    assert np.max(np.abs(w.astype(np.float64) - w_o)) <= W_ATOL


@pytest.mark.parametrize("name", ["mixtral_decode", "skewed_bf16"])
def test_router_reproduces_the_workload_routing(name):
    """The seeded configurations' stored logits give back the ids the layer inputs were built
    from (the generator's own routing), bit for bit."""
    cfg = CONFIGS[name]
    say(f"router on {name}")
    # only the logits are needed: a tiny stand-in shape with the same T, E, topk and seed draw order
    rng = np.random.default_rng(cfg.seed)
    rng.standard_normal((cfg.T, cfg.K))                    # X is drawn first
    logits = rng.standard_normal((cfg.T, cfg.E)).astype(np.float32)
    bias = skew_bias(cfg.E) if name == "skewed_bf16" else None
    ids, w = run_router(logits, bias, cfg.topk)
    ids_o, w_o = O.route_topk(logits, cfg.topk, bias=bias)
    np.testing.assert_array_equal(ids, ids_o)
    assert np.max(np.abs(w.astype(np.float64) - w_o)) <= W_ATOL


def run_route_align(logits, bias, topk, block_m):
    T, E = logits.shape
    ld = torch.from_numpy(np.ascontiguousarray(logits, dtype=np.float32)).cuda()
    bd = None if bias is None else torch.from_numpy(np.ascontiguousarray(bias, dtype=np.float32)).cuda()
    cap = M.moe_align_capacity(T, topk, E, block_m)
    ids = torch.full((T, topk), -7, dtype=torch.int32, device="cuda")
    w = torch.full((T, topk), float("nan"), dtype=torch.float32, device="cuda")
    out = {
        "expert_counts": torch.full((E,), -7, dtype=torch.int32, device="cuda"),
        "expert_offsets": torch.full((E + 1,), -7, dtype=torch.int32, device="cuda"),
        "sorted_slot_ids": torch.full((max(cap, 1),), -7, dtype=torch.int32, device="cuda"),
        "block_expert_ids": torch.full((max(cap // block_m, 1),), -7, dtype=torch.int32, device="cuda"),
        "num_padded": torch.full((1,), -7, dtype=torch.int32, device="cuda"),
    }
    M.moe_route_align(ld, bd, block_m, ids, w, out["expert_counts"], out["expert_offsets"], out["sorted_slot_ids"],
                      out["block_expert_ids"], out["num_padded"])
    torch.cuda.synchronize()
    out["capacity"] = cap
    return ids.cpu().numpy(), w.cpu().numpy(), out


def config_logits(cfg):
    """The logits of a seeded configuration (drawn after X), raw: the skew bias is handed to the router."""
    rng = np.random.default_rng(cfg.seed)
    rng.standard_normal((cfg.T, cfg.K))
    return rng.standard_normal((cfg.T, cfg.E)).astype(np.float32), (skew_bias(cfg.E) if cfg.skew else None)


@pytest.mark.parametrize("name", ["tiny", "mixtral_decode", "deepseek_decode", "deepseek_prefill", "skewed_bf16"])
def test_route_align_on_the_five_configurations(name):
    """Router fused with the bucketing (one launch up to 64 tokens, the two kernels beyond): ids and
    tables bit for bit those of the oracle's router followed by its bucketing, on the logits of the
    five seeded configurations, in the block size the layer uses for them."""
    cfg = CONFIGS[name]
    block_m = M.moe_layer_block_m_for(cfg.T, cfg.K, cfg.N, cfg.E, cfg.topk, cfg.group)
    say(f"route + align on {name} (T={cfg.T}, block_m={block_m})")
    logits, bias = config_logits(cfg)
    ids, w, tables = run_route_align(logits, bias, cfg.topk, block_m)
    ids_o, w_o = O.route_topk(logits, cfg.topk, bias=bias)
    np.testing.assert_array_equal(ids, ids_o)
    assert np.max(np.abs(w.astype(np.float64) - w_o)) <= W_ATOL
    U.assert_align_equal(tables, O.align_by_expert(ids_o, cfg.E, block_m), block_m)


@pytest.mark.parametrize("T,E,topk,block_m,with_bias", [
    (1, 8, 2, 16, False), (63, 100, 5, 32, True), (64, 256, 8, 16, False), (65, 256, 8, 16, False),
    (50, 256, 16, 16, True), (50, 256, 17, 32, False), (33, 257, 8, 16, False),      # 16-lane rows / whole-wave routing
    (60, 1024, 64, 64, False), (300, 1024, 64, 64, False), (40, 1, 1, 256, False), (0, 4, 2, 16, False),
])
def test_route_align_edges(T, E, topk, block_m, with_bias):
    say(f"route + align T={T} E={E} topk={topk} block_m={block_m} bias={with_bias}")
    rng = np.random.default_rng(2000 + T + E)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    if T > 2:
        logits[1, :] = 0.25                                # an all-tie row
    bias = skew_bias(E) if with_bias else None
    ids, w, tables = run_route_align(logits, bias, topk, block_m)
    if T == 0:
        assert tables["num_padded"].item() == 0
        return
    ids_o, w_o = O.route_topk(logits, topk, bias=bias)
    np.testing.assert_array_equal(ids, ids_o)
    assert np.max(np.abs(w.astype(np.float64) - w_o)) <= W_ATOL
    U.assert_align_equal(tables, O.align_by_expert(ids_o, E, block_m), block_m)


def test_router_error_paths():
    say("router errors")
    ld = torch.zeros((4, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(M.MoEError) as e:                   # topk > E
        M.moe_route_topk(ld, None, torch.zeros((4, 9), dtype=torch.int32, device="cuda"),
                         torch.zeros((4, 9), dtype=torch.float32, device="cuda"))
    assert e.value.status == 2
    with pytest.raises(M.MoEError) as e:                   # topk == 0
        M.moe_route_topk(ld, None, torch.zeros((4, 0), dtype=torch.int32, device="cuda"),
                         torch.zeros((4, 0), dtype=torch.float32, device="cuda"))
    assert e.value.status == 1
    big = torch.zeros((1, 1025), dtype=torch.float32, device="cuda")
    with pytest.raises(M.MoEError) as e:                   # E > 1024
        M.moe_route_topk(big, None, torch.zeros((1, 2), dtype=torch.int32, device="cuda"),
                         torch.zeros((1, 2), dtype=torch.float32, device="cuda"))
    assert e.value.status == 2


def test_router_feeds_the_layer():
    """Router output used directly as the layer's routing input equals the oracle chain."""
    cfg = MoEConfig("routed", T=40, K=256, N=128, E=12, topk=3, group=128, dtype="f16", seed=31)
    say(f"router + layer {cfg}")
    inp = make_inputs(cfg)
    d = U.DevInputs(inp)
    ld = torch.from_numpy(inp.logits).cuda()
    ids = torch.empty((cfg.T, cfg.topk), dtype=torch.int32, device="cuda")
    w = torch.empty((cfg.T, cfg.topk), dtype=torch.float32, device="cuda")
    M.moe_route_topk(ld, None, ids, w)
    d.ids, d.w = ids, w
    out = U.run_layer(d)
    ids_o, w_o = O.route_topk(inp.logits, cfg.topk)
    want = O.layer(O.decode_bits(inp.x_bits, "f16"), ids_o, w_o.astype(np.float32), inp.qw1,
                   O.decode_bits(inp.s1_bits, "f16"), inp.z1, inp.qw2, O.decode_bits(inp.s2_bits, "f16"), inp.z2,
                   cfg.group, "f16")
    U.assert_close(U.dev_to_f64(out), want, "routed layer")


@pytest.mark.parametrize("name,dtype,with_bias", [("a", "f16", False), ("b", "bf16", True)])
def test_routed_layer_entry_point(name, dtype, with_bias):
    """Router and layer behind one call (routing tables in the workspace) against the oracle chain."""
    cfg = MoEConfig("routed_" + name, T=33, K=256, N=256, E=10, topk=4, group=64, dtype=dtype, seed=51)
    say(f"routed layer {cfg} bias={with_bias}")
    inp = make_inputs(cfg)
    d = U.DevInputs(inp)
    bias = skew_bias(cfg.E) if with_bias else None
    ld = torch.from_numpy(inp.logits).cuda()
    bd = None if bias is None else torch.from_numpy(bias).cuda()
    mdt = M.MOE_F16 if dtype == "f16" else M.MOE_BF16
    ws = torch.empty(M.moe_w4a16_routed_layer_workspace_bytes(cfg.T, cfg.K, cfg.N, cfg.E, cfg.topk, mdt),
                     dtype=torch.uint8, device="cuda")
    out = torch.full((cfg.T, cfg.K), float("nan"), dtype=U.TORCH_DT[dtype], device="cuda")
    M.moe_w4a16_routed_layer(d.X, ld, bd, d.qw1, d.s1, d.z1, d.qw2, d.s2, d.z2, out, cfg.topk, cfg.group, ws)
    torch.cuda.synchronize()
    ids_o, w_o = O.route_topk(inp.logits, cfg.topk, bias=bias)
    want = O.layer(O.decode_bits(inp.x_bits, dtype), ids_o, w_o.astype(np.float32), inp.qw1,
                   O.decode_bits(inp.s1_bits, dtype), inp.z1, inp.qw2, O.decode_bits(inp.s2_bits, dtype), inp.z2,
                   cfg.group, dtype)
    U.assert_close(U.dev_to_f64(out), want, "routed layer entry point")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(M.MoEError) as e:
        M.moe_w4a16_routed_layer(d.X, ld, bd, d.qw1, d.s1, d.z1, d.qw2, d.s2, d.z2, out, cfg.topk, cfg.group, small)
    assert e.value.status == 3


# ------------------------------------------------------------------ dense GEMM
@pytest.mark.parametrize("M_rows,N,K,group,dtype", [
    (1, 256, 128, 128, "f16"), (16, 320, 224, 32, "f16"), (17, 256, 1024, 128, "f16"), (50, 768, 1024, 128, "bf16"),
    (200, 512, 2048, 128, "f16"), (33, 128, 512, 64, "bf16"), (128, 1024, 1024, 128, "f16"),
])
def test_dense_gemm_matches_oracle(M_rows, N, K, group, dtype):
    say(f"dense gemm M={M_rows} N={N} K={K} g={group} {dtype}")
    cfg = MoEConfig("dense", T=M_rows, K=K, N=N // 2, E=1, topk=1, group=group, dtype=dtype, seed=40 + M_rows)
    inp = make_inputs(cfg)                                  # W1 of the single expert is [N, K]
    d = U.DevInputs(inp)
    C = torch.full((M_rows, N), float("nan"), dtype=U.TORCH_DT[dtype], device="cuda")
    M.moe_w4a16_dense_gemm(d.X, d.qw1[0], d.s1[0], d.z1[0], group, C)
    torch.cuda.synchronize()
    want = O.dense_gemm(O.decode_bits(inp.x_bits, dtype), inp.qw1[0], O.decode_bits(inp.s1_bits[0], dtype),
                        inp.z1[0], group, dtype)
    U.assert_close(U.dev_to_f64(C), want, "dense gemm")


def test_dense_gemm_equals_grouped_gemm_with_one_expert_bitwise():
    cfg = MoEConfig("dense_eq", T=70, K=1024, N=384, E=1, topk=1, group=128, dtype="f16", seed=44)
    say(f"dense vs grouped {cfg}")
    inp = make_inputs(cfg)
    d = U.DevInputs(inp)
    C1 = torch.zeros((cfg.T, 2 * cfg.N), dtype=torch.float16, device="cuda")
    C2 = torch.zeros_like(C1)
    M.moe_w4a16_dense_gemm(d.X, d.qw1[0], d.s1[0], d.z1[0], cfg.group, C1)
    al = U.run_align(d.ids, 1, 64)
    M.moe_w4a16_grouped_gemm(d.X, 1, d.qw1, d.s1, d.z1, al["sorted_slot_ids"], al["block_expert_ids"],
                             al["num_padded"], cfg.T, cfg.group, 64, C2)
    torch.cuda.synchronize()
    assert torch.equal(C1, C2)


def test_dense_gemm_empty_and_errors():
    say("dense gemm M=0 / bad shape")
    cfg = MoEConfig("dense0", T=4, K=128, N=128, E=1, topk=1, group=128, dtype="f16", seed=45)
    d = U.DevInputs(make_inputs(cfg))
    C = torch.zeros((0, 256), dtype=torch.float16, device="cuda")
    M.moe_w4a16_dense_gemm(d.X[:0], d.qw1[0], d.s1[0], d.z1[0], 128, C)
    with pytest.raises(M.MoEError) as e:
        M.moe_w4a16_dense_gemm(d.X, d.qw1[0], d.s1[0], d.z1[0], 48, torch.zeros((4, 256), dtype=torch.float16, device="cuda"))
    assert e.value.status == 2


def test_roof_probes_run():
    say("roof probes")
    src = torch.ones(1 << 24, dtype=torch.int32, device="cuda")       # 64 MiB
    sink = torch.zeros(1 << 18, dtype=torch.int32, device="cuda")     # 1 MiB
    M.moe_probe_stream_read(src, sink)
    M.moe_probe_mfma(sink, 100)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ operand-order (prepacked) weights
@pytest.mark.parametrize("E,N_out,K,paired", [(1, 16, 128, False), (3, 96, 384, False), (2, 64, 1024, True),
                                              (5, 352, 256, True), (2, 2048, 2048, False)])
def test_repack_matches_oracle_permutation(E, N_out, K, paired):
    say(f"repack E={E} N_out={N_out} K={K} paired={paired}")
    rng = np.random.default_rng(60 + N_out)
    q = rng.integers(0, 2 ** 32, size=(E, N_out, K // 8), dtype=np.uint32).view(np.int32)
    qd = torch.from_numpy(q).cuda()
    out = torch.full_like(qd, -1)
    M.moe_repack_qweight(qd, paired, out)
    torch.cuda.synchronize()
    want = O.repack_qweight(q, paired).reshape(E, N_out, K // 8)
    np.testing.assert_array_equal(out.cpu().numpy(), want)


def _prepacked(d):
    p1, p2 = torch.empty_like(d.qw1), torch.empty_like(d.qw2)
    M.moe_repack_qweight(d.qw1, False, p1)
    M.moe_repack_qweight(d.qw2, True, p2)
    return p1, p2


@pytest.mark.parametrize("tile", [(1, 2), (2, 2), (4, 2), (4, 4)])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_prepacked_layer_equals_layer_bitwise(tile, dtype):
    """Same operand words in the same order: the layer on repacked weights must reproduce the
    layer on the original tensors bit for bit, and both sit within the bound of the oracle."""
    cfg = MoEConfig("pre", T=40, K=1024, N=1024, E=5, topk=2, group=128, dtype=dtype, seed=61)
    say(f"prepacked layer tile={tile} {cfg}")
    inp = make_inputs(cfg)
    d = U.DevInputs(inp)
    p1, p2 = _prepacked(d)
    mdt = M.MOE_F16 if dtype == "f16" else M.MOE_BF16
    ws = torch.empty(M.moe_w4a16_layer_workspace_bytes(cfg.T, cfg.K, cfg.N, cfg.E, cfg.topk, mdt),
                     dtype=torch.uint8, device="cuda")
    out_a = torch.full((cfg.T, cfg.K), float("nan"), dtype=U.TORCH_DT[dtype], device="cuda")
    out_b = torch.full_like(out_a, float("nan"))
    M.moe_set_tile_override(*tile)
    try:
        M.moe_w4a16_layer(d.X, d.ids, d.w, d.qw1, d.s1, d.z1, d.qw2, d.s2, d.z2, out_a, cfg.group, ws)
        M.moe_w4a16_layer_prepacked(d.X, d.ids, d.w, p1, d.s1, d.z1, p2, d.s2, d.z2, out_b, cfg.group, ws)
        torch.cuda.synchronize()
    finally:
        M.moe_set_tile_override(0, 0)
    assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16))
    want = O.layer(O.decode_bits(inp.x_bits, dtype), inp.topk_ids, inp.topk_weights, inp.qw1,
                   O.decode_bits(inp.s1_bits, dtype), inp.z1, inp.qw2, O.decode_bits(inp.s2_bits, dtype), inp.z2,
                   cfg.group, dtype)
    U.assert_close(U.dev_to_f64(out_b), want, "prepacked layer")


@pytest.mark.parametrize("T,K,N,E,topk,splits", [(20, 1024, 3072, 3, 2, 2), (130, 2048, 1024, 7, 3, 0), (9, 1024, 2048, 40, 4, 3)])
def test_prepacked_layer_shapes_and_splits(T, K, N, E, topk, splits):
    cfg = MoEConfig("pre_s", T=T, K=K, N=N, E=E, topk=topk, group=128, dtype="f16", seed=62)
    say(f"prepacked layer shapes {cfg} splits={splits}")
    inp = make_inputs(cfg)
    d = U.DevInputs(inp)
    p1, p2 = _prepacked(d)
    ws = torch.empty(M.moe_w4a16_layer_workspace_bytes(T, K, N, E, topk, M.MOE_F16), dtype=torch.uint8, device="cuda")
    out = torch.full((T, K), float("nan"), dtype=torch.float16, device="cuda")
    M.moe_set_reduction_splits(splits)
    try:
        M.moe_w4a16_layer_prepacked(d.X, d.ids, d.w, p1, d.s1, d.z1, p2, d.s2, d.z2, out, cfg.group, ws)
        torch.cuda.synchronize()
    finally:
        M.moe_set_reduction_splits(0)
    want = O.layer(O.decode_bits(inp.x_bits, "f16"), inp.topk_ids, inp.topk_weights, inp.qw1,
                   O.decode_bits(inp.s1_bits, "f16"), inp.z1, inp.qw2, O.decode_bits(inp.s2_bits, "f16"), inp.z2,
                   cfg.group, "f16")
    U.assert_close(U.dev_to_f64(out), want, "prepacked layer shapes")


def test_prepacked_layer_rejects_other_group_sizes():
    cfg = MoEConfig("pre_bad", T=8, K=1024, N=1024, E=2, topk=1, group=64, dtype="f16", seed=63)
    say(f"prepacked layer unsupported {cfg}")
    d = U.DevInputs(make_inputs(cfg))
    ws = torch.empty(M.moe_w4a16_layer_workspace_bytes(8, 1024, 1024, 2, 1, M.MOE_F16), dtype=torch.uint8, device="cuda")
    out = torch.zeros((8, 1024), dtype=torch.float16, device="cuda")
    with pytest.raises(M.MoEError) as e:
        M.moe_w4a16_layer_prepacked(d.X, d.ids, d.w, d.qw1, d.s1, d.z1, d.qw2, d.s2, d.z2, out, 64, ws)
    assert e.value.status == 2


def test_layer_is_graph_capturable_and_replays_identically():
    """The layer allocates nothing, never synchronises and launches only on the given stream, so
    it can be recorded into a HIP graph; every replay (with eager work and synchronisations in
    between) must reproduce the eager result bit for bit."""
    cfg = MoEConfig("graph", T=24, K=1024, N=1024, E=6, topk=2, group=128, dtype="f16", seed=71)
    say(f"graph capture {cfg}")
    inp = make_inputs(cfg)
    d = U.DevInputs(inp)
    ws = torch.empty(M.moe_w4a16_layer_workspace_bytes(cfg.T, cfg.K, cfg.N, cfg.E, cfg.topk, M.MOE_F16),
                     dtype=torch.uint8, device="cuda")
    eager = torch.full((cfg.T, cfg.K), float("nan"), dtype=torch.float16, device="cuda")
    M.moe_w4a16_layer(d.X, d.ids, d.w, d.qw1, d.s1, d.z1, d.qw2, d.s2, d.z2, eager, cfg.group, ws)
    torch.cuda.synchronize()
    out = torch.zeros_like(eager)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        M.moe_w4a16_layer(d.X, d.ids, d.w, d.qw1, d.s1, d.z1, d.qw2, d.s2, d.z2, out, cfg.group, ws)   # warm-up on the side stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            M.moe_w4a16_layer(d.X, d.ids, d.w, d.qw1, d.s1, d.z1, d.qw2, d.s2, d.z2, out, cfg.group, ws, stream=side)
    for rep in range(3):
        out.fill_(float("nan"))
        ws.random_(0, 255)                      # scratch contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {rep}"
        junk = torch.randn(1 << 16, device="cuda").sum().item()      # eager work between replays
        assert junk == junk
