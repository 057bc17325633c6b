"""GPU parity of the blockwise-scaled FP8 GEMM against the CPU oracle.

Bound, per output element (derived from the arithmetic, not tuned to pass):
    |gpu - oracle| <= 2^-7 |oracle|  +  2^-10 * sum_kb a_scale[m,kb] b_scale[n/128,kb] amaxA[m,kb] amaxB[n,kb]
* first term: one unit in the last place of the 16-bit result (8 significant bits for bf16; fp16
  is finer) -- a near-tie that the float32 and the float64 sums round to different neighbours;
* second term: the matrix instruction sums the 128 exact products of a block with its own
  internal alignment, not in full float32: measured on uniformly random codes (the test with
  float32 output below), the error of one block sum reaches 2^-11.1 of the block's largest product
  over 16384 outputs (median 2^-14.4) -- what truncating each of the 128 products some 18 bits
  below the largest one would give, whose worst case is 2^-10 of the largest product.  The bound
  takes 2^-10 of the largest POSSIBLE product of the block (amaxA * amaxB >= the largest actual
  one); the float32 scale product and the K/128-term float32 accumulation (2^-24 each) vanish
  next to it.
For the benchmark's inputs the second term is about half a bf16 ulp of a typical output."""
from __future__ import annotations

import json
import os
import sys

import numpy as np
import pytest
import torch

from moe_workloads.fp8 import FP8_CONFIGS, Fp8GemmConfig, make_fp8_inputs
from oracle import fp8_oracle as F
from oracle import moe_oracle as O

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2504_16214_amd as M_


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def error_bound(want, a_codes, a_scale, b_codes, b_scale):
    A = np.abs(F.decode_e4m3(a_codes))
    B = np.abs(F.decode_e4m3(b_codes))
    Mr, K = A.shape
    N = B.shape[0]
    KB = K // 128
    amaxA = A.reshape(Mr, KB, 128).max(axis=2) * a_scale.astype(np.float64)            # [M, KB]
    sb_rows = np.repeat(b_scale.astype(np.float64), 128, axis=0)[:N]                     # [N, KB]
    amaxB = B.reshape(N, KB, 128).max(axis=2) * sb_rows                                  # [N, KB]
    return 2.0 ** -7 * np.abs(want) + 2.0 ** -10 * (amaxA @ amaxB.T)


def run_gemm(a_codes, a_scale, b_codes, b_scale, dtype=torch.bfloat16):
    Mr, K = a_codes.shape
    N = b_codes.shape[0]
    A = torch.from_numpy(a_codes).cuda()
    B = torch.from_numpy(b_codes).cuda()
    sa = torch.from_numpy(a_scale).cuda()
    sb = torch.from_numpy(b_scale).cuda()
    C = torch.full((Mr, N), float("nan"), dtype=dtype, device="cuda")
    nbytes = M_.fp8_blockwise_gemm_workspace_bytes(Mr, N, K)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda") if nbytes else None
    M_.fp8_blockwise_gemm(A, sa, B, sb, C, ws)
    torch.cuda.synchronize()
    return C.to(torch.float64).cpu().numpy()


def check(inp, dtype=torch.bfloat16, what=""):
    got = run_gemm(inp.a_codes, inp.a_scale, inp.b_codes, inp.b_scale, dtype)
    want = F.blockwise_gemm(inp.a_codes, inp.a_scale, inp.b_codes, inp.b_scale,
                            "bf16" if dtype == torch.bfloat16 else "f16")
    bound = error_bound(want, inp.a_codes, inp.a_scale, inp.b_codes, inp.b_scale)
    err = np.abs(got - want)
    assert not np.isnan(got).any(), f"{what}: NaN in the output"
    worst = float((err / bound).max())
    say(f"{what}: max err / bound = {worst:.3f}, max |want| = {np.abs(want).max():.3g}")
    assert worst <= 1.0, f"{what}: {int((err > bound).sum())} of {err.size} outside the bound"


@pytest.mark.parametrize("mt,nt,splits", [(mt, nt, sp) for mt in (1, 2, 4, 8) for nt in (1, 2, 4) for sp in (1, 3)]
                         + [(16, 4, 1), (16, 4, 3), (16, 2, 1), (16, 2, 2)])
def test_every_tile_variant_matches_oracle(mt, nt, splits):
    """Each compiled tile, with and without a split reduction, on a shape with two row blocks (the
    second one ragged), two feature blocks and an odd number of reduction blocks."""
    Mr = 16 * mt + 5
    cfg = Fp8GemmConfig(f"v{mt}{nt}{splits}", M=Mr, N=2 * 64 * nt, K=128 * 7, seed=100 + 10 * mt + nt)
    say(f"fp8 gemm tile ({mt},{nt}) splits {splits} M={cfg.M} N={cfg.N} K={cfg.K}")
    inp = make_fp8_inputs(cfg)
    M_.fp8_set_plan_override(mt, nt, splits, 3)
    try:
        check(inp, what=f"tile ({mt},{nt}) splits {splits}")
    finally:
        M_.fp8_set_plan_override(0, 0, 0, 0)


@pytest.mark.parametrize("Mr,N,K", [(1, 64, 128), (16, 192, 384), (17, 576, 256), (37, 192, 384), (64, 1024, 1024),
                                    (100, 320, 640), (130, 2048, 512), (300, 1280, 1152)])
def test_default_plan_matches_oracle(Mr, N, K):
    say(f"fp8 gemm default plan M={Mr} N={N} K={K}")
    check(make_fp8_inputs(Fp8GemmConfig("d", M=Mr, N=N, K=K, seed=Mr + N)), what=f"M={Mr} N={N} K={K}")


def test_fp16_output():
    say("fp8 gemm fp16 output")
    check(make_fp8_inputs(Fp8GemmConfig("h", M=40, N=256, K=512, seed=9)), dtype=torch.float16, what="fp16 out")


def test_uniform_random_codes_and_wide_scales():
    """Every non-NaN code equally likely (the widest dynamic range a block can have) and scales
    over four decades."""
    rng = np.random.default_rng(12)
    Mr, N, K = 33, 256, 640
    a = rng.integers(0, 256, size=(Mr, K), dtype=np.uint8); a[(a & 0x7F) == 0x7F] = 0x38
    b = rng.integers(0, 256, size=(N, K), dtype=np.uint8); b[(b & 0x7F) == 0x7F] = 0xB8
    sa = np.exp(rng.uniform(np.log(1e-4), np.log(1.0), size=(Mr, K // 128))).astype(np.float32)
    sb = np.exp(rng.uniform(np.log(1e-4), np.log(1.0), size=(N // 128, K // 128))).astype(np.float32)
    say(f"fp8 gemm uniform codes M={Mr} N={N} K={K}")
    got = run_gemm(a, sa, b, sb)
    want = F.blockwise_gemm(a, sa, b, sb)
    bound = error_bound(want, a, sa, b, sb)
    worst = float((np.abs(got - want) / bound).max())
    say(f"uniform codes: max err / bound = {worst:.3f}")
    assert worst <= 1.0


@pytest.mark.parametrize("name", ["fp8_qkv_decode", "fp8_down_decode", "fp8_gateup_decode", "fp8_qkv_prefill"])
def test_benchmark_shapes_sampled(name):
    """Full-size launches in the benchmark's configuration; the oracle recomputes sampled
    128-row blocks of B (whole scale blocks) against sampled rows of A."""
    cfg = FP8_CONFIGS[name]
    say(f"fp8 gemm {name} M={cfg.M} N={cfg.N} K={cfg.K} (sampled)")
    inp = make_fp8_inputs(cfg)
    got = run_gemm(inp.a_codes, inp.a_scale, inp.b_codes, inp.b_scale)
    rng = np.random.default_rng(1)
    rows = np.sort(rng.choice(cfg.M, size=min(cfg.M, 24), replace=False))
    rows[-1] = cfg.M - 1
    blocks = np.sort(rng.choice(cfg.N // 128, size=3, replace=False))
    blocks[-1] = cfg.N // 128 - 1
    cols = np.concatenate([np.arange(128 * b, 128 * b + 128) for b in blocks])
    want = F.blockwise_gemm(inp.a_codes[rows], inp.a_scale[rows], inp.b_codes[cols], inp.b_scale[blocks])
    bound = error_bound(want, inp.a_codes[rows], inp.a_scale[rows], inp.b_codes[cols], inp.b_scale[blocks])
    sub = got[np.ix_(rows, cols)]
    assert not np.isnan(got).any()
    worst = float((np.abs(sub - want) / bound).max())
    say(f"{name}: max err / bound = {worst:.3f} on {sub.size} sampled outputs")
    assert worst <= 1.0


def test_matches_golden_fixture():
    with open(os.path.join(os.path.dirname(__file__), "golden", "small_fp8_gemm.json")) as f:
        doc = json.load(f)
    c = doc["config"]
    say(f"fp8 gemm golden M={c['M']} N={c['N']} K={c['K']}")
    inp = make_fp8_inputs(Fp8GemmConfig("golden_fp8", M=c["M"], N=c["N"], K=c["K"], seed=c["seed"]))
    got = run_gemm(inp.a_codes, inp.a_scale, inp.b_codes, inp.b_scale)
    want = O.decode_bits(np.array(doc["out_bits"], np.uint16), "bf16")
    bound = error_bound(want, inp.a_codes, inp.a_scale, inp.b_codes, inp.b_scale)
    assert float((np.abs(got - want) / bound).max()) <= 1.0


def test_empty_and_error_paths():
    say("fp8 gemm M=0 / errors")
    inp = make_fp8_inputs(Fp8GemmConfig("e", M=4, N=128, K=256, seed=2))
    A, B = torch.from_numpy(inp.a_codes).cuda(), torch.from_numpy(inp.b_codes).cuda()
    sa, sb = torch.from_numpy(inp.a_scale).cuda(), torch.from_numpy(inp.b_scale).cuda()
    M_.fp8_blockwise_gemm(A[:0], sa[:0], B, sb, torch.empty((0, 128), dtype=torch.bfloat16, device="cuda"))
    lib = M_.load_library()
    C = torch.empty((4, 128), dtype=torch.bfloat16, device="cuda")
    p = lambda t: t.data_ptr()
    assert lib.fp8_blockwise_gemm(p(A), p(sa), p(B), p(sb), p(C), 4, 128, 200, 1, None, 0, None) == 2     # K % 128
    assert lib.fp8_blockwise_gemm(p(A), p(sa), p(B), p(sb), p(C), 4, 100, 256, 1, None, 0, None) == 2     # N % 64
    assert lib.fp8_blockwise_gemm(None, p(sa), p(B), p(sb), p(C), 4, 128, 256, 1, None, 0, None) == 1
    assert lib.fp8_blockwise_gemm(p(A), p(sa), p(B), p(sb), p(C), 4, 128, 256, 7, None, 0, None) == 1      # dtype
    M_.fp8_set_plan_override(1, 1, 2, 0)
    try:
        assert M_.fp8_blockwise_gemm_workspace_bytes(4, 128, 256) == 2 * 4 * 128 * 4
        assert lib.fp8_blockwise_gemm(p(A), p(sa), p(B), p(sb), p(C), 4, 128, 256, 1, None, 0, None) == 3  # workspace
    finally:
        M_.fp8_set_plan_override(0, 0, 0, 0)


def test_mfma_probe_runs():
    say("fp8 mfma probe")
    sink = torch.zeros(512 * 256, dtype=torch.float32, device="cuda")
    M_.fp8_probe_mfma(sink, 64)
    torch.cuda.synchronize()
    assert torch.isfinite(sink).all()


# ------------------------------------------------------------------ grouped (one matrix per expert)
def _grouped_case(T, topk, E, N, K, row_div_is_topk, seed, bad_ids=False):
    """Seeded routed workload: random expert ids (optionally with ignored ids), activations and E
    weight matrices quantised by the generator's recipe."""
    rng = np.random.default_rng(seed)
    ids = rng.integers(0, E, size=(T, topk)).astype(np.int32)
    if bad_ids:
        ids[0, 0] = -1
        ids[T - 1, topk - 1] = E + 3
    rows = T if row_div_is_topk else T * topk
    a = make_fp8_inputs(Fp8GemmConfig("ga", M=rows, N=128, K=K, seed=seed))
    ws = [make_fp8_inputs(Fp8GemmConfig("gb", M=1, N=N, K=K, seed=seed + 1 + e)) for e in range(E)]
    b = np.stack([w.b_codes for w in ws])
    sb = np.stack([w.b_scale for w in ws])
    return ids, a.a_codes, a.a_scale, b, sb


@pytest.mark.parametrize("T,topk,E,N,K,block_m,row_div_is_topk,bad_ids", [
    (5, 2, 3, 128, 256, 16, True, False),          # tiny
    (40, 2, 4, 192, 384, 16, True, True),          # N % 128 != 0 (64-feature tiles), ignored ids
    (64, 4, 8, 256, 512, 32, False, False),        # A already per slot (row_div 1)
    (300, 2, 5, 256, 384, 64, True, True),         # several row blocks per expert, ragged last ones
    (700, 1, 3, 384, 256, 128, True, False),       # 128-slot tiles
    (900, 2, 2, 256, 256, 256, False, False),      # 256-slot eight-wave tile
])
def test_grouped_gemm_matches_oracle(T, topk, E, N, K, block_m, row_div_is_topk, bad_ids):
    import gpu_util as U
    say(f"fp8 grouped gemm T={T} topk={topk} E={E} N={N} K={K} block_m={block_m} row_div={'topk' if row_div_is_topk else 1}")
    ids, a, sa, b, sb = _grouped_case(T, topk, E, N, K, row_div_is_topk, seed=500 + T + block_m, bad_ids=bad_ids)
    row_div = topk if row_div_is_topk else 1
    S = T * topk
    al = U.run_align(torch.from_numpy(ids).cuda(), E, block_m)
    C = torch.full((S, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    M_.fp8_moe_grouped_gemm(torch.from_numpy(a).cuda(), torch.from_numpy(sa).cuda(), row_div,
                            torch.from_numpy(b).cuda(), torch.from_numpy(sb).cuda(),
                            al["sorted_slot_ids"], al["block_expert_ids"], al["num_padded"], S, block_m, C)
    torch.cuda.synchronize()
    got = C.to(torch.float64).cpu().numpy()
    want, valid = F.grouped_blockwise_gemm(a, sa, row_div, b, sb, ids.reshape(-1))
    assert np.isnan(got[~valid]).all(), "rows of ignored slots must stay untouched"
    assert not np.isnan(got[valid]).any()
    worst = 0.0
    flat = ids.reshape(-1)
    for e in range(E):
        slots = np.nonzero(flat == e)[0]
        if slots.size == 0:
            continue
        rows = slots // row_div
        bound = error_bound(want[slots], a[rows], sa[rows], b[e], sb[e])
        worst = max(worst, float((np.abs(got[slots] - want[slots]) / bound).max()))
    say(f"grouped: max err / bound = {worst:.3f}")
    assert worst <= 1.0


def test_grouped_gemm_one_expert_equals_dense_bitwise():
    import gpu_util as U
    say("fp8 grouped gemm, one expert == dense")
    inp = make_fp8_inputs(Fp8GemmConfig("g1", M=70, N=256, K=512, seed=77))
    A, B = torch.from_numpy(inp.a_codes).cuda(), torch.from_numpy(inp.b_codes).cuda()
    sa, sb = torch.from_numpy(inp.a_scale).cuda(), torch.from_numpy(inp.b_scale).cuda()
    C1 = torch.zeros((70, 256), dtype=torch.bfloat16, device="cuda")
    C2 = torch.zeros_like(C1)
    M_.fp8_set_plan_override(4, 2, 1, 0)                       # the tile the grouped call uses at block_m 64
    try:
        M_.fp8_blockwise_gemm(A, sa, B, sb, C1, None)
    finally:
        M_.fp8_set_plan_override(0, 0, 0, 0)
    al = U.run_align(torch.zeros((70, 1), dtype=torch.int32, device="cuda"), 1, 64)
    M_.fp8_moe_grouped_gemm(A, sa, 1, B[None].contiguous(), sb[None].contiguous(), al["sorted_slot_ids"],
                            al["block_expert_ids"], al["num_padded"], 70, 64, C2)
    torch.cuda.synchronize()
    assert torch.equal(C1, C2)


def test_grouped_gemm_empty_and_errors():
    say("fp8 grouped gemm: no slots / errors")
    lib = M_.load_library()
    p = 0x10000
    assert lib.fp8_moe_grouped_gemm(None, None, 1, None, None, None, None, None, 0, 4, 128, 256, 16, 1, None, None) == 0
    assert lib.fp8_moe_grouped_gemm(p, p, 1, p, p, p, p, p, 8, 4, 128, 200, 16, 1, 2 * p, None) == 2      # K % 128
    assert lib.fp8_moe_grouped_gemm(p, p, 1, p, p, p, p, p, 8, 4, 128, 256, 24, 1, 2 * p, None) == 1      # block_m
    assert lib.fp8_moe_grouped_gemm(p, p, 0, p, p, p, p, p, 8, 4, 128, 256, 16, 1, 2 * p, None) == 1      # row_div
    assert lib.fp8_moe_grouped_gemm(p, p, 1, p, p, None, p, p, 8, 4, 128, 256, 16, 1, 2 * p, None) == 1   # null table


# ------------------------------------------------------------------ float32 output: the accumulator itself
def test_float32_output_and_the_block_sum_error_of_the_matrix_instruction():
    """With float32 output and unit scales a single reduction block shows the matrix instruction's
    own summation error: uniformly random codes (the widest dynamic range a block can have), exact
    float64 block sums from the oracle.  Observed: up to 2^-11.1 of the block's largest product
    (median 2^-14.4); the parity bound of this file allows 2^-10 of the largest possible product.
    A float32-exact summation would sit near 2^-24 * 128 = 2^-17."""
    rng = np.random.default_rng(99)
    Mr, N, K = 64, 256, 128
    a = rng.integers(0, 256, size=(Mr, K), dtype=np.uint8); a[(a & 0x7F) == 0x7F] = 0x38
    b = rng.integers(0, 256, size=(N, K), dtype=np.uint8); b[(b & 0x7F) == 0x7F] = 0xB8
    ones_a, ones_b = np.ones((Mr, 1), np.float32), np.ones((N // 128, 1), np.float32)
    say(f"fp8 gemm float32 output, one block, M={Mr} N={N}")
    got = run_gemm(a, ones_a, b, ones_b, dtype=torch.float32)
    want = F.blockwise_gemm(a, ones_a, b, ones_b, out_dt=None)
    A, B = np.abs(F.decode_e4m3(a)), np.abs(F.decode_e4m3(b))
    maxprod = (A[:, None, :] * B[None, :, :]).max(axis=2)                 # largest |a_k b_k| per output
    rel = np.abs(got - want) / maxprod
    say(f"block-sum error of the matrix instruction: max = 2^{np.log2(rel.max()):.1f} of the largest product, "
        f"median = 2^{np.log2(np.median(rel[rel > 0])):.1f}")
    assert rel.max() <= 2.0 ** -10


@pytest.mark.parametrize("splits", [1, 3])
def test_float32_output_matches_unrounded_oracle(splits):
    cfg = Fp8GemmConfig("f32", M=45, N=256, K=896, seed=61)
    say(f"fp8 gemm float32 output, splits {splits}")
    inp = make_fp8_inputs(cfg)
    M_.fp8_set_plan_override(2, 2, splits, 0)
    try:
        got = run_gemm(inp.a_codes, inp.a_scale, inp.b_codes, inp.b_scale, dtype=torch.float32)
    finally:
        M_.fp8_set_plan_override(0, 0, 0, 0)
    want = F.blockwise_gemm(inp.a_codes, inp.a_scale, inp.b_codes, inp.b_scale, out_dt=None)
    # no 16-bit rounding: only the block-sum term of the bound (and float32 accumulation, 2^-22 with room)
    bound = error_bound(np.zeros_like(want), inp.a_codes, inp.a_scale, inp.b_codes, inp.b_scale) + 2.0 ** -22 * np.abs(want)
    worst = float((np.abs(got - want) / bound).max())
    say(f"float32 out: max err / bound = {worst:.3f}")
    assert worst <= 1.0


def test_gemm_with_split_reduction_is_graph_capturable():
    """Nothing is allocated, nothing synchronises and both kernels go to the given stream, so the
    call (GEMM into float32 planes + plane reduction) can be recorded into a HIP graph; every replay,
    with eager work and synchronisations in between and with the workspace overwritten, equals the
    eager result bit for bit."""
    cfg = Fp8GemmConfig("graph", M=24, N=1024, K=2048, seed=71)
    say(f"fp8 gemm graph capture {cfg}")
    inp = make_fp8_inputs(cfg)
    A, B = torch.from_numpy(inp.a_codes).cuda(), torch.from_numpy(inp.b_codes).cuda()
    sa, sb = torch.from_numpy(inp.a_scale).cuda(), torch.from_numpy(inp.b_scale).cuda()
    nbytes = M_.fp8_blockwise_gemm_workspace_bytes(cfg.M, cfg.N, cfg.K)
    assert nbytes > 0, "the shape is meant to take the split-reduction path"
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    eager = torch.full((cfg.M, cfg.N), float("nan"), dtype=torch.bfloat16, device="cuda")
    M_.fp8_blockwise_gemm(A, sa, B, sb, eager, ws)
    torch.cuda.synchronize()
    out = torch.zeros_like(eager)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        M_.fp8_blockwise_gemm(A, sa, B, sb, out, ws)                       # warm-up on the side stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            M_.fp8_blockwise_gemm(A, sa, B, sb, out, ws, stream=side)
    for rep in range(3):
        out.fill_(float("nan"))
        ws.random_(0, 255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {rep}"
        junk = torch.randn(1 << 16, device="cuda").sum().item()
        assert junk == junk
