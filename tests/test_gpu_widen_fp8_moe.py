"""GPU parity of the FP8 mixture-of-experts layer (widening: the FP8 workload family of the paper's
serving evaluation, Section VII-D, on the grouped kernel structure of Section VII-B) against the
CPU oracle, through the C ABI.

* the activation quantiser decides integer codes in float32 steps both sides take identically:
  codes and scales BIT-EXACT against the oracle, including zero tiles, subnormal codes and exact ties;
* the fused SiLU-and-multiply quantiser: bit-exact against the oracle's quantiser applied to the
  16-bit activation the staged SiLU-and-multiply kernel produces (same float32 SiLU);
* the layer: within the bound derived below.

Layer bound.  Every product of the layer is exact; the two sides differ by (a) the matrix
instruction's alignment of a 128-term block sum and float32 accumulation (bounded per output by
2^-10 of the largest possible block products, as for the FP8 GEMM), (b) a flipped 16-bit rounding
of H, act or out (one ulp = 2^-8 relative in bf16), and (c) wherever a flipped activation sits on
an e4m3 rounding boundary, one code moving by one step (at most 2^-3 of that one product).  (c) has
no useful worst case: it is bounded statistically.  With a fraction p of moved codes, the down
projection moves by about sqrt(p * N) * 2^-3 * rms(product) = sqrt(p) * 2^-3 * rms(Y); p is
measured (and asserted) below 2 %, giving 0.018 * rms(Y); the test takes about three times that
as the bound a correct output meets,
    |gpu - oracle| <= 2^-6 * |oracle| + 0.05 * rms(oracle).
Being statistical, the term has a tail: ONE moved code shifts every output of its slot by
2^-3 * |product| at worst, and where a large activation meets a large weight that is several
times 0.05 * rms(Y) (seen on random shapes at one output in 10^4 ... 10^5).  That tail has a
worst case of its own, which the test adds per output (moved_code_allowance): one e4m3 step of the
activation code, at the worst of the sixteen largest activations of each of the token's slots,
times the weight it meets.  So
    |gpu - oracle| <= 2^-6 * |oracle| + 0.05 * rms(oracle) + sum_j w_j * max_n step(aq[j, n]) * |W2[c, n]|
for every output; planted mistakes (a neighbouring scale, swapped gate/up) must leave more than a
tenth of the outputs outside the bound (measured: 86 %)."""
from __future__ import annotations

import sys

import numpy as np
import pytest
import torch

from moe_workloads.fp8 import FP8_MOE_CONFIGS, Fp8MoEConfig, make_fp8_moe_inputs
from oracle import fp8_oracle as F
from oracle import moe_oracle as O

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2504_16214_amd as M
    import gpu_util as U


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def gpu_quantize(x_vals, dt):
    X = U.vals_to_dev(x_vals, dt)
    R, K = x_vals.shape
    codes = torch.full((R, K), 0xAA, dtype=torch.uint8, device="cuda")
    scales = torch.full((R, K // 128), -1.0, dtype=torch.float32, device="cuda")
    M.fp8_quantize_rows(X, codes, scales)
    torch.cuda.synchronize()
    return codes.cpu().numpy(), scales.cpu().numpy()


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_quantize_rows_bit_exact(dt):
    say(f"fp8 quantize rows dt={dt}")
    rng = np.random.default_rng(61)
    R, K = 67, 1024
    x = O.rnd(rng.standard_normal((R, K)) * np.exp(rng.uniform(-8, 4, (R, 1))), dt)
    x[3, :128] = 0.0                                   # an all-zero tile (clamped maximum)
    x[4, 128:256] = O.rnd(rng.standard_normal(128) * 1e-6, dt)     # a tile far below the clamp
    # exact ties: maximum 448 * 2^-3, so 448 / m is a power of two and x * ratio is exact
    c = 2.0 ** -3
    x[5, 256:384] = 0.0
    x[5, 256:272] = np.array([448, 17, 19, 1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10, 7.5 * 2.0 ** -9,
                              -17, -19, 464 * 0 + 33, 35, 0.09375 + 2.0 ** -7, -0.0, 2.0 ** -9, 240]) * c
    x = O.rnd(x, dt)
    got_c, got_s = gpu_quantize(x, dt)
    want_c, want_s = F.quantize_rows(x)
    np.testing.assert_array_equal(got_s.view(np.uint32), want_s.view(np.uint32))
    bad = np.nonzero(got_c != want_c)
    assert bad[0].size == 0, (bad[0][:5], bad[1][:5], got_c[bad][:5], want_c[bad][:5], x[bad][:5])


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_silu_mul_quantize_equals_staged_silu_then_oracle_quantiser(dt):
    say(f"fp8 silu-mul quantize dt={dt}")
    rng = np.random.default_rng(62)
    S, N = 45, 384
    H = O.rnd(rng.standard_normal((S, 2 * N)) * 3.0, dt)
    H[0, :4] = [-30.0, 30.0, 0.0, -0.0]
    Hd = U.vals_to_dev(H, dt)
    act = torch.empty((S, N), dtype=U.TORCH_DT[dt], device="cuda")
    M.moe_silu_mul(Hd, act)
    codes = torch.zeros((S, N), dtype=torch.uint8, device="cuda")
    scales = torch.zeros((S, N // 128), dtype=torch.float32, device="cuda")
    M.fp8_silu_mul_quantize(Hd, codes, scales)
    torch.cuda.synchronize()
    want_c, want_s = F.quantize_rows(U.dev_to_f64(act))
    np.testing.assert_array_equal(scales.cpu().numpy().view(np.uint32), want_s.view(np.uint32))
    np.testing.assert_array_equal(codes.cpu().numpy(), want_c)
    U.assert_close(U.dev_to_f64(act), O.silu_mul(H, dt), "staged silu_mul")


def run_fp8_layer(inp, block_m=0):
    c = inp.cfg
    X = U.bits_to_dev(inp.x_bits, c.dtype)
    ids, w = U.i32(inp.topk_ids), torch.from_numpy(inp.topk_weights).cuda()
    w1, s1 = torch.from_numpy(inp.w1_codes).cuda(), torch.from_numpy(inp.w1_scale).cuda()
    w2, s2 = torch.from_numpy(inp.w2_codes).cuda(), torch.from_numpy(inp.w2_scale).cuda()
    out = torch.full((c.T, c.K), float("nan"), dtype=U.TORCH_DT[c.dtype], device="cuda")
    ws = torch.empty(max(M.fp8_moe_layer_workspace_bytes(c.T, c.K, c.N, c.E, c.topk), 256), dtype=torch.uint8, device="cuda")
    M.fp8_set_layer_block_m(block_m)
    try:
        M.fp8_moe_layer(X, ids, w, w1, s1, w2, s2, out, ws)
        torch.cuda.synchronize()
    finally:
        M.fp8_set_layer_block_m(0)
    return U.dev_to_f64(out)


def oracle_fp8_layer(inp, **kw):
    c = inp.cfg
    return F.moe_layer(O.decode_bits(inp.x_bits, c.dtype), inp.topk_ids, inp.topk_weights, inp.w1_codes, inp.w1_scale,
                       inp.w2_codes, inp.w2_scale, c.dtype, **kw)


def layer_bound(want):
    return 2.0 ** -6 * np.abs(want) + 0.05 * np.sqrt(np.mean(want ** 2))


def moved_code_allowance(inp, mid, tokens=None):
    """Per output [T', K]: one e4m3 step of an activation code, at the worst of the sixteen largest
    activations of each slot of the token, times the down-projection weight it meets, times the
    routing weight.  mid: the oracle's intermediates for the same tokens."""
    c = inp.cfg
    ids = inp.topk_ids if tokens is None else inp.topk_ids[tokens]
    w = (inp.topk_weights if tokens is None else inp.topk_weights[tokens]).astype(np.float64).reshape(-1)
    se = ids.reshape(-1)
    code = np.abs(F.decode_e4m3(mid["aq"]))                                  # [S', N] code values
    step = np.where(code >= 2.0 ** -6, 2.0 ** (np.floor(np.log2(np.maximum(code, 2.0 ** -9))) - 3), 2.0 ** -9)
    blk = np.repeat(mid["sa"].astype(np.float64), 128, axis=1)               # [S', N] tile scales
    val, step = code * blk, step * blk
    extra = np.zeros((se.size, c.K))
    row_blk = np.arange(c.K) // 128
    for s in np.nonzero((se >= 0) & (se < c.E))[0]:
        e = se[s]
        top = np.argsort(val[s])[-16:]
        W = np.abs(F.decode_e4m3(inp.w2_codes[e][:, top])) * inp.w2_scale[e].astype(np.float64)[row_blk][:, top // 128]
        extra[s] = (W * step[s, top][None, :]).max(axis=1)
    return (extra * w[:, None]).reshape(ids.shape[0], c.topk, c.K).sum(axis=1)


def assert_layer_close(got, want, what, allowance=None):
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    plain = layer_bound(want)
    err = np.abs(got - want)
    ratio = err / (plain + (0.0 if allowance is None else allowance))
    say(f"{what}: max err / bound = {ratio.max():.3f}, {int((err > plain).sum())} of {err.size} beyond the "
        f"statistical part alone, rms(ref) = {np.sqrt(np.mean(want ** 2)):.4g}")
    assert ratio.max() <= 1.0, f"{what}: {int((ratio > 1).sum())} of {ratio.size} outside the bound"
    return float(ratio.max())


def check_fp8_layer(inp, what, block_m=0, tokens=None, got=None):
    if got is None:
        got = run_fp8_layer(inp, block_m)
    want, mid = oracle_fp8_layer(inp, return_intermediates=True, **({} if tokens is None else {"tokens": tokens}))
    g = got if tokens is None else got[tokens]
    return assert_layer_close(g, want, what, moved_code_allowance(inp, mid, tokens))


FP8_LAYER_SHAPES = [
    FP8_MOE_CONFIGS["fp8_moe_tiny"],
    Fp8MoEConfig("fp8_mid", T=70, K=512, N=384, E=12, topk=3, seed=3),
    Fp8MoEConfig("fp8_mid_f16", T=33, K=1024, N=256, E=5, topk=2, dtype="f16", seed=4),
    Fp8MoEConfig("fp8_one_token", T=1, K=256, N=128, E=8, topk=2, seed=5),
    Fp8MoEConfig("fp8_big_blocks", T=600, K=256, N=128, E=4, topk=2, seed=7),
]


@pytest.mark.parametrize("cfg", FP8_LAYER_SHAPES, ids=lambda c: c.name)
def test_fp8_layer_matches_oracle(cfg):
    say(f"fp8 layer {cfg}")
    inp = make_fp8_moe_inputs(cfg)
    check_fp8_layer(inp, cfg.name)


@pytest.mark.parametrize("block_m", [16, 64, 128, 256])
def test_fp8_layer_every_block_size(block_m):
    cfg = Fp8MoEConfig("fp8_blocks", T=300, K=384, N=256, E=5, topk=2, seed=8)
    say(f"fp8 layer block_m={block_m}")
    inp = make_fp8_moe_inputs(cfg)
    check_fp8_layer(inp, f"block_m {block_m}", block_m=block_m)


def test_fp8_layer_moved_codes_are_rare_and_mistakes_are_caught():
    """The statistical term of the bound rests on few activation codes differing between the two
    sides; measure it on the staged pieces.  And the bound still separates right from wrong."""
    cfg = Fp8MoEConfig("fp8_stat", T=96, K=1024, N=512, E=6, topk=2, seed=9)
    say(f"fp8 layer code statistics {cfg}")
    inp = make_fp8_moe_inputs(cfg)
    want, mid = oracle_fp8_layer(inp, return_intermediates=True)
    # GPU pieces: quantise X (bit-exact), grouped product, fused SiLU quantiser
    X = U.bits_to_dev(inp.x_bits, cfg.dtype)
    xq = torch.empty((cfg.T, cfg.K), dtype=torch.uint8, device="cuda")
    sx = torch.empty((cfg.T, cfg.K // 128), dtype=torch.float32, device="cuda")
    M.fp8_quantize_rows(X, xq, sx)
    al = U.run_align(U.i32(inp.topk_ids), cfg.E, 32)
    H = torch.zeros((cfg.S, 2 * cfg.N), dtype=U.TORCH_DT[cfg.dtype], device="cuda")
    M.fp8_moe_grouped_gemm(xq, sx, cfg.topk, torch.from_numpy(inp.w1_codes).cuda(), torch.from_numpy(inp.w1_scale).cuda(),
                           al["sorted_slot_ids"], al["block_expert_ids"], al["num_padded"], cfg.S, 32, H)
    aq = torch.empty((cfg.S, cfg.N), dtype=torch.uint8, device="cuda")
    sa = torch.empty((cfg.S, cfg.N // 128), dtype=torch.float32, device="cuda")
    M.fp8_silu_mul_quantize(H, aq, sa)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(xq.cpu().numpy(), mid["xq"])
    moved = float(np.mean(aq.cpu().numpy() != mid["aq"]))
    h_flips = float(np.mean(U.dev_to_f64(H) != mid["H"]))
    say(f"  H elements that differ: {h_flips:.4%}; activation codes that differ: {moved:.4%}")
    assert moved < 0.02
    got = run_fp8_layer(inp)
    assert_layer_close(got, want, "layer", moved_code_allowance(inp, mid))
    # planted mistakes, in the oracle: neighbouring block scale of W2, gate and up swapped
    wrong_scale = F.moe_layer(O.decode_bits(inp.x_bits, cfg.dtype), inp.topk_ids, inp.topk_weights, inp.w1_codes,
                              inp.w1_scale, inp.w2_codes, np.roll(inp.w2_scale, 1, axis=2), cfg.dtype)
    N = cfg.N
    swapped = np.concatenate([inp.w1_codes[:, N:], inp.w1_codes[:, :N]], axis=1)
    wrong_gate = F.moe_layer(O.decode_bits(inp.x_bits, cfg.dtype), inp.topk_ids, inp.topk_weights, swapped,
                             np.concatenate([inp.w1_scale[:, N // 128:], inp.w1_scale[:, :N // 128]], axis=1),
                             inp.w2_codes, inp.w2_scale, cfg.dtype)
    for name, wrong in (("neighbouring W2 block scale", wrong_scale), ("gate/up swapped", wrong_gate)):
        r = np.abs(got - wrong) / layer_bound(wrong)
        say(f"  planted mistake '{name}': max err / bound = {r.max():.1f}, outside the bound: {np.mean(r > 1):.1%}")
        assert r.max() > 5.0 and np.mean(r > 1) > 0.1


def test_fp8_layer_invalid_ids_permutation_and_errors():
    cfg = Fp8MoEConfig("fp8_inv", T=24, K=256, N=128, E=6, topk=3, seed=10)
    say(f"fp8 layer invalid ids / permutation {cfg}")
    inp = make_fp8_moe_inputs(cfg)
    inp.topk_ids[2, 0] = 6
    inp.topk_ids[5, 2] = -1
    inp.topk_ids[7, :] = 100
    got = run_fp8_layer(inp)
    want, mid = oracle_fp8_layer(inp, return_intermediates=True)
    assert np.all(want[7] == 0) and np.all(got[7] == 0)
    assert_layer_close(got, want, "invalid ids", moved_code_allowance(inp, mid))
    perm = np.random.default_rng(1).permutation(cfg.T)
    inp.x_bits, inp.topk_ids, inp.topk_weights = inp.x_bits[perm], inp.topk_ids[perm], inp.topk_weights[perm]
    assert np.array_equal(run_fp8_layer(inp), got[perm]), "a token's result must not depend on its position"
    # error paths
    X = U.bits_to_dev(inp.x_bits, cfg.dtype)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    out = torch.empty((cfg.T, cfg.K), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(M.MoEError) as e:
        M.fp8_moe_layer(X, U.i32(inp.topk_ids), torch.from_numpy(inp.topk_weights).cuda(),
                        torch.from_numpy(inp.w1_codes).cuda(), torch.from_numpy(inp.w1_scale).cuda(),
                        torch.from_numpy(inp.w2_codes).cuda(), torch.from_numpy(inp.w2_scale).cuda(), out, small)
    assert e.value.status == 3
    with pytest.raises(M.MoEError) as e:
        M.fp8_quantize_rows(X[:, :200].contiguous(), small, small.view(torch.float32))
    assert e.value.status == 2


def test_fp8_layer_full_size_decode_sampled_tokens():
    """The DeepSeek-shaped decode batch (256 experts, 11 GB of e4m3 weights): the layer on tokens
    chosen to cover as many experts as possible, in the launch configuration the benchmark times."""
    cfg = FP8_MOE_CONFIGS["fp8_moe_decode"]
    say(f"fp8 layer full size {cfg}: generating")
    inp = make_fp8_moe_inputs(cfg)
    got = run_fp8_layer(inp)
    chosen, seen = [], set()
    while len(chosen) < 8:
        gain = np.array([len(set(r.tolist()) - seen) for r in inp.topk_ids])
        gain[chosen] = -1
        t = int(np.argmax(gain))
        chosen.append(t)
        seen.update(int(e) for e in inp.topk_ids[t])
    tokens = sorted(chosen)
    say(f"fp8 layer full size: oracle for tokens {tokens} ({len(seen)} distinct experts)")
    check_fp8_layer(inp, "fp8_moe_decode sampled tokens", tokens=tokens, got=got)
    assert np.array_equal(got, run_fp8_layer(inp)), "layer is not run-to-run deterministic"


def test_fp8_layer_full_size_prefill_sampled_tokens():
    """The DeepSeek-shaped prefill batch (T = 4096, about 128 rows per expert: 128-slot blocks, most
    experts own one full block and a second, partly filled one): the first and the last token plus
    tokens chosen to cover many experts, in the launch configuration the benchmark times."""
    cfg = FP8_MOE_CONFIGS["fp8_moe_prefill"]
    say(f"fp8 layer full size {cfg}: generating")
    inp = make_fp8_moe_inputs(cfg)
    got = run_fp8_layer(inp)
    chosen, seen = [0, cfg.T - 1], set()
    for t in chosen:
        seen.update(int(e) for e in inp.topk_ids[t])
    while len(chosen) < 8:
        gain = np.array([len(set(r.tolist()) - seen) for r in inp.topk_ids])
        gain[chosen] = -1
        t = int(np.argmax(gain))
        chosen.append(t)
        seen.update(int(e) for e in inp.topk_ids[t])
    tokens = sorted(chosen)
    say(f"fp8 layer full size: oracle for tokens {tokens} ({len(seen)} distinct experts)")
    check_fp8_layer(inp, "fp8_moe_prefill sampled tokens", tokens=tokens, got=got)


def test_fp8_layer_on_random_shapes():
    """Thirty seeded random shapes (1 to 900 tokens, 1 to 32 experts, K up to 1536, N up to 1024,
    both 16-bit types), whole output against the oracle with the bound of this module."""
    rng = np.random.default_rng(21)
    for case in range(30):
        K = 128 * int(rng.integers(1, 13))
        N = 128 * int(rng.integers(1, 9))
        E = int(rng.integers(1, 33))
        topk = int(rng.integers(1, min(E, 8) + 1))
        T = int(rng.choice([1, 3, 16, 40, 130, 300, 900]))
        dt = "bf16" if rng.random() < 0.6 else "f16"
        cfg = Fp8MoEConfig(f"fp8_random{case}", T=T, K=K, N=N, E=E, topk=topk, dtype=dt, seed=500 + case)
        say(f"fp8 layer random shape {case}: {cfg}")
        inp = make_fp8_moe_inputs(cfg)
        check_fp8_layer(inp, cfg.name)
