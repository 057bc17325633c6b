"""Pins for the blockwise-scaled FP8 GEMM oracle (no GPU).  The paper names the operator
(Table II; Section VII-D) and prints no numeric example, so the pins are: the 8-bit decode against
a library cast and hand values from the format's definition, an exact-rational scalar brute
force, the unit-scale special case (a plain library matmul), a closed form, and block-scale
linearity; mutation checks show the brute force catches a transposed scale index, a wrong block
and a wrong exponent bias."""
from __future__ import annotations

import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from moe_workloads.fp8 import FP8_CONFIGS, Fp8GemmConfig, make_fp8_inputs
from oracle import fp8_oracle as F
from oracle import moe_oracle as O


def valid_codes(rng, shape):
    c = rng.integers(0, 256, size=shape, dtype=np.uint8)
    c[(c & 0x7F) == 0x7F] = 0x38
    return c


# ------------------------------------------------------------------ the 8-bit format
def test_decode_table_matches_library_cast():
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = F.decode_e4m3(codes)
    assert np.array_equal(np.isnan(got), np.isnan(lib))
    assert np.array_equal(got[~np.isnan(got)], lib[~np.isnan(lib)])
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF]) and np.isnan(got).sum() == 2


def test_decode_hand_values():
    """From the definition: bias 7, 3 mantissa bits, subnormals m/8 * 2^-6, no infinities."""
    want = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x38: 1.0, 0x39: 1.125,
            0x40: 2.0, 0x7E: 448.0, 0x78: 256.0, 0xB8: -1.0, 0xC0: -2.0, 0xFE: -448.0}
    for code, v in want.items():
        assert F.decode_e4m3(np.array([code], dtype=np.uint8))[0] == v, hex(code)
    assert np.signbit(F.decode_e4m3(np.array([0x80], dtype=np.uint8))[0])
    finite = F.decode_e4m3(np.arange(256, dtype=np.uint8))
    assert np.nanmax(finite) == 448.0 and not np.isinf(finite).any()
    # monotone in the code within a sign
    pos = finite[:0x7F]
    assert np.all(np.diff(pos) > 0)


# ------------------------------------------------------------------ exact-rational brute force
def frac_decode(code: int, bias: int = 7) -> Fraction:
    s = -1 if code & 0x80 else 1
    e, m = (code >> 3) & 15, code & 7
    if e == 0:
        return s * Fraction(m, 8) * Fraction(1, 2 ** (bias - 1))
    return s * (1 + Fraction(m, 8)) * (Fraction(2) ** (e - bias))


def brute(a, sa, b, sb, block, scale_index=lambda n, kb, block: (n // block, kb), bias=7):
    M, K = a.shape
    N = b.shape[0]
    out = np.empty((M, N))
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                kb = k // block
                i, j = scale_index(n, kb, block)
                acc += (Fraction(float(sa[m, kb])) * Fraction(float(sb[i, j])) *
                        frac_decode(int(a[m, k]), bias) * frac_decode(int(b[n, k]), bias))
            out[m, n] = float(acc)
    return out


@pytest.mark.parametrize("M,N,K,block,seed", [(3, 5, 8, 4, 1), (2, 9, 12, 4, 2), (4, 4, 16, 8, 3), (1, 3, 4, 2, 4)])
def test_blockwise_gemm_against_rational_brute_force(M, N, K, block, seed):
    rng = np.random.default_rng(seed)
    a, b = valid_codes(rng, (M, K)), valid_codes(rng, (N, K))
    sa = rng.uniform(0.5, 2.0, size=(M, K // block)).astype(np.float32)
    sb = rng.uniform(0.5, 2.0, size=(-(-N // block), K // block)).astype(np.float32)
    want = brute(a, sa, b, sb, block)
    got = F.blockwise_gemm(a, sa, b, sb, out_dt=None, block=block)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-9)
    np.testing.assert_array_equal(F.blockwise_gemm(a, sa, b, sb, "bf16", block), O.rnd(got, "bf16"))


def test_brute_force_is_sensitive_to_plausible_mistakes():
    """A transposed block-scale index, the neighbouring reduction block's scale and a wrong exponent
    bias all move the brute-force result away from the oracle's (so agreeing with it means something)."""
    rng = np.random.default_rng(5)
    M, N, K, block = 2, 8, 8, 4
    a, b = valid_codes(rng, (M, K)), valid_codes(rng, (N, K))
    sa = rng.uniform(0.5, 2.0, size=(M, 2)).astype(np.float32)
    sb = rng.uniform(0.5, 2.0, size=(2, 2)).astype(np.float32)
    got = F.blockwise_gemm(a, sa, b, sb, out_dt=None, block=block)
    np.testing.assert_allclose(got, brute(a, sa, b, sb, block), rtol=1e-13)
    assert not np.allclose(brute(a, sa, b, sb, block, scale_index=lambda n, kb, bl: (kb, n // bl)), got, rtol=1e-6)
    assert not np.allclose(brute(a, sa, b, sb, block, scale_index=lambda n, kb, bl: (n // bl, 1 - kb)), got, rtol=1e-6)
    assert not np.allclose(brute(a, sa, b, sb, block, bias=8), got, rtol=1e-6)


# ------------------------------------------------------------------ special cases and invariants
def test_unit_scales_reduce_to_a_plain_matmul():
    rng = np.random.default_rng(7)
    M, N, K = 9, 200, 256
    a, b = valid_codes(rng, (M, K)), valid_codes(rng, (N, K))
    Ad = torch.from_numpy(a).view(torch.float8_e4m3fn).to(torch.float64)
    Bd = torch.from_numpy(b).view(torch.float8_e4m3fn).to(torch.float64)
    want = (Ad @ Bd.T).numpy()
    ones_a = np.ones((M, K // 128), np.float32)
    ones_b = np.ones((2, K // 128), np.float32)
    got = F.blockwise_gemm(a, ones_a, b, ones_b, out_dt=None)
    np.testing.assert_array_equal(got, want)        # every partial sum is exact in float64
    # bf16 rounding against the library's cast of the (float32-exact) result
    small = np.abs(want) < 2.0 ** 20
    lib = torch.from_numpy(want).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(F.blockwise_gemm(a, ones_a, b, ones_b)[small], lib[small])


def test_partial_sums_are_exact_in_float64():
    """128 products of two 4-bit significands with exponents in [-18, 17]: an integer multiple of
    2^-18 below 2^25 -- far inside 53 bits, whatever the order of summation."""
    rng = np.random.default_rng(8)
    a, b = valid_codes(rng, (4, 128)), valid_codes(rng, (6, 128))
    A, B = F.decode_e4m3(a), F.decode_e4m3(b)
    want = np.array([[float(sum(Fraction(float(x)) * Fraction(float(y)) for x, y in zip(A[m], B[n])))
                      for n in range(6)] for m in range(4)])
    np.testing.assert_array_equal(A @ B.T, want)
    np.testing.assert_array_equal(A[:, ::-1] @ B[:, ::-1].T, want)


def test_closed_form_constant_operands():
    M, N, K = 5, 130, 384
    a = np.full((M, K), 0x38, np.uint8)            # 1.0
    b = np.full((N, K), 0xC0, np.uint8)            # -2.0
    sa = np.full((M, 3), 0.5, np.float32)
    sb = np.array([[0.25, 0.5, 1.0], [2.0, 4.0, 8.0]], np.float32)
    got = F.blockwise_gemm(a, sa, b, sb, out_dt=None)
    assert np.all(got[:, :128] == -2.0 * 128 * 0.5 * (0.25 + 0.5 + 1.0))
    assert np.all(got[:, 128:] == -2.0 * 128 * 0.5 * (2.0 + 4.0 + 8.0))


def test_block_scale_linearity():
    """Doubling b_scale[nb, kb] moves only the columns of block nb, by that block's partial product
    times the old scales; doubling a_scale[m, kb] moves only row m."""
    inp = make_fp8_inputs(FP8_CONFIGS["fp8_tiny"])
    base = F.blockwise_gemm(inp.a_codes, inp.a_scale, inp.b_codes, inp.b_scale, out_dt=None)
    nb, kb, m = 1, 2, 5
    sb2 = inp.b_scale.copy(); sb2[nb, kb] *= 2
    moved = F.blockwise_gemm(inp.a_codes, inp.a_scale, inp.b_codes, sb2, out_dt=None) - base
    A, B = F.decode_e4m3(inp.a_codes), F.decode_e4m3(inp.b_codes)
    part = A[:, 128 * kb:128 * kb + 128] @ B[128 * nb:, 128 * kb:128 * kb + 128].T
    want = inp.a_scale[:, kb].astype(np.float64)[:, None] * float(inp.b_scale[nb, kb]) * part
    np.testing.assert_allclose(moved[:, 128 * nb:], want, rtol=1e-9, atol=1e-12)
    assert np.all(moved[:, :128 * nb] == 0)
    sa2 = inp.a_scale.copy(); sa2[m, kb] *= 2
    moved = F.blockwise_gemm(inp.a_codes, sa2, inp.b_codes, inp.b_scale, out_dt=None) - base
    assert np.all(np.delete(moved, m, axis=0) == 0) and np.any(moved[m] != 0)


# ------------------------------------------------------------------ grouped (one matrix per expert)
def test_grouped_against_brute_force_per_slot():
    rng = np.random.default_rng(31)
    E, N, K, block, R, row_div = 3, 6, 8, 4, 4, 2
    a = valid_codes(rng, (R, K))
    b = valid_codes(rng, (E, N, K))
    sa = rng.uniform(0.5, 2.0, size=(R, K // block)).astype(np.float32)
    sb = rng.uniform(0.5, 2.0, size=(E, -(-N // block), K // block)).astype(np.float32)
    slot_expert = np.array([2, 0, 1, 7, 0, -1, 2, 2])                 # two ignored ids
    C, valid = F.grouped_blockwise_gemm(a, sa, row_div, b, sb, slot_expert, out_dt=None, block=block)
    assert valid.tolist() == [True, True, True, False, True, False, True, True]
    for s_, e in enumerate(slot_expert):
        if not valid[s_]:
            assert np.all(C[s_] == 0)
            continue
        r = s_ // row_div
        want = brute(a[r:r + 1], sa[r:r + 1], b[e], sb[e], block)
        np.testing.assert_allclose(C[s_:s_ + 1], want, rtol=1e-13, atol=1e-9)


def test_grouped_special_cases():
    """One expert and row_div = 1 is the dense product; row_div = k equals the same call on A with
    every row repeated k times; permuting the experts (and the ids alike) changes nothing."""
    inp = make_fp8_inputs(Fp8GemmConfig("g1", M=6, N=128, K=256, seed=5))
    dense = F.blockwise_gemm(inp.a_codes, inp.a_scale, inp.b_codes, inp.b_scale)
    C, valid = F.grouped_blockwise_gemm(inp.a_codes, inp.a_scale, 1, inp.b_codes[None], inp.b_scale[None],
                                        np.zeros(6, np.int32))
    assert valid.all() and np.array_equal(C, dense)
    rng = np.random.default_rng(6)
    E = 3
    b = np.stack([make_fp8_inputs(Fp8GemmConfig("g", M=1, N=128, K=256, seed=10 + e)).b_codes for e in range(E)])
    sb = np.stack([make_fp8_inputs(Fp8GemmConfig("g", M=1, N=128, K=256, seed=10 + e)).b_scale for e in range(E)])
    ids = rng.integers(0, E, size=12)
    C2, _ = F.grouped_blockwise_gemm(inp.a_codes, inp.a_scale, 2, b, sb, ids)
    C1, _ = F.grouped_blockwise_gemm(np.repeat(inp.a_codes, 2, axis=0), np.repeat(inp.a_scale, 2, axis=0), 1, b, sb, ids)
    assert np.array_equal(C1, C2)
    perm = np.array([2, 0, 1])                                         # new expert j is old expert perm[j]
    inv = np.argsort(perm)
    C3, _ = F.grouped_blockwise_gemm(inp.a_codes, inp.a_scale, 2, b[perm], sb[perm], inv[ids])
    assert np.array_equal(C3, C2)


def test_generator_shapes_and_range():
    inp = make_fp8_inputs(Fp8GemmConfig("g", M=7, N=130, K=256, seed=3))
    assert inp.a_codes.shape == (7, 256) and inp.a_scale.shape == (7, 2) and inp.a_scale.dtype == np.float32
    assert inp.b_codes.shape == (130, 256) and inp.b_scale.shape == (2, 2)
    A = F.decode_e4m3(inp.a_codes)
    assert not np.isnan(A).any() and np.abs(A).max() == 448.0
    # every 1 x 128 tile of the activations reaches the largest finite code
    assert np.all(np.abs(A).reshape(7, 2, 128).max(axis=2) == 448.0)
    again = make_fp8_inputs(Fp8GemmConfig("g", M=7, N=130, K=256, seed=3))
    assert np.array_equal(again.b_codes, inp.b_codes) and np.array_equal(again.a_scale, inp.a_scale)


def test_oracle_reproduces_golden_fixture():
    """Regression guard: the frozen output of the pinned oracle on a small seeded case (also the
    generator's codes and scales, so a change of the input recipe shows up here)."""
    with open(os.path.join(os.path.dirname(__file__), "golden", "small_fp8_gemm.json")) as f:
        doc = json.load(f)
    c = doc["config"]
    inp = make_fp8_inputs(Fp8GemmConfig("golden_fp8", M=c["M"], N=c["N"], K=c["K"], seed=c["seed"]))
    assert inp.a_codes[0].tolist() == doc["a_codes_row0"]
    assert [[float(v).hex() for v in r] for r in inp.a_scale] == doc["a_scale"]
    assert [[float(v).hex() for v in r] for r in inp.b_scale] == doc["b_scale"]
    out = F.blockwise_gemm(inp.a_codes, inp.a_scale, inp.b_codes, inp.b_scale, "bf16")
    assert O.encode_bits(out, "bf16").tolist() == doc["out_bits"]


# ------------------------------------------------------------------ e4m3 encoder, activation quantiser
def all_positive_e4m3():
    """(value as Fraction, code) for the 127 non-negative finite codes, from the format definition."""
    return [(frac_decode(c), c) for c in range(0x7F)]


def frac_encode(y: Fraction) -> int:
    """Nearest e4m3 value by exact comparison, ties to the even mantissa, saturating at 448."""
    table = all_positive_e4m3()
    a = abs(y)
    best = min(table, key=lambda vc: (abs(vc[0] - a), vc[1] & 1))      # on a tie the even code wins
    return best[1] | (0x80 if y < 0 else 0)


def test_encode_matches_library_cast_and_inverts_decode():
    rng = np.random.default_rng(11)
    y = (rng.standard_normal(300000) * np.exp(rng.uniform(-14, 6.2, 300000))).astype(np.float32)
    y = y[np.abs(y) <= 448.0]
    lib = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(F.encode_e4m3(y.astype(np.float64)), lib)
    finite = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    np.testing.assert_array_equal(F.encode_e4m3(F.decode_e4m3(finite)), finite)


def test_encode_hand_values_and_ties():
    cases = {1.0: 0x38, 1.0625: 0x38, 1.1875: 0x3A, 1.125: 0x39, 448.0: 0x7E, 500.0: 0x7E, -448.0: 0xFE,
             2.0 ** -9: 0x01, 2.0 ** -10: 0x00, 3 * 2.0 ** -10: 0x02, 2.0 ** -6: 0x08, 7.5 * 2.0 ** -9: 0x08,
             0.0: 0x00, 224.0: 0x76, 112.0: 0x6E, -3.0: 0xC4}
    for v, code in cases.items():
        assert F.encode_e4m3(np.array([v]))[0] == code, (v, hex(code))
    assert F.encode_e4m3(np.array([-0.0]))[0] == 0x80
    assert F.encode_e4m3(np.array([np.nan]))[0] == 0x7F


def test_encode_against_exact_rational_nearest_value():
    rng = np.random.default_rng(12)
    ys = np.concatenate([(rng.standard_normal(400) * np.exp(rng.uniform(-9, 6, 400))).astype(np.float32),
                         np.array([1.0625, 1.1875, 17.0, 19.0, 2.0 ** -10, 3 * 2.0 ** -10, 447.9, 0.0], np.float32)])
    ys = ys[np.abs(ys) <= 448.0]
    got = F.encode_e4m3(ys.astype(np.float64))
    for y, c in zip(ys, got):
        assert int(c) == frac_encode(Fraction(float(y))) or (y == 0 and int(c) & 0x7F == 0), float(y)


def test_quantize_rows_hand_example_and_zero_tile():
    x = np.array([[1.0, -2.0, 0.5, 0.0, 0.0, 0.0, 0.0, 0.0]])
    codes, scale = F.quantize_rows(x, block=4)
    assert scale.dtype == np.float32
    assert scale[0, 0] == np.float32(2.0) / np.float32(448.0)
    np.testing.assert_array_equal(codes[0, :4], [0x76, 0xFE, 0x6E, 0x00])      # 224, -448, 112, 0
    assert scale[0, 1] == np.float32(1e-4) / np.float32(448.0)                  # all-zero tile: clamped maximum
    np.testing.assert_array_equal(codes[0, 4:], 0)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_quantize_rows_invariants_and_scalar_walk(dt):
    rng = np.random.default_rng(13)
    x = O.rnd(rng.standard_normal((6, 256)) * np.exp(rng.uniform(-6, 3, (6, 1))), dt)
    x[2, :128] = 0.0
    x[3, 5] = 0.0
    codes, scale = F.quantize_rows(x)
    t = x.reshape(6, 2, 128)
    # the largest element of every non-zero tile maps to +-448
    for r in range(6):
        for b in range(2):
            if np.abs(t[r, b]).max() > 1e-4:
                i = int(np.argmax(np.abs(t[r, b])))
                assert codes[r, 128 * b + i] & 0x7F == 0x7E
    # decode(code) * scale is within half an e4m3 step of x (step 2^-3 relative below the binade top,
    # 2^-9 of the scaled range in the subnormals), plus the float32 roundings of the two scale operations
    back = F.decode_e4m3(codes) * np.repeat(scale.astype(np.float64), 128, axis=1)
    assert np.all(np.abs(back - x) <= np.abs(x) * (2.0 ** -4 + 2.0 ** -20) + np.repeat(scale, 128, axis=1) * 2.0 ** -10)
    # scalar walk of the stated float32 steps, nearest value found in exact rationals
    for r, b in [(0, 0), (1, 1), (2, 0), (3, 0), (5, 1)]:
        m = np.float32(max(float(np.abs(t[r, b]).max()), 1e-4))
        m = max(m, np.float32(1e-4))
        ratio = np.float32(448.0) / m
        assert scale[r, b] == m / np.float32(448.0)
        for i in range(0, 128, 7):
            y = np.float32(t[r, b, i]) * ratio
            assert int(codes[r, 128 * b + i]) & 0x7F == frac_encode(Fraction(float(y))) & 0x7F


# ------------------------------------------------------------------ the FP8 mixture-of-experts layer
def brute_fp8_layer(X, ids, w, w1c, w1s, w2c, w2s, dt, block):
    """Scalar walk of the layer: per token and routed expert, quantise (float32 steps, nearest code by
    exact comparison), both products in exact rationals, float64 SiLU, roundings by the 16-bit oracle."""
    import math
    T, K = X.shape
    E, N2, _ = w1c.shape
    N = N2 // 2

    def quant(row):
        codes, scales = [], []
        for b0 in range(0, len(row), block):
            tile = [np.float32(v) for v in row[b0:b0 + block]]
            m = max(max(abs(v) for v in tile), np.float32(1e-4))
            ratio = np.float32(448.0) / np.float32(m)
            scales.append(np.float32(m) / np.float32(448.0))
            codes += [frac_encode(Fraction(float(np.float32(v) * ratio))) | (0x80 if np.signbit(v) else 0) for v in tile]
        return codes, scales

    def product(codes, scales, wc, ws, n):
        acc = Fraction(0)
        for k in range(len(codes)):
            kb = k // block
            acc += (Fraction(float(scales[kb])) * Fraction(float(ws[n // block, kb])) *
                    frac_decode(codes[k]) * frac_decode(int(wc[n, k])))
        return acc

    out = np.zeros((T, K))
    for t in range(T):
        xq, sx = quant(X[t])
        tot = [0.0] * K
        for j in range(ids.shape[1]):
            e = int(ids[t, j])
            if e < 0 or e >= E:
                continue
            H = [float(O.rnd(float(product(xq, sx, w1c[e], w1s[e], n)), dt)) for n in range(2 * N)]
            act = [float(O.rnd(H[n] / (1.0 + math.exp(-H[n])) * H[N + n], dt)) for n in range(N)]
            aq, sa = quant(act)
            for c in range(K):
                tot[c] += float(w[t, j]) * float(product(aq, sa, w2c[e], w2s[e], c))
        out[t] = O.rnd(np.array(tot), dt)
    return out


def tiny_fp8_layer_case(seed, T=3, K=8, N=8, E=3, topk=2, block=4, dt="bf16"):
    rng = np.random.default_rng(seed)
    X = O.rnd(rng.standard_normal((T, K)) * 0.7, dt)
    ids = np.stack([rng.permutation(E)[:topk] for _ in range(T)]).astype(np.int32)
    w = rng.dirichlet(np.ones(topk), T).astype(np.float32)
    w1c, w2c = valid_codes(rng, (E, 2 * N, K)), valid_codes(rng, (E, K, N))
    # keep magnitudes modest: exponent field at most 9 (|v| < 8)
    w1c = (w1c & 0x87) | (((w1c >> 3) & 15) % 10 << 3)
    w2c = (w2c & 0x87) | (((w2c >> 3) & 15) % 10 << 3)
    w1s = rng.uniform(0.05, 0.2, (E, 2 * N // block, K // block)).astype(np.float32)
    w2s = rng.uniform(0.05, 0.2, (E, K // block, N // block)).astype(np.float32)
    return X, ids, w, w1c.astype(np.uint8), w1s, w2c.astype(np.uint8), w2s, dt, block


@pytest.mark.parametrize("seed,dt", [(21, "bf16"), (22, "f16"), (23, "bf16")])
def test_fp8_layer_against_scalar_brute_force(seed, dt):
    X, ids, w, w1c, w1s, w2c, w2s, dt, block = tiny_fp8_layer_case(seed, dt=dt)
    got = F.moe_layer(X, ids, w, w1c, w1s, w2c, w2s, dt, block=block)
    want = brute_fp8_layer(X, ids, w, w1c, w1s, w2c, w2s, dt, block)
    # the two sum the same exact products in a different order: equal up to float64 rounding of the sums,
    # which can flip a final 16-bit rounding only on an exact near-tie
    np.testing.assert_allclose(got, want, rtol=2.0 ** -7, atol=1e-12)
    assert np.mean(got == want) > 0.9


def test_fp8_layer_brute_force_catches_plausible_mistakes():
    X, ids, w, w1c, w1s, w2c, w2s, dt, block = tiny_fp8_layer_case(24)
    want = brute_fp8_layer(X, ids, w, w1c, w1s, w2c, w2s, dt, block)
    swapped = np.concatenate([w1c[:, w1c.shape[1] // 2:], w1c[:, :w1c.shape[1] // 2]], axis=1)   # gate <-> up
    assert not np.allclose(F.moe_layer(X, ids, w, swapped, w1s, w2c, w2s, dt, block=block), want, rtol=1e-2)
    assert not np.allclose(F.moe_layer(X, ids, w, w1c, w1s[:, ::-1], w2c, w2s, dt, block=block), want, rtol=1e-2)
    assert not np.allclose(F.moe_layer(X, ids[:, ::-1], w, w1c, w1s, w2c, w2s, dt, block=block), want, rtol=1e-2)


def test_fp8_layer_one_hot_routing_is_the_dense_chain():
    rng = np.random.default_rng(25)
    T, K, N, E = 5, 256, 128, 3
    X = O.rnd(rng.standard_normal((T, K)) * 0.5, "bf16")
    w1c, w2c = valid_codes(rng, (E, 2 * N, K)), valid_codes(rng, (E, K, N))
    w1c, w2c = (w1c & 0xB7).astype(np.uint8), (w2c & 0xB7).astype(np.uint8)      # exponent field <= 6: |v| < 1
    w1s = rng.uniform(0.01, 0.03, (E, 2, 2)).astype(np.float32)
    w2s = rng.uniform(0.01, 0.03, (E, 2, 1)).astype(np.float32)
    ids = np.full((T, 1), 1, np.int32)
    got = F.moe_layer(X, ids, np.ones((T, 1), np.float32), w1c, w1s, w2c, w2s, "bf16")
    xq, sx = F.quantize_rows(X)
    H = F.blockwise_gemm(xq, sx, w1c[1], w1s[1], "bf16")
    act = O.silu_mul(H, "bf16")
    aq, sa = F.quantize_rows(act)
    np.testing.assert_array_equal(got, F.blockwise_gemm(aq, sa, w2c[1], w2s[1], "bf16"))


def test_fp8_layer_token_permutation_and_ignored_slots():
    from moe_workloads.fp8 import FP8_MOE_CONFIGS, make_fp8_moe_inputs
    inp = make_fp8_moe_inputs(FP8_MOE_CONFIGS["fp8_moe_tiny"])
    c = inp.cfg
    X = O.decode_bits(inp.x_bits, c.dtype)
    args = (inp.w1_codes, inp.w1_scale, inp.w2_codes, inp.w2_scale, c.dtype)
    base = F.moe_layer(X, inp.topk_ids, inp.topk_weights, *args)
    perm = np.random.default_rng(2).permutation(c.T)
    np.testing.assert_array_equal(F.moe_layer(X[perm], inp.topk_ids[perm], inp.topk_weights[perm], *args), base[perm])
    np.testing.assert_array_equal(F.moe_layer(X, inp.topk_ids, inp.topk_weights, *args, tokens=[3, 9]), base[[3, 9]])
    ids = inp.topk_ids.copy()
    ids[4, :] = c.E + 5
    assert np.all(F.moe_layer(X, ids, inp.topk_weights, *args)[4] == 0)
    # the workload's codes hold no NaN pattern and its weights have the stated spread
    assert not ((inp.w1_codes & 0x7F) == 0x7F).any() and not ((inp.w2_codes & 0x7F) == 0x7F).any()
    wd = F.decode_e4m3(inp.w1_codes[0]) * np.repeat(np.repeat(inp.w1_scale[0], 128, 0), 128, 1)
    assert 0.015 < wd.std() < 0.025
