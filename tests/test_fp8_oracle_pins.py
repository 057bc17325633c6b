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
