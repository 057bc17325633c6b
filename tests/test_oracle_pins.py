"""Pins for the CPU oracle (no GPU).  The paper prints no worked numeric
example for the mixed-type MoE layer (Section VII-B gives only ratios and
Table III's instruction widths), so the oracle is pinned by: an independent
exact-rational scalar brute force, closed forms, invariants, special cases
that collapse to a dense library GEMM, and rounding against library casts and
hand-derived ties.  A few mutation checks show the pins are sensitive to the
plausible mistakes (nibble order, zero-point sign, gate/up swap, group index,
row map)."""
from __future__ import annotations

import numpy as np
import pytest
import torch
from hypothesis import given, settings, strategies as st

import bruteforce as bf
from moe_workloads import MoEConfig, make_inputs, route_topk as gen_route, to_bits, skew_bias, CONFIGS
from oracle import moe_oracle as O


def tiny_cfg(dtype="f16", **kw):
    base = dict(name="t", T=3, K=16, N=8, E=2, topk=2, group=8, dtype=dtype, seed=7)
    base.update(kw)
    return MoEConfig(**base)


def frac_to_np(rows):
    return np.array([[float(v) for v in r] for r in rows], dtype=np.float64)


def oracle_layer(inp, **kw):
    c = inp.cfg
    return O.layer(O.decode_bits(inp.x_bits, c.dtype), inp.topk_ids, inp.topk_weights,
                   inp.qw1, O.decode_bits(inp.s1_bits, c.dtype), inp.z1,
                   inp.qw2, O.decode_bits(inp.s2_bits, c.dtype), inp.z2, c.group, c.dtype, **kw)


# ------------------------------------------------------------------ rounding
def test_rnd_f16_matches_numpy_cast():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-9, 5, 20000),
                        [0.0, -0.0, 65504.0, 65519.99, 65520.0, 7e4, -7e4, 2.0 ** -24, 2.0 ** -25,
                         1.5 * 2.0 ** -25, 2.0 ** -14, np.inf, -np.inf]])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).astype(np.float64)
    np.testing.assert_array_equal(O.rnd(x, "f16"), want)


def test_rnd_bf16_matches_torch_cast_on_float32_inputs():
    rng = np.random.default_rng(2)
    x32 = (rng.standard_normal(20000) * 10.0 ** rng.integers(-20, 20, 20000)).astype(np.float32)
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.rnd(x32.astype(np.float64), "bf16"), want)


def test_rnd_hand_derived_ties_and_single_rounding():
    # bf16 keeps 8 significant bits: spacing 2^-7 in [1, 2)
    assert O.rnd(1 + 2.0 ** -8, "bf16") == 1.0                    # tie -> even
    assert O.rnd(1 + 3 * 2.0 ** -8, "bf16") == 1 + 2.0 ** -6      # tie -> even (up)
    # just above the tie: must go up; a detour through float32 would lose the 2^-40
    assert O.rnd(1 + 2.0 ** -8 + 2.0 ** -40, "bf16") == 1 + 2.0 ** -7
    assert O.rnd(1 + 2.0 ** -11, "f16") == 1.0
    assert O.rnd(1 + 3 * 2.0 ** -11, "f16") == 1 + 2.0 ** -9
    assert O.rnd(1 + 2.0 ** -11 + 2.0 ** -40, "f16") == 1 + 2.0 ** -10
    assert O.rnd(-0.3, "f16") == -float(np.float16(0.3))


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_bits_roundtrip_all_patterns(dt):
    bits = np.arange(1 << 16, dtype=np.uint16)
    expo_all_ones = ((bits >> 10) & 0x1F) == 0x1F if dt == "f16" else ((bits >> 7) & 0xFF) == 0xFF
    finite = bits[~expo_all_ones]
    v = O.decode_bits(finite, dt)
    np.testing.assert_array_equal(O.encode_bits(v, dt), finite)
    np.testing.assert_array_equal(O.rnd(v, dt), v)        # representable values are fixed points
    # decode agrees with the format definition evaluated exactly
    for b in (0x0001, 0x03FF, 0x3C00, 0x7BFF, 0xC123, 0x0080, 0x3F80):
        if int(b) in set(finite.tolist()):
            assert float(bf.bits_to_fraction(b, dt)) == O.decode_bits(np.array([b], np.uint16), dt)[0]


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_rnd_matches_exact_rational_rounding(dt):
    from fractions import Fraction
    rng = np.random.default_rng(3)
    xs = rng.standard_normal(300) * 10.0 ** rng.integers(-3, 3, 300)
    got = O.rnd(xs, dt)
    for x, g in zip(xs, got):
        assert Fraction(g) == bf.round_fraction(Fraction(float(x)), dt)


# ------------------------------------------------------------------ packing / dequant
def test_unpack_reference_vector():
    w = np.array([0x76543210, 0xFEDCBA98 - (1 << 32)], dtype=np.int64).astype(np.int32)
    np.testing.assert_array_equal(O.unpack_int4(w), np.arange(16, dtype=np.uint8))


@given(st.lists(st.integers(0, 2 ** 32 - 1), min_size=1, max_size=16))
@settings(max_examples=200, deadline=None)
def test_pack_unpack_roundtrip(words):
    w = np.array(words, dtype=np.uint32).view(np.int32)
    q = O.unpack_int4(w)
    assert q.dtype == np.uint8 and q.max() <= 15
    np.testing.assert_array_equal(O.pack_int4(q), w)
    for j, word in enumerate(words):               # against Python integer arithmetic
        for i in range(8):
            assert q[8 * j + i] == bf.nibble(word, i)


def test_dequant_zero_nibbles_give_minus_z_times_s():
    rng = np.random.default_rng(4)
    s = O.decode_bits(to_bits(rng.uniform(0.002, 0.02, (3, 5, 4)), "f16"), "f16")
    z = rng.integers(0, 16, (3, 5, 4), dtype=np.uint8)
    W = O.dequant(np.zeros((3, 5, 4 * 32 // 8), np.int32), s, z, 32)
    want = np.repeat(-(z.astype(np.float64)) * s, 32, axis=-1)
    np.testing.assert_array_equal(W, want)


def test_dequant_q_equal_z_is_zero_and_one_hot_probe():
    g, G = 16, 3
    z = np.array([[5, 0, 15]], dtype=np.uint8)
    s = np.array([[0.5, 0.25, 2.0]])
    q = np.repeat(z, g, axis=-1)
    np.testing.assert_array_equal(O.dequant(O.pack_int4(q), s, z, g), np.zeros((1, g * G)))
    q2 = q.copy()
    q2[0, 17] = 9                      # element 17 lies in group 1: (9 - 0) * 0.25
    W = O.dequant(O.pack_int4(q2), s, z, g)
    assert W[0, 17] == 2.25 and np.count_nonzero(W) == 1


# ------------------------------------------------------------------ bucketing
@given(st.integers(1, 9), st.integers(1, 4), st.integers(1, 6), st.sampled_from([1, 2, 4, 16]),
       st.integers(0, 2 ** 31 - 1), st.booleans())
@settings(max_examples=150, deadline=None)
def test_align_matches_bruteforce_and_invariants(T, topk, E, block_m, seed, with_invalid):
    rng = np.random.default_rng(seed)
    lo, hi = (-1, E + 1) if with_invalid else (0, E)
    ids = rng.integers(lo, hi, size=(T, topk)).astype(np.int32)
    got = O.align_by_expert(ids, E, block_m)
    counts, offsets, sorted_ids, blocks = bf.bucket(ids.reshape(-1).tolist(), E, block_m)
    np.testing.assert_array_equal(got["expert_counts"], counts)
    np.testing.assert_array_equal(got["expert_offsets"], offsets)
    np.testing.assert_array_equal(got["sorted_slot_ids"], sorted_ids)
    np.testing.assert_array_equal(got["block_expert_ids"], blocks)
    assert got["num_padded"][0] == offsets[-1]
    S = T * topk
    assert len(sorted_ids) == O.align_capacity(T, topk, E, block_m)
    assert got["num_padded"][0] <= len(sorted_ids)
    valid = [s for s in range(S) if 0 <= ids.reshape(-1)[s] < E]
    real = [s for s in got["sorted_slot_ids"].tolist() if s != S]
    assert sorted(real) == valid                       # each valid slot exactly once
    assert all(o % block_m == 0 for o in got["expert_offsets"].tolist())
    be = [b for b in got["block_expert_ids"].tolist() if b >= 0]
    assert be == sorted(be)


def test_align_empty_and_single_expert():
    got = O.align_by_expert(np.zeros((0, 2), np.int32), 4, 16)
    assert got["num_padded"][0] == 0 and got["sorted_slot_ids"].size == 0
    got = O.align_by_expert(np.full((5, 1), 2, np.int32), 4, 4)
    np.testing.assert_array_equal(got["expert_counts"], [0, 0, 5, 0])
    np.testing.assert_array_equal(got["expert_offsets"], [0, 0, 0, 8, 8])
    np.testing.assert_array_equal(got["sorted_slot_ids"][:8], [0, 1, 2, 3, 4, 5, 5, 5])
    np.testing.assert_array_equal(got["block_expert_ids"][:3], [2, 2, -1])


# ------------------------------------------------------------------ routing
def test_router_generator_matches_oracle_and_sums_to_one():
    rng = np.random.default_rng(5)
    logits = rng.standard_normal((40, 16)).astype(np.float32)
    logits[3, 4] = logits[3, 9] = logits[3].max() + 1.0          # a tie: lower index first
    ids_g, w_g = gen_route(logits, 4)
    ids_o, w_o = O.route_topk(logits, 4)
    np.testing.assert_array_equal(ids_g, ids_o)
    assert list(ids_g[3, :2]) == [4, 9]
    np.testing.assert_allclose(w_g, w_o, rtol=0, atol=1e-7)
    assert np.all(np.abs(w_g.astype(np.float64).sum(axis=1) - 1.0) <= 1e-6)
    # softmax over the selected logits only == full softmax renormalised
    sel = np.take_along_axis(logits.astype(np.float64), ids_o.astype(np.int64), axis=1)
    p = np.exp(sel - sel.max(axis=1, keepdims=True))
    np.testing.assert_allclose(w_o, p / p.sum(axis=1, keepdims=True), rtol=1e-13)


def test_router_against_scalar_selection_and_library_softmax():
    """ids: repeated arg-max with the tie rule written out as a scalar loop; weights for k = E:
    scipy's softmax; k = 1: exactly one; invariance under a common shift of the logits."""
    from scipy.special import softmax
    rng = np.random.default_rng(6)
    T, E, k = 30, 24, 5
    logits = rng.standard_normal((T, E)).astype(np.float32)
    logits[0, :] = 0.25                                   # all equal: ids 0..k-1
    logits[1, 7] = logits[1, 3] = 9.0                     # tie for the first place
    logits[2, 5] = -0.0; logits[2, 6] = 0.0; logits[2, [0, 1, 2, 3, 4]] = -1.0   # signed zeros compare equal
    logits[2, 7:] = -2.0
    ids, w = O.route_topk(logits, k)
    for t in range(T):
        taken, want = set(), []
        for _ in range(k):
            best = None
            for e in range(E):
                if e in taken:
                    continue
                if best is None or float(logits[t, e]) > float(logits[t, best]):
                    best = e                               # strict '>' keeps the lower index on ties
            taken.add(best); want.append(best)
        assert list(ids[t]) == want, (t, list(ids[t]), want)
    assert list(ids[0]) == [0, 1, 2, 3, 4] and list(ids[1][:2]) == [3, 7] and list(ids[2][:2]) == [5, 6]
    ids_all, w_all = O.route_topk(logits, E)
    full = softmax(logits.astype(np.float64), axis=1)
    np.testing.assert_allclose(w_all, np.take_along_axis(full, ids_all.astype(np.int64), axis=1), rtol=1e-12)
    ids1, w1 = O.route_topk(logits, 1)
    assert np.all(w1 == 1.0) and np.array_equal(ids1[:, 0], ids[:, 0])
    ids_s, w_s = O.route_topk(logits.astype(np.float64) + 3.0, k)
    np.testing.assert_array_equal(ids_s, ids)
    np.testing.assert_allclose(w_s, w, rtol=1e-12)


def test_router_bias_is_added_in_float32():
    rng = np.random.default_rng(7)
    logits = rng.standard_normal((12, 16)).astype(np.float32)
    bias = skew_bias(16)
    ids_b, w_b = O.route_topk(logits, 3, bias=bias)
    ids_r, w_r = O.route_topk((logits + bias[None, :]).astype(np.float32), 3)
    np.testing.assert_array_equal(ids_b, ids_r)
    np.testing.assert_array_equal(w_b, w_r)
    # mutation check: adding the bias in float64 instead changes at least the weights' last bits
    ids_m, w_m = O.route_topk(logits.astype(np.float64) + bias.astype(np.float64)[None, :], 3)
    assert not np.array_equal(w_m, w_b)


def test_dense_gemm_closed_form_and_independent_dequant():
    """q = z + 1 everywhere with all-ones activations gives K * s per output when the scale is
    constant along the row; random data against nibbles taken from the words' hex digits."""
    rng = np.random.default_rng(8)
    M, N, K, g = 5, 12, 64, 32
    z = rng.integers(0, 15, size=(N, K // g), dtype=np.uint8)
    q = np.repeat(z, g, axis=1) + 1
    s = np.repeat(rng.uniform(0.01, 0.02, size=(N, 1)), K // g, axis=1)
    C = O.dense_gemm(np.ones((M, K)), O.pack_int4(q), s, z, g)
    np.testing.assert_allclose(C, np.broadcast_to(K * s[:, 0], (M, N)), rtol=1e-13)
    words = rng.integers(0, 2 ** 32, size=(N, K // 8), dtype=np.uint32)
    zr = rng.integers(0, 16, size=(N, K // g), dtype=np.uint8)
    sr = O.decode_bits(to_bits(rng.uniform(0.002, 0.02, size=(N, K // g)).astype(np.float32), "f16"), "f16")
    A = O.decode_bits(to_bits((0.5 * rng.standard_normal((M, K))).astype(np.float32), "f16"), "f16")
    W = np.empty((N, K))
    for n in range(N):
        for j in range(K // 8):
            digits = f"{int(words[n, j]):08x}"[::-1]      # least significant nibble first
            for i in range(8):
                k = 8 * j + i
                W[n, k] = (int(digits[i], 16) - int(zr[n, k // g])) * sr[n, k // g]
    want = np.array([[sum(A[m, k] * W[n, k] for k in range(K)) for n in range(N)] for m in range(M)])
    np.testing.assert_allclose(O.dense_gemm(A, words.view(np.int32), sr, zr, g), want, rtol=1e-12, atol=1e-12)
    # the grouped GEMM with one expert is the same product
    Cg = O.grouped_gemm(A, 1, words.view(np.int32)[None], sr[None], zr[None], np.zeros(M, np.int32), g)
    np.testing.assert_array_equal(Cg, O.dense_gemm(A, words.view(np.int32), sr, zr, g))


@pytest.mark.parametrize("paired", [False, True])
def test_repack_is_the_documented_permutation(paired):
    """Every packed word lands exactly once; lane (n, j), word i of block (b, c) carries the eight
    weights of row r(b, n) at reduction indices 128c + 8(4j + i) .. + 7 (checked through the
    oracle's own nibble unpack of the ORIGINAL tensor); undoing the permutation with a scalar loop
    gives the original back."""
    E, N, K = 2, 64, 256
    q = np.arange(E * N * (K // 8), dtype=np.int64).reshape(E, N, K // 8).astype(np.int32)   # all words distinct
    r = O.repack_qweight(q, paired)
    assert r.shape == (E, N // 16, K // 128, 64, 4)
    assert np.array_equal(np.sort(r.reshape(-1)), np.sort(q.reshape(-1)))
    rng = np.random.default_rng(9)
    qr = rng.integers(0, 2 ** 32, size=(E, N, K // 8), dtype=np.uint32).view(np.int32)
    rr = O.repack_qweight(qr, paired)
    W = O.unpack_int4(qr)                                     # [E, N, K] nibbles of the original
    back = np.empty_like(qr)
    for e in range(E):
        for b in range(N // 16):
            for c in range(K // 128):
                for j in range(4):
                    for n in range(16):
                        row = 32 * (b // 2) + 2 * n + (b & 1) if paired else 16 * b + n
                        for i in range(4):
                            word = int(rr[e, b, c, 16 * j + n, i]) & 0xFFFFFFFF
                            k0 = 128 * c + 8 * (4 * j + i)
                            assert [(word >> (4 * t)) & 15 for t in range(8)] == list(W[e, row, k0:k0 + 8])
                            back[e, row, (k0 // 8)] = rr[e, b, c, 16 * j + n, i]
    assert np.array_equal(back, qr)


# ------------------------------------------------------------------ AWQ checkpoint import
def _awq_pack_scalar(M):
    """[R, C] integers 0..15 -> [R, C/8] words, written from the format's packing rule: word c takes,
    for p = 0..7, column 8c + (0, 2, 4, 6, 1, 3, 5, 7)[p] into bits [4p, 4p + 4)."""
    R, C = M.shape
    out = np.zeros((R, C // 8), dtype=np.uint32)
    for r in range(R):
        for c in range(C // 8):
            word = 0
            for p, col in enumerate((0, 2, 4, 6, 1, 3, 5, 7)):
                word |= int(M[r, 8 * c + col]) << (4 * p)
            out[r, c] = word
    return out.view(np.int32)


def test_import_awq_hand_vector():
    """Word 0x76543210 (nibble p holds the value p): column n of the word is the value stored at
    position (0, 4, 1, 5, 2, 6, 3, 7)[n] (the inverse of the packing order); a sequential reading
    would give 0..7."""
    K, N, g = 8, 8, 8
    words = np.full((1, K, 1), 0x76543210, dtype=np.uint32).view(np.int32)
    zw = np.full((1, 1, 1), 0xFEDCBA98, dtype=np.uint32).view(np.int32)
    sc = np.arange(8, dtype=np.float64).reshape(1, 1, 8)
    qw, s, z = O.import_awq(words, zw, sc)
    assert qw.shape == (1, 8, 1) and s.shape == (1, 8, 1) and z.shape == (1, 8, 1)
    cols = [0, 4, 1, 5, 2, 6, 3, 7]
    for n in range(8):
        assert list(O.unpack_int4(qw)[0, n]) == [cols[n]] * 8          # every k holds the same word
        assert int(z[0, n, 0]) == 8 + cols[n]
        assert s[0, n, 0] == float(n)
    assert [int(O.unpack_int4(qw)[0, n, 0]) for n in range(8)] != list(range(8))


def test_import_awq_against_scalar_pack_and_matmul():
    """Logical integer weights packed by a scalar walk of the packing rule come back transposed and
    sequential; x @ W with W taken nibble by nibble from the AWQ words (shift 4 * (0, 4, 1, 5, 2, 6,
    3, 7)[n % 8], the format's other statement) equals the oracle's GEMM on the imported tensors."""
    rng = np.random.default_rng(21)
    E, K, N, g = 2, 32, 24, 16
    Q = rng.integers(0, 16, size=(E, K, N))
    Z = rng.integers(0, 16, size=(E, K // g, N))
    S = O.rnd(rng.uniform(0.01, 0.05, size=(E, K // g, N)), "f16")
    aq = np.stack([_awq_pack_scalar(Q[e]) for e in range(E)])
    az = np.stack([_awq_pack_scalar(Z[e]) for e in range(E)])
    qw, s, z = O.import_awq(aq, az, S)
    assert qw.dtype == np.int32 and qw.shape == (E, N, K // 8) and z.dtype == np.uint8
    assert np.array_equal(O.unpack_int4(qw), np.swapaxes(Q, 1, 2))
    assert np.array_equal(z, np.swapaxes(Z, 1, 2)) and np.array_equal(s, np.swapaxes(S, 1, 2))
    shift = [4 * v for v in (0, 4, 1, 5, 2, 6, 3, 7)]
    x = O.rnd(rng.standard_normal((3, K)), "f16")
    for e in range(E):
        W = np.empty((K, N))
        for k in range(K):
            for n in range(N):
                qv = (int(aq[e, k, n // 8]) & 0xFFFFFFFF) >> shift[n % 8] & 15
                zv = (int(az[e, k // g, n // 8]) & 0xFFFFFFFF) >> shift[n % 8] & 15
                W[k, n] = (qv - zv) * S[e, k // g, n]
        np.testing.assert_allclose(O.dense_gemm(x, qw[e], s[e], z[e], g), x @ W, rtol=1e-12, atol=1e-12)


def test_skew_bias_formula():
    b = skew_bias(8)
    np.testing.assert_allclose(b, [2 * np.log(1 / (r ** 1.2)) for r in range(1, 9)], rtol=1e-6)


# ------------------------------------------------------------------ brute force on tiny shapes
@pytest.mark.parametrize("dtype,kw", [
    ("f16", {}),
    ("bf16", {}),
    ("f16", dict(T=4, K=32, N=16, E=3, topk=1, group=16, seed=11)),
    ("bf16", dict(T=2, K=16, N=16, E=4, topk=3, group=16, seed=12)),
])
def test_layer_matches_exact_rational_bruteforce(dtype, kw):
    inp = make_inputs(tiny_cfg(dtype, **kw))
    c = inp.cfg
    out, mid = oracle_layer(inp, return_intermediates=True)
    H, act, Y, outb = bf.layer(inp.x_bits.tolist(), inp.topk_ids.tolist(), inp.topk_weights.tolist(),
                               inp.qw1.tolist(), inp.s1_bits.tolist(), inp.z1.tolist(),
                               inp.qw2.tolist(), inp.s2_bits.tolist(), inp.z2.tolist(), c.group, c.dtype)
    np.testing.assert_array_equal(mid["H"], frac_to_np(H))
    np.testing.assert_array_equal(mid["act"], frac_to_np(act))
    np.testing.assert_allclose(mid["Y"], frac_to_np(Y), rtol=1e-13, atol=1e-300)   # unrounded: fp64 vs exact
    np.testing.assert_array_equal(out, frac_to_np(outb))
    # unrounded chain: float64 accumulation vs exact rationals
    out64 = oracle_layer(inp, round_intermediates=False)
    *_, outx = bf.layer(inp.x_bits.tolist(), inp.topk_ids.tolist(), inp.topk_weights.tolist(),
                        inp.qw1.tolist(), inp.s1_bits.tolist(), inp.z1.tolist(),
                        inp.qw2.tolist(), inp.s2_bits.tolist(), inp.z2.tolist(), c.group, c.dtype,
                        rounded=False)
    np.testing.assert_array_equal(out64, O.rnd(frac_to_np(outx), c.dtype))


def test_gemm_entry_matches_full_gemm_and_bruteforce():
    inp = make_inputs(tiny_cfg("f16", T=5, K=32, N=16, E=3, topk=2, group=16, seed=3))
    c = inp.cfg
    X = O.decode_bits(inp.x_bits, c.dtype)
    s1 = O.decode_bits(inp.s1_bits, c.dtype)
    se = inp.topk_ids.reshape(-1)
    full = O.grouped_gemm(X, c.topk, inp.qw1, s1, inp.z1, se, c.group, None)
    for s, n in [(0, 0), (3, 7), (9, 31), (4, 8)]:
        one = O.gemm_entry(X, c.topk, inp.qw1, s1, inp.z1, se, c.group, s, n)
        assert abs(one - full[s, n]) <= 1e-12 * max(1.0, abs(one))
        exact = sum(bf.bits_to_fraction(int(inp.x_bits[s // c.topk, k]), c.dtype) *
                    bf.weight(inp.qw1, inp.s1_bits, inp.z1, int(se[s]), n, k, c.group, c.dtype)
                    for k in range(c.K))
        assert abs(one - float(exact)) <= 1e-12 * max(1.0, abs(one))


def test_grouped_gemm_leaves_invalid_rows_at_fill():
    inp = make_inputs(tiny_cfg("f16"))
    c = inp.cfg
    se = inp.topk_ids.reshape(-1).copy()
    se[1], se[4] = -1, c.E
    C = O.grouped_gemm(O.decode_bits(inp.x_bits, c.dtype), c.topk, inp.qw1,
                       O.decode_bits(inp.s1_bits, c.dtype), inp.z1, se, c.group, c.dtype, fill=123.0)
    assert np.all(C[[1, 4]] == 123.0) and not np.any(C[[0, 2, 3, 5]] == 123.0)


# ------------------------------------------------------------------ collapse to dense library GEMMs
def independent_dense_weights(qw, s_bits, z, g, dt):
    """Dequantise through a different route than the oracle: hex digits of each word."""
    E, R, Wn = qw.shape
    q = np.empty((E, R, Wn * 8), dtype=np.float64)
    for e in range(E):
        for r in range(R):
            digits = "".join(format(int(w) & 0xFFFFFFFF, "08x")[::-1] for w in qw[e, r])
            q[e, r] = [int(ch, 16) for ch in digits]
    sv = s_bits.view(np.float16).astype(np.float64) if dt == "f16" else \
        torch.from_numpy(s_bits.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    return (q - np.repeat(z.astype(np.float64), g, axis=-1)) * np.repeat(sv, g, axis=-1)


def cast_like_library(v, dt):
    if dt == "f16":
        return v.astype(np.float16).astype(np.float64)
    # torch goes double -> float -> bf16; only used where that double rounding is harmless
    return torch.from_numpy(v).to(torch.float32).to(torch.bfloat16).double().numpy()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_one_hot_routing_reduces_to_dense_chain(dtype):
    cfg = tiny_cfg(dtype, T=6, K=32, N=16, E=3, topk=1, group=16, seed=21)
    for e_sel in range(cfg.E):
        logits = np.full((cfg.T, cfg.E), -30.0, np.float32)
        logits[:, e_sel] = 30.0
        inp = make_inputs(cfg, logits_override=logits)
        assert np.all(inp.topk_ids == e_sel) and np.all(inp.topk_weights == 1.0)
        out = oracle_layer(inp)
        W1 = independent_dense_weights(inp.qw1, inp.s1_bits, inp.z1, cfg.group, dtype)[e_sel]
        W2 = independent_dense_weights(inp.qw2, inp.s2_bits, inp.z2, cfg.group, dtype)[e_sel]
        X = cast_like_library(O.decode_bits(inp.x_bits, dtype), dtype)
        H = cast_like_library(X @ W1.T, dtype)
        gate, up = H[:, :cfg.N], H[:, cfg.N:]
        act = cast_like_library(gate / (1 + np.exp(-gate)) * up, dtype)
        want = cast_like_library(act @ W2.T, dtype)       # weight 1, one expert: out = rnd(Y)
        if dtype == "f16":
            np.testing.assert_array_equal(out, want)
        else:   # library bf16 cast double-rounds through float32: allow one bf16 ulp on rare ties
            np.testing.assert_allclose(out, want, rtol=2.0 ** -7, atol=0)
            assert np.mean(out == want) > 0.99


def test_single_expert_is_a_dense_mlp_with_topk_weights():
    cfg = tiny_cfg("f16", T=5, K=32, N=32, E=1, topk=1, group=32, seed=22)
    inp = make_inputs(cfg)
    out = oracle_layer(inp)
    W1 = independent_dense_weights(inp.qw1, inp.s1_bits, inp.z1, cfg.group, "f16")[0]
    W2 = independent_dense_weights(inp.qw2, inp.s2_bits, inp.z2, cfg.group, "f16")[0]
    X = O.decode_bits(inp.x_bits, "f16")
    H = cast_like_library(np.einsum("tk,nk->tn", X, W1), "f16")
    act = cast_like_library(H[:, :cfg.N] / (1 + np.exp(-H[:, :cfg.N])) * H[:, cfg.N:], "f16")
    Y = cast_like_library(np.einsum("tn,cn->tc", act, W2), "f16")
    np.testing.assert_array_equal(out, Y)          # softmax over one expert = weight 1


# ------------------------------------------------------------------ invariants of the whole layer
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_token_permutation_permutes_output_bit_identically(dtype):
    inp = make_inputs(tiny_cfg(dtype, T=9, K=32, N=16, E=4, topk=2, group=16, seed=31))
    c = inp.cfg
    base = oracle_layer(inp)
    perm = np.random.default_rng(0).permutation(c.T)
    X = O.decode_bits(inp.x_bits, dtype)
    out_p = O.layer(X[perm], inp.topk_ids[perm], inp.topk_weights[perm], inp.qw1,
                    O.decode_bits(inp.s1_bits, dtype), inp.z1, inp.qw2,
                    O.decode_bits(inp.s2_bits, dtype), inp.z2, c.group, dtype)
    np.testing.assert_array_equal(out_p, base[perm])
    # the token-subset form of the layer is the same thing
    np.testing.assert_array_equal(oracle_layer(inp, tokens=[7, 2]), base[[7, 2]])


def test_doubling_w2_scales_doubles_output():
    inp = make_inputs(tiny_cfg("f16", T=6, K=32, N=16, E=3, topk=2, group=16, seed=32))
    c = inp.cfg
    base = oracle_layer(inp)
    s2 = O.decode_bits(inp.s2_bits, "f16") * 2.0          # power of two: exact in fp16
    out2 = O.layer(O.decode_bits(inp.x_bits, "f16"), inp.topk_ids, inp.topk_weights, inp.qw1,
                   O.decode_bits(inp.s1_bits, "f16"), inp.z1, inp.qw2, s2, inp.z2, c.group, "f16")
    # every rounding commutes with *2 while results stay in fp16's normal range;
    # below it (spacing 2^-24) doubling may differ by one subnormal step
    normal = np.abs(base) >= 2.0 ** -13
    assert normal.mean() > 0.9
    np.testing.assert_array_equal(out2[normal], 2.0 * base[normal])
    assert np.all(np.abs(out2 - 2.0 * base) <= 2.0 ** -24)


def test_combine_topk1_identity_linearity_and_order():
    rng = np.random.default_rng(33)
    Y = O.rnd(rng.standard_normal((12, 8)) * 20, "f16")
    np.testing.assert_array_equal(O.combine(Y, np.ones((12, 1), np.float32), "f16"), Y)
    w = rng.uniform(0, 1, (4, 3)).astype(np.float32)
    a = O.combine(Y, w)
    b = O.combine(Y, (2 * w).astype(np.float32))
    np.testing.assert_array_equal(b, 2 * a)
    want = np.einsum("tj,tjc->tc", w.astype(np.float64), Y.reshape(4, 3, 8))
    np.testing.assert_allclose(a, want, rtol=1e-14)
    valid = np.ones(12, bool)
    valid[[1, 5]] = False
    w0 = w.astype(np.float64).copy().reshape(-1)
    w0[[1, 5]] = 0
    np.testing.assert_array_equal(O.combine(Y, w, slot_valid=valid),
                                  O.combine(Y, w0.reshape(4, 3)))


def test_silu_mul_closed_forms():
    H = np.array([[0.0, 1.0, -1.0, 30.0, 3.0, 2.0, 2.0, 0.5]])
    act = O.silu_mul(H)
    np.testing.assert_allclose(act[0], [0.0, 1 / (1 + np.exp(-1)) * 2, -1 / (1 + np.e) * 2, 15.0],
                               rtol=1e-12)
    big = O.silu_mul(np.array([[-800.0, 1.0]]))         # exp overflow must not produce nan
    assert big[0, 0] == 0.0


def test_invalid_expert_ids_contribute_zero():
    inp = make_inputs(tiny_cfg("f16", T=4, K=16, N=8, E=2, topk=2, group=8, seed=34))
    c = inp.cfg
    ids = inp.topk_ids.copy()
    ids[1, 0] = 7
    ids[2, 1] = -3
    X, s1, s2 = (O.decode_bits(b, "f16") for b in (inp.x_bits, inp.s1_bits, inp.s2_bits))
    got = O.layer(X, ids, inp.topk_weights, inp.qw1, s1, inp.z1, inp.qw2, s2, inp.z2, c.group, "f16")
    w = inp.topk_weights.copy()
    w[1, 0] = 0
    w[2, 1] = 0
    safe = np.where((ids >= 0) & (ids < c.E), ids, 0)
    want = O.layer(X, safe, w, inp.qw1, s1, inp.z1, inp.qw2, s2, inp.z2, c.group, "f16")
    np.testing.assert_array_equal(got, want)


# ------------------------------------------------------------------ mutation checks: the pins bite
def _bruteforce_agrees(inp) -> bool:
    c = inp.cfg
    out = oracle_layer(inp)
    *_, outb = bf.layer(inp.x_bits.tolist(), inp.topk_ids.tolist(), inp.topk_weights.tolist(),
                        inp.qw1.tolist(), inp.s1_bits.tolist(), inp.z1.tolist(),
                        inp.qw2.tolist(), inp.s2_bits.tolist(), inp.z2.tolist(), c.group, c.dtype)
    return np.array_equal(out, frac_to_np(outb))


def test_planted_mistakes_in_the_oracle_are_caught(monkeypatch):
    inp = make_inputs(tiny_cfg("f16"))
    assert _bruteforce_agrees(inp)
    real_unpack, real_dequant, real_silu, real_gemm = O.unpack_int4, O.dequant, O.silu_mul, O.grouped_gemm

    monkeypatch.setattr(O, "unpack_int4", lambda w: real_unpack(w).reshape(w.shape[:-1] + (-1, 8))[..., ::-1]
                        .reshape(w.shape[:-1] + (-1,)))               # reversed nibble order
    assert not _bruteforce_agrees(inp)
    monkeypatch.setattr(O, "unpack_int4", real_unpack)

    monkeypatch.setattr(O, "dequant", lambda q, s, z, g: real_dequant(q, s, 0 * np.asarray(z), g)
                        + np.repeat(np.asarray(z) * np.asarray(s), g, axis=-1))   # +z*s instead of -z*s
    assert not _bruteforce_agrees(inp)
    monkeypatch.setattr(O, "dequant", lambda q, s, z, g: real_dequant(
        q, np.roll(s, 1, axis=-1), z, g))                               # wrong group index
    assert not _bruteforce_agrees(inp)
    monkeypatch.setattr(O, "dequant", real_dequant)

    def swapped(H, dt=None):
        H = np.asarray(H)
        N = H.shape[1] // 2
        return real_silu(np.concatenate([H[:, N:], H[:, :N]], axis=1), dt)
    monkeypatch.setattr(O, "silu_mul", swapped)                       # gate/up swapped
    assert not _bruteforce_agrees(inp)
    monkeypatch.setattr(O, "silu_mul", real_silu)

    monkeypatch.setattr(O, "grouped_gemm", lambda A, row_div, *a, **k: real_gemm(
        np.repeat(A, row_div, axis=0)[::-1] if row_div > 1 else A, 1, *a, **k))   # wrong row map
    assert not _bruteforce_agrees(inp)
    monkeypatch.setattr(O, "grouped_gemm", real_gemm)
    assert _bruteforce_agrees(inp)


# ------------------------------------------------------------------ generator sanity
def test_generator_is_deterministic_and_shaped():
    c = CONFIGS["tiny"]
    a, b = make_inputs(c), make_inputs(c)
    for name in ("x_bits", "logits", "topk_ids", "topk_weights", "qw1", "s1_bits", "z1", "qw2", "s2_bits", "z2"):
        np.testing.assert_array_equal(getattr(a, name), getattr(b, name))
    assert a.x_bits.shape == (16, 256) and a.qw1.shape == (8, 1024, 32) and a.qw2.shape == (8, 256, 64)
    assert a.s1_bits.shape == (8, 1024, 2) and a.z2.shape == (8, 256, 4) and a.z1.max() <= 15
    s = O.decode_bits(a.s1_bits, "f16")
    assert s.min() >= 0.002 - 1e-5 and s.max() <= 0.02 + 1e-5
    q = O.unpack_int4(a.qw1)
    assert abs(q.mean() - 7.5) < 0.05 and np.bincount(q.reshape(-1), minlength=16).min() > 0
    x = O.decode_bits(a.x_bits, "f16")
    assert abs(x.std() - 0.5) < 0.02


def test_generator_bf16_cast_matches_torch():
    v = np.random.default_rng(6).standard_normal(5000).astype(np.float32)
    want = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(to_bits(v, "bf16"), want)


# ------------------------------------------------------------------ frozen fixture (regression guard)
@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_oracle_reproduces_golden_fixture(dt):
    import json
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", f"small_layer_{dt}.json")) as f:
        doc = json.load(f)
    c = doc["config"]
    cfg = MoEConfig("golden_small", T=c["T"], K=c["K"], N=c["N"], E=c["E"], topk=c["topk"],
                    group=c["group"], dtype=dt, seed=c["seed"])
    inp = make_inputs(cfg)
    np.testing.assert_array_equal(inp.topk_ids, doc["topk_ids"])
    out = oracle_layer(inp)
    np.testing.assert_array_equal(O.encode_bits(out, dt), np.array(doc["out_bits"], np.uint16))
    al = O.align_by_expert(inp.topk_ids, cfg.E, c["block_m"])
    for k, v in doc["align"].items():
        np.testing.assert_array_equal(al[k], v)
