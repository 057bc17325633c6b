"""Scalar, exact-rational brute force of the W4A16 MoE layer for tiny shapes.

Independent of oracle/: pure Python loops over `fractions.Fraction`, nibbles
pulled out of the packed words with Python integer arithmetic, rounding to the
16-bit formats by exact rational comparison.  Used only to pin the oracle.
"""
from __future__ import annotations

import math
from fractions import Fraction

SIG = {"f16": 11, "bf16": 8}
EMIN = {"f16": -14, "bf16": -126}


def bits_to_fraction(b: int, dt: str) -> Fraction:
    """Decode a 16-bit pattern by the format definition (sign, exponent, fraction)."""
    ebits, mbits = (5, 10) if dt == "f16" else (8, 7)
    sign = -1 if (b >> 15) & 1 else 1
    e = (b >> mbits) & ((1 << ebits) - 1)
    m = b & ((1 << mbits) - 1)
    bias = (1 << (ebits - 1)) - 1
    assert e != (1 << ebits) - 1, "inf/nan not expected in inputs"
    if e == 0:
        return sign * Fraction(m, 1 << mbits) * Fraction(2) ** (1 - bias)
    return sign * (1 + Fraction(m, 1 << mbits)) * Fraction(2) ** (e - bias)


def round_fraction(x: Fraction, dt: str) -> Fraction:
    """Nearest representable value, ties to even, no overflow handling (tiny tests)."""
    if x == 0:
        return Fraction(0)
    sig, emin = SIG[dt], EMIN[dt]
    a = abs(x)
    e = 0
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    while Fraction(2) ** e > a:
        e -= 1
    qexp = max(e - (sig - 1), emin - (sig - 1))
    q = Fraction(2) ** qexp
    n = a / q
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    r = lo * q
    return r if x > 0 else -r


def nibble(word: int, i: int) -> int:
    return ((word & 0xFFFFFFFF) >> (4 * i)) & 0xF


def weight(qw, s_bits, z, e, n, k, g, dt) -> Fraction:
    q = nibble(int(qw[e][n][k // 8]), k % 8)
    return (q - int(z[e][n][k // g])) * bits_to_fraction(int(s_bits[e][n][k // g]), dt)


def bucket(topk_ids_flat, E, block_m):
    S = len(topk_ids_flat)
    valid = [s for s in range(S) if 0 <= topk_ids_flat[s] < E]
    order = sorted(valid, key=lambda s: (topk_ids_flat[s], s))
    counts = [sum(1 for s in valid if topk_ids_flat[s] == e) for e in range(E)]
    offsets = [0]
    for c in counts:
        offsets.append(offsets[-1] + (c + block_m - 1) // block_m * block_m)
    cap = (S + min(E, S) * (block_m - 1) + block_m - 1) // block_m * block_m
    sorted_ids = [S] * cap
    it = iter(order)
    for e in range(E):
        for i in range(counts[e]):
            sorted_ids[offsets[e] + i] = next(it)
    blocks = [-1] * (cap // block_m)
    for e in range(E):
        for b in range(offsets[e] // block_m, offsets[e + 1] // block_m):
            blocks[b] = e
    return counts, offsets, sorted_ids, blocks


def layer(x_bits, ids, w, qw1, s1_bits, z1, qw2, s2_bits, z2, g, dt, rounded=True):
    """Returns (H, act, Y, out) as nested lists of Fractions (floats for act/out
    when the transcendental enters)."""
    T, K = len(x_bits), len(x_bits[0])
    topk = len(ids[0])
    E, N2 = len(qw1), len(qw1[0])
    N = N2 // 2
    r = (lambda v: round_fraction(v, dt)) if rounded else (lambda v: v)
    X = [[bits_to_fraction(int(b), dt) for b in row] for row in x_bits]
    S = T * topk
    H = [[Fraction(0)] * N2 for _ in range(S)]
    act = [[Fraction(0)] * N for _ in range(S)]
    Y = [[Fraction(0)] * K for _ in range(S)]
    out = [[Fraction(0)] * K for _ in range(T)]
    for s in range(S):
        t, j = divmod(s, topk)
        e = int(ids[t][j])
        if not 0 <= e < E:
            continue
        for n in range(N2):
            acc = Fraction(0)
            for k in range(K):
                acc += X[t][k] * weight(qw1, s1_bits, z1, e, n, k, g, dt)
            H[s][n] = r(acc)
        for n in range(N):
            gate, up = float(H[s][n]), float(H[s][N + n])
            a = gate / (1.0 + math.exp(-gate)) * up
            act[s][n] = r(Fraction(a))
        for c in range(K):
            acc = Fraction(0)
            for n in range(N):
                acc += act[s][n] * weight(qw2, s2_bits, z2, e, c, n, g, dt)
            Y[s][c] = acc          # the layer combines the down projection unrounded
    for t in range(T):
        for c in range(K):
            acc = Fraction(0)
            for j in range(topk):
                e = int(ids[t][j])
                if 0 <= e < E:
                    acc += Fraction(float(w[t][j])) * Y[t * topk + j][c]
            out[t][c] = r(acc)
    return H, act, Y, out
