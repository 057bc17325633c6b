"""CPU oracle for the blockwise-scaled FP8 GEMM (TEST INFRASTRUCTURE).

Plain NumPy in float64; nothing is blocked beyond what the definition itself states, nothing is
shared with the HIP path.  Only tests, the smoke check and the benchmark's cpu_baseline leg may
import this module.

Operator.  The paper lists a "blockwise scaled FP8 GEMM" among its kernels (Table II, the FP8
row for H100; Section VII-D names the serving workload that uses it; the appendix figure on
blockwise scaled FP8 GEMM layers) but does not write the operator down.  The reading used here is
the published one of the model family the paper serves (fine-grained quantisation with
1 x 128 activation tiles and 128 x 128 weight blocks):

    C[m, n] = sum over reduction blocks kb of
                  a_scale[m, kb] * b_scale[n // 128, kb] * sum_{k in block kb} A[m, k] * B[n, k]

* A [M, K], B [N, K]: 8-bit floats, format e4m3 in the OCP "fn" flavour: 1 sign, 4 exponent
  (bias 7), 3 mantissa bits; exponent field 0 is subnormal (m/8 * 2^-6); there are no infinities;
  the two codes with all exponent and mantissa bits set (0x7f, 0xff) are NaN; the largest finite
  value is 448.
* a_scale [M, K/128] float32: one scale per row and per block of 128 reduction indices.
* b_scale [ceil(N/128), K/128] float32: one scale per 128 x 128 block of B.
* C is rounded once to the 16-bit output type (bf16 by default).

The block length is a parameter (128 in the operator) so that an exact-rational brute force can
walk tiny cases.

Parity pins (tests/test_fp8_oracle_pins.py): the 256-entry decode table against a library's e4m3
cast and hand values; an exact-rational brute force on tiny shapes; unit scales => the plain
product of the decoded matrices; a closed form; linearity in one block scale (only the outputs
of that block move, by exactly that block's partial product); the grouped form against the
brute force per slot, its one-expert case (= the dense product) and the row_div gather.
"""
from __future__ import annotations

import numpy as np

from .moe_oracle import rnd

BLOCK = 128


def decode_e4m3(codes) -> np.ndarray:
    """uint8 codes -> float64 values (NaN for 0x7f / 0xff)."""
    c = np.ascontiguousarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c >= 128, -1.0, 1.0)
    e = (c >> 3) & 15
    m = c & 7
    normal = np.ldexp(1.0 + m / 8.0, (e - 7).astype(np.int64))
    sub = np.ldexp(m / 8.0, -6)
    v = np.where(e == 0, sub, normal)
    v = np.where((e == 15) & (m == 7), np.nan, v)
    return sign * v


def blockwise_gemm(a_codes, a_scale, b_codes, b_scale, out_dt="bf16", block: int = BLOCK) -> np.ndarray:
    """The operator above.  a_codes [M, K] uint8, a_scale [M, K/block], b_codes [N, K] uint8,
    b_scale [ceil(N/block), K/block].  Returns float64 values rounded to out_dt (None: unrounded)."""
    A = decode_e4m3(a_codes)
    B = decode_e4m3(b_codes)
    sa = np.asarray(a_scale, dtype=np.float64)
    sb = np.asarray(b_scale, dtype=np.float64)
    M, K = A.shape
    N = B.shape[0]
    assert B.shape[1] == K and K % block == 0
    KB = K // block
    NB = -(-N // block)
    assert sa.shape == (M, KB) and sb.shape == (NB, KB), (sa.shape, sb.shape)
    C = np.zeros((M, N), dtype=np.float64)
    for kb in range(KB):
        k0 = kb * block
        part = A[:, k0:k0 + block] @ B[:, k0:k0 + block].T           # exact in float64 (see tests)
        col_scale = np.repeat(sb[:, kb], block)[:N]                   # b_scale[n // block, kb]
        C += sa[:, kb][:, None] * col_scale[None, :] * part
    return C if out_dt is None else rnd(C, out_dt)


def grouped_blockwise_gemm(a_codes, a_scale, row_div: int, b_codes, b_scale, slot_expert,
                           out_dt="bf16", block: int = BLOCK):
    """The same product with one weight matrix per expert (the FP8 form of the paper's grouped
    mixture-of-experts GEMM, Section VII-B: one launch over all experts): slot s multiplies row
    s // row_div of A with the matrix of expert slot_expert[s],

        C[s, :] = blockwise_gemm(A[s // row_div], a_scale[s // row_div], B[e], b_scale[e]),  e = slot_expert[s].

    a_codes [R, K], a_scale [R, K/block], b_codes [E, N, K], b_scale [E, ceil(N/block), K/block],
    slot_expert [S] (ids outside [0, E) are ignored).  Returns (C [S, N] float64 values rounded to
    out_dt, rows of ignored slots zero; valid [S] bool)."""
    a_codes = np.asarray(a_codes)
    b_codes = np.asarray(b_codes)
    slot_expert = np.asarray(slot_expert)
    E, N, K = b_codes.shape
    S = slot_expert.shape[0]
    C = np.zeros((S, N), dtype=np.float64)
    valid = (slot_expert >= 0) & (slot_expert < E)
    for e in range(E):
        slots = np.nonzero(slot_expert == e)[0]
        if slots.size == 0:
            continue
        rows = slots // row_div
        C[slots] = blockwise_gemm(a_codes[rows], np.asarray(a_scale)[rows], b_codes[e], np.asarray(b_scale)[e],
                                  out_dt, block)
    return C, valid
