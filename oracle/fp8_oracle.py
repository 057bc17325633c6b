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

The FP8 mixture-of-experts layer (`moe_layer`) puts that grouped product on both projections of
the gated expert MLP, with the activations quantised on the fly the way the same published scheme
does it: per row and per 128 reduction indices, scale = max(|x|) / 448 (the maximum clamped from
below at 1e-4), code = e4m3(x * (448 / max)), all of it in float32 (`quantize_rows`).

Parity pins (tests/test_fp8_oracle_pins.py): the 256-entry decode table against a library's e4m3
cast and hand values; an exact-rational brute force on tiny shapes; unit scales => the plain
product of the decoded matrices; a closed form; linearity in one block scale (only the outputs
of that block move, by exactly that block's partial product); the grouped form against the
brute force per slot, its one-expert case (= the dense product) and the row_div gather.
"""
from __future__ import annotations

import numpy as np

from .moe_oracle import combine, rnd, silu_mul

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


# --------------------------------------------------------------------------
# activation quantisation (1 x 128 tiles) and the FP8 mixture-of-experts layer
# --------------------------------------------------------------------------
E4M3_MAX = 448.0
AMAX_FLOOR = np.float32(1e-4)      # lower clamp of a tile's maximum (keeps an all-zero tile finite)


def encode_e4m3(values) -> np.ndarray:
    """Round-to-nearest-even of real values to e4m3 ("fn": bias 7, subnormal spacing 2^-9, no
    infinities), returned as uint8 codes.  Magnitudes that would round beyond 448 saturate to 448
    (the quantiser below never produces them: its inputs are at most 448 up to one float32
    rounding); NaN gives 0x7f."""
    y = np.asarray(values, dtype=np.float64)
    a = np.where(np.isnan(y), 0.0, np.abs(y))
    _, e = np.frexp(a)                                   # a = m * 2**e, m in [0.5, 1)
    qexp = np.maximum(e - 4, -9)                         # spacing 2**(e-1-3), floored at the subnormal one
    q = np.ldexp(1.0, qexp)
    r = np.rint(a / q) * q                               # ties to even; a / q is exact
    r = np.minimum(r, E4M3_MAX)
    _, er = np.frexp(r)                                  # r = mr * 2**er
    normal = r >= 2.0 ** -6
    efield = np.where(normal, er - 1 + 7, 0)
    mant = np.where(normal, np.rint((r / np.ldexp(1.0, er - 1) - 1.0) * 8.0), np.rint(r * 2.0 ** 9))
    code = (efield.astype(np.int64) << 3) | mant.astype(np.int64)
    code = np.where(np.signbit(y), code | 0x80, code)
    code = np.where(np.isnan(y), 0x7F, code)
    return code.astype(np.uint8)


def quantize_rows(x, block: int = BLOCK):
    """x [R, K] values of a 16-bit float type (float64 array) -> (codes [R, K] uint8, scale
    [R, K/block] float32), one scale per row and block of reduction indices, in float32 exactly as
    stated:  m = max(max|x| over the tile, 1e-4);  scale = m / 448;  code = e4m3(x * (448 / m))
    (one float32 division for 448 / m, one float32 product per element, one float32 division for
    the scale).  decode(code) * scale reproduces x to within half an e4m3 step."""
    x32 = np.asarray(x, dtype=np.float64).astype(np.float32)      # exact: 16-bit values
    R, K = x32.shape
    assert K % block == 0
    t = x32.reshape(R, K // block, block)
    m = np.maximum(np.abs(t).max(axis=2), AMAX_FLOOR).astype(np.float32)
    r = (np.float32(E4M3_MAX) / m).astype(np.float32)
    y = (t * r[:, :, None]).astype(np.float32)
    scale = (m / np.float32(E4M3_MAX)).astype(np.float32)
    return encode_e4m3(y.astype(np.float64)).reshape(R, K), scale


def moe_layer(X, topk_ids, topk_weights, w1_codes, w1_scale, w2_codes, w2_scale, dt: str,
              tokens=None, return_intermediates: bool = False, block: int = BLOCK):
    """The gated expert MLP with FP8 weights and on-the-fly FP8 activations:

        out[t] = sum_j w[t, j] * W2[e] . q( silu(W1g[e] . q(x_t)) * (W1u[e] . q(x_t)) ),   e = topk_ids[t, j]

    X [T, K] values of dt; W1 codes [E, 2N, K] (rows [0, N) gate, [N, 2N) up) with block scales
    [E, 2N/128, K/128]; W2 codes [E, K, N] with [E, K/128, N/128] (`block` replaces 128 so that a
    brute force can walk tiny cases).  q() is quantize_rows; both
    products are grouped_blockwise_gemm.  Rounding points as in the 16-bit layer: the gate/up
    product H and the activation are rounded to dt (the activation is a 16-bit tensor before it is
    quantised), the down projection goes into the weighted combine unrounded, the result is
    rounded once.  Slots with an expert id outside [0, E) contribute zero."""
    X = np.asarray(X, dtype=np.float64)
    ids = np.asarray(topk_ids)
    w = np.asarray(topk_weights)
    if tokens is not None:
        tokens = np.asarray(tokens, dtype=np.int64)
        X, ids, w = X[tokens], ids[tokens], w[tokens]
    T, topk = ids.shape
    slot_expert = ids.reshape(-1)
    xq, sx = quantize_rows(X, block)
    H, valid = grouped_blockwise_gemm(xq, sx, topk, w1_codes, w1_scale, slot_expert, out_dt=dt, block=block)
    act = silu_mul(H, dt)
    aq, sa = quantize_rows(act, block)
    Y, _ = grouped_blockwise_gemm(aq, sa, 1, w2_codes, w2_scale, slot_expert, out_dt=None, block=block)
    out = combine(Y, w, dt, slot_valid=valid)
    if return_intermediates:
        return out, {"xq": xq, "sx": sx, "H": H, "act": act, "aq": aq, "sa": sa, "Y": Y}
    return out
