"""CPU oracle for the W4A16 mixture-of-experts layer (TEST INFRASTRUCTURE).

Plain, slow, obviously-correct NumPy: explicit nibble unpack, exact
dequantisation, float64 matmuls, explicit rounding to the 16-bit storage type
at the tensors the staged interface materialises (H, act, Y, out; the whole-layer
form keeps Y unrounded, see `layer`), and a float64 weighted combine.  Nothing here is blocked, fused or reordered, and
nothing is shared with the HIP path.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import this module; the product path must
never route through it.

Operator definition.  The paper's mixed-type MoE evaluation (Section VII-B,
"Mixed-type MoE", Table III) fixes only the operand set A (fp16 activations),
B (int4 weights), scale and zp, and the FP16xINT4 semantics of Section II-C /
Fig. 4(b) (weights are cast to the activation type and contracted on the
matrix units).  The remaining choices follow the benchmark statement:

* int4 packing: eight unsigned nibbles per 32-bit word, element 8j+i of a row
  sits in bits [4i, 4i+4) of word j (sequential order, little-endian
  significance).
* group-wise asymmetric quantisation along the reduction (last) dimension:
  W[n, k] = (q[n, k] - z[n, k // g]) * s[n, k // g].
* W1 [E, 2N, K]: rows [0, N) are the gate projection (goes through SiLU),
  rows [N, 2N) the up projection.  W2 [E, K, N] is the down projection.
* slot s = t * topk + j is routed to expert topk_ids[t, j]; ids outside
  [0, E) are ignored (not bucketed, contribute zero to the output).

Every floating tensor is handled in "value space": float64 arrays whose values
are exactly representable in the 16-bit type.  `decode_bits` / `encode_bits`
move between value space and raw uint16 patterns.

Parity pins (tests/test_oracle_*.py): exact rational brute force on tiny
shapes, pack/unpack round trip and the 0x76543210 vector, all-zero nibbles
=> -z*s, one-hot routing => dense GEMM chain, E=1 => dense MLP, top-k weights
sum to one, top-k against a scalar selection loop and (k = E) a library softmax,
the dense GEMM against a closed form and an independent dequantisation,
token permutation equivariance (bit-identical), W2-scale doubling
doubles the output, combine linearity, rounding against NumPy's fp16 cast,
PyTorch's bf16 cast and hand-derived tie cases, the AWQ import against a scalar
walk of the format definition and the x @ W it defines.  The paper prints no worked
numeric example for this operator, so there is no paper-valued fixture.
"""
from __future__ import annotations

import numpy as np

_FORMATS = {
    # name: (significand bits incl. hidden one, min normal exponent, max finite value)
    "f16": (11, -14, 65504.0),
    "bf16": (8, -126, float.fromhex("0x1.fep127")),
}


# --------------------------------------------------------------------------
# 16-bit storage formats
# --------------------------------------------------------------------------
def rnd(x, dt: str) -> np.ndarray:
    """IEEE round-to-nearest-even of float64 values to fp16 / bf16, returned as
    float64 (value space).  Rounds once, straight from float64."""
    sig, emin, vmax = _FORMATS[dt]
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    _, e = np.frexp(a)                      # a = m * 2**e, m in [0.5, 1)
    # spacing of representable numbers around a: 2**(e - sig), floored at the subnormal spacing
    qexp = np.maximum(e - sig, emin - (sig - 1))
    q = np.ldexp(1.0, qexp)
    r = np.rint(a / q) * q                  # rint = ties to even; a / q is exact (power of two)
    # overflow: at or beyond (largest finite + half an ulp of the top binade) rounds to inf
    half_ulp_top = np.ldexp(1.0, int(np.frexp(vmax)[1]) - sig - 1)
    r = np.where(a >= vmax + half_ulp_top, np.inf, r)
    r = np.where(np.isnan(x), np.nan, r)
    return np.copysign(r, x)


def decode_bits(bits, dt: str) -> np.ndarray:
    """uint16 bit patterns -> float64 values."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    if dt == "f16":
        return b.view(np.float16).astype(np.float64)
    if dt == "bf16":
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dt)


def encode_bits(values, dt: str) -> np.ndarray:
    """float64 values already representable in dt -> uint16 bit patterns."""
    v = rnd(values, dt)
    if dt == "f16":
        return v.astype(np.float16).view(np.uint16)
    if dt == "bf16":
        return (v.astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dt)


# --------------------------------------------------------------------------
# int4 packing and dequantisation
# --------------------------------------------------------------------------
def unpack_int4(words) -> np.ndarray:
    """[..., W] 32-bit words -> [..., 8W] uint8 nibbles; element 8j+i = bits [4i,4i+4) of word j."""
    w = np.ascontiguousarray(words).view(np.uint32)
    out = np.empty(w.shape + (8,), dtype=np.uint8)
    for i in range(8):
        out[..., i] = (w >> np.uint32(4 * i)) & np.uint32(0xF)
    return out.reshape(w.shape[:-1] + (w.shape[-1] * 8,))


def pack_int4(q) -> np.ndarray:
    """Inverse of unpack_int4: [..., 8W] values 0..15 -> [..., W] int32 words."""
    q = np.asarray(q)
    assert q.shape[-1] % 8 == 0 and q.min(initial=0) >= 0 and q.max(initial=0) <= 15
    q8 = q.reshape(q.shape[:-1] + (q.shape[-1] // 8, 8)).astype(np.uint32)
    w = np.zeros(q8.shape[:-1], dtype=np.uint32)
    for i in range(8):
        w |= q8[..., i] << np.uint32(4 * i)
    return w.view(np.int32)


def dequant(qweight, scales, zeros, group: int) -> np.ndarray:
    """W[..., n, k] = (q - z[..., n, k//g]) * s[..., n, k//g] in float64 (exact:
    |q - z| <= 15 and the scale has at most 11 significant bits).

    qweight [..., rows, red/8] words, scales [..., rows, red/g] float64 values,
    zeros [..., rows, red/g] integers 0..15."""
    q = unpack_int4(qweight)
    zeros = np.asarray(zeros)
    scales = np.asarray(scales, dtype=np.float64)
    G = zeros.shape[-1]
    assert q.shape[-1] == G * group and scales.shape == zeros.shape, (q.shape, zeros.shape, scales.shape)
    qg = q.reshape(q.shape[:-1] + (G, group)).astype(np.int16)
    d = qg - zeros.astype(np.int16)[..., None]                  # integer q - z, |d| <= 15
    W = d.astype(np.float64) * scales[..., None]
    return W.reshape(q.shape)


# --------------------------------------------------------------------------
# offline weight repack (a permutation of 16-byte chunks, no arithmetic)
# --------------------------------------------------------------------------
def repack_qweight(qweight, paired: bool) -> np.ndarray:
    """Packed weights [E, N_out, K_in/8] int32 -> the operand-order layout
    [E, N_out/16, K_in/128, 64, 4] int32 the prepacked kernels stream.

    The matrix is cut into blocks of 16 feature rows x 128 reduction indices (64 packed bytes per
    row).  Block (b, c) of an expert is stored as 64 consecutive 16-byte chunks; chunk 16*j + n
    holds bytes [64*c + 16*j, 64*c + 16*j + 16) of the block's row n (j = 0..3, n = 0..15), which
    is what lane 16*j + n of a wave feeds to its four matrix instructions of that step.  Blocks
    of one row set follow each other along the reduction, row sets follow each other.

    paired = False: row set b is rows 16*b .. 16*b + 15 (gate/up weights).
    paired = True : row sets come in pairs over runs of 32 rows, set 2*q taking the even and
    set 2*q + 1 the odd rows of rows 32*q .. 32*q + 31 (down-projection weights: a lane then owns
    two adjacent output columns).  Needs N_out % 32 == 0."""
    q = np.ascontiguousarray(qweight)
    E, N_out, KW = q.shape
    K_in = 8 * KW
    assert K_in % 128 == 0 and N_out % (32 if paired else 16) == 0
    out = np.empty((E, N_out // 16, K_in // 128, 64, 4), dtype=np.int32)
    for b in range(N_out // 16):
        if paired:
            rows = [32 * (b // 2) + 2 * n + (b & 1) for n in range(16)]
        else:
            rows = [16 * b + n for n in range(16)]
        for c in range(K_in // 128):
            for j in range(4):
                for n in range(16):
                    out[:, b, c, 16 * j + n, :] = q[:, rows[n], 16 * c + 4 * j: 16 * c + 4 * j + 4]
    return out


# --------------------------------------------------------------------------
# import of AWQ-packed checkpoints (a permutation of nibbles / elements, no arithmetic)
# --------------------------------------------------------------------------
# The paper's layer comes from an AWQ checkpoint (Section VII-B, VII-D).  The publicly documented
# AWQ "GEMM" tensor format stores a linear layer y = x @ W, W [in, out], as
#   qweight [in, out/8] int32, qzeros [in/g, out/8] int32, scales [in/g, out] (16-bit float),
# each word holding eight neighbouring OUTPUT columns, and not in sequential order: the nibble
# at bits [4p, 4p+4) of word c is column 8c + AWQ_NIBBLE_COLUMN[p].  W[k, n] = (q[k, n] -
# z[k // g, n]) * s[k // g, n].
AWQ_NIBBLE_COLUMN = (0, 2, 4, 6, 1, 3, 5, 7)


def import_awq(awq_qweight, awq_qzeros, awq_scales):
    """AWQ-format tensors of E linear layers -> this library's format.

    awq_qweight [E, K_in, N_out/8] words, awq_qzeros [E, K_in/g, N_out/8] words, awq_scales
    [E, K_in/g, N_out] (any array; moved as is).  Returns (qweight [E, N_out, K_in/8] int32 in
    sequential nibble order along the reduction, scales [E, N_out, K_in/g], zeros
    [E, N_out, K_in/g] uint8): the same q, z and s, transposed so that the reduction index is
    the contiguous one."""
    wq = np.ascontiguousarray(awq_qweight).view(np.uint32)
    wz = np.ascontiguousarray(awq_qzeros).view(np.uint32)
    sc = np.asarray(awq_scales)
    E, K_in, NW = wq.shape
    N_out = 8 * NW
    G = wz.shape[1]
    assert wz.shape == (E, G, NW) and sc.shape == (E, G, N_out) and K_in % 8 == 0
    q = np.empty((E, K_in, N_out), dtype=np.uint8)       # logical integer weights [e, k, n]
    z = np.empty((E, G, N_out), dtype=np.uint8)
    for p in range(8):
        col = AWQ_NIBBLE_COLUMN[p]
        q[:, :, col::8] = (wq >> np.uint32(4 * p)) & np.uint32(0xF)
        z[:, :, col::8] = (wz >> np.uint32(4 * p)) & np.uint32(0xF)
    qweight = pack_int4(np.swapaxes(q, 1, 2))             # [E, N_out, K_in] -> words along k
    return qweight, np.ascontiguousarray(np.swapaxes(sc, 1, 2)), np.ascontiguousarray(np.swapaxes(z, 1, 2))


# --------------------------------------------------------------------------
# routing weights (input preparation; kept here to pin the generator's router)
# --------------------------------------------------------------------------
def route_topk(logits, topk: int, bias=None):
    """Top-k experts per token (descending logit, ties to the lower index) and the
    full softmax renormalised over the selected experts, in float64.

    `bias` [E] (optional) is added to every token's logits first, in float32 with one
    rounding per element (router logits and the per-expert bias are float32 tensors);
    everything after that is exact comparisons and float64 arithmetic."""
    if bias is not None:
        logits = np.asarray(logits, dtype=np.float32) + np.asarray(bias, dtype=np.float32)[None, :]
    logits = np.asarray(logits, dtype=np.float64)
    T, E = logits.shape
    ids = np.empty((T, topk), dtype=np.int32)
    w = np.empty((T, topk), dtype=np.float64)
    for t in range(T):
        full = np.exp(logits[t] - logits[t].max())
        full /= full.sum()
        order = sorted(range(E), key=lambda e: (-logits[t, e], e))[:topk]
        ids[t] = order
        w[t] = full[order] / full[order].sum()
    return ids, w


# --------------------------------------------------------------------------
# step 1: expert bucketing
# --------------------------------------------------------------------------
def align_capacity(T: int, topk: int, E: int, block_m: int) -> int:
    S = T * topk
    worst = S + min(E, S) * (block_m - 1)
    return -(-worst // block_m) * block_m


def align_by_expert(topk_ids, E: int, block_m: int) -> dict:
    """Stable counting sort of the T*topk slots by expert, each non-empty expert
    padded to a multiple of block_m.  All outputs int32.

    expert_counts[e]   number of slots routed to e (unpadded)
    expert_offsets     exclusive prefix sum of the padded counts, length E+1
    sorted_slot_ids    [capacity]; segment e holds its slots in ascending slot
                       order, then the sentinel S; everything past num_padded is S
    block_expert_ids   [capacity/block_m]; expert owning each block, -1 past the end
    num_padded         expert_offsets[E]
    """
    ids = np.asarray(topk_ids, dtype=np.int64).reshape(-1)
    S = ids.size
    T_topk_cap = -(-(S + min(E, S) * (block_m - 1)) // block_m) * block_m
    counts = np.zeros(E, dtype=np.int64)
    for e in range(E):
        counts[e] = int(np.count_nonzero(ids == e))
    padded = -(-counts // block_m) * block_m
    offsets = np.concatenate([[0], np.cumsum(padded)])
    sorted_ids = np.full(T_topk_cap, S, dtype=np.int64)
    block_e = np.full(T_topk_cap // block_m, -1, dtype=np.int64)
    for e in range(E):
        slots = np.nonzero(ids == e)[0]           # ascending slot id
        sorted_ids[offsets[e]:offsets[e] + slots.size] = slots
        block_e[offsets[e] // block_m: offsets[e + 1] // block_m] = e
    return {
        "expert_counts": counts.astype(np.int32),
        "expert_offsets": offsets.astype(np.int32),
        "sorted_slot_ids": sorted_ids.astype(np.int32),
        "block_expert_ids": block_e.astype(np.int32),
        "num_padded": np.array([offsets[-1]], dtype=np.int32),
    }


# --------------------------------------------------------------------------
# steps 2 and 4: grouped W4A16 GEMM
# --------------------------------------------------------------------------
def grouped_gemm(A, row_div: int, qweight, scales, zeros, slot_expert, group: int,
                 dt=None, fill=np.nan) -> np.ndarray:
    """C[s, n] = sum_k A[s // row_div, k] * W[e_s, n, k],  e_s = slot_expert[s].

    A [rows, K_in] float64 values; qweight [E, N_out, K_in/8]; scales float64
    values [E, N_out, K_in/g]; zeros [E, N_out, K_in/g].  Accumulates in
    float64 and rounds once to dt (dt=None keeps float64).  Rows of slots whose
    expert id is outside [0, E) are left at `fill` (the HIP entry point leaves
    such rows untouched)."""
    A = np.asarray(A, dtype=np.float64)
    slot_expert = np.asarray(slot_expert).reshape(-1)
    E, N_out = qweight.shape[0], qweight.shape[1]
    S = slot_expert.size
    C = np.full((S, N_out), fill, dtype=np.float64)
    for e in range(E):
        slots = np.nonzero(slot_expert == e)[0]
        if slots.size == 0:
            continue
        W = dequant(qweight[e], scales[e], zeros[e], group)       # [N_out, K_in]
        C[slots] = A[slots // row_div] @ W.T
    if dt is not None:
        C = np.where(np.isnan(C), C, rnd(C, dt))
    return C


def dense_gemm(A, qweight, scales, zeros, group: int, dt=None) -> np.ndarray:
    """The plain FP16xINT4 GEMM of Section II-C / Fig. 4(b): C = A @ W^T with
    W[n, k] = (q[n, k] - z[n, k // g]) * s[n, k // g].  A [M, K] float64 values,
    qweight [N, K/8], scales float64 values [N, K/g], zeros [N, K/g].  float64
    accumulation, one rounding to dt (None keeps float64)."""
    W = dequant(qweight, scales, zeros, group)                    # [N, K]
    C = np.asarray(A, dtype=np.float64) @ W.T
    return C if dt is None else rnd(C, dt)


def gemm_entry(A, row_div: int, qweight, scales, zeros, slot_expert, group: int,
               s: int, n: int) -> float:
    """One output element of grouped_gemm, unrounded, by the definition (used to
    sample outputs at sizes where the full product is too slow)."""
    e = int(np.asarray(slot_expert).reshape(-1)[s])
    W = dequant(qweight[e, n:n + 1], np.asarray(scales)[e, n:n + 1], zeros[e, n:n + 1], group)[0]
    return float(np.dot(np.asarray(A, dtype=np.float64)[s // row_div], W))


# --------------------------------------------------------------------------
# step 3: SiLU-and-multiply, step 5: combine
# --------------------------------------------------------------------------
def silu_mul(H, dt=None) -> np.ndarray:
    """act[s, n] = silu(H[s, n]) * H[s, N + n], silu(x) = x / (1 + exp(-x))."""
    H = np.asarray(H, dtype=np.float64)
    N = H.shape[1] // 2
    g, u = H[:, :N], H[:, N:]
    with np.errstate(over="ignore"):
        act = g / (1.0 + np.exp(-g)) * u
    return rnd(act, dt) if dt is not None else act


def combine(Y, topk_weights, dt=None, slot_valid=None) -> np.ndarray:
    """out[t, c] = sum_j w[t, j] * Y[t*topk + j, c], summed in j order in float64.
    Slots flagged invalid contribute zero."""
    w = np.asarray(topk_weights, dtype=np.float64)
    T, topk = w.shape
    Y = np.asarray(Y, dtype=np.float64).reshape(T, topk, -1)
    out = np.zeros((T, Y.shape[2]), dtype=np.float64)
    for j in range(topk):
        term = w[:, j:j + 1] * Y[:, j, :]
        if slot_valid is not None:
            ok = np.asarray(slot_valid).reshape(T, topk)[:, j:j + 1]
            term = np.where(ok, term, 0.0)
        out += term
    return rnd(out, dt) if dt is not None else out


# --------------------------------------------------------------------------
# whole layer
# --------------------------------------------------------------------------
def layer(X, topk_ids, topk_weights, qw1, s1, z1, qw2, s2, z2, group: int, dt: str,
          round_intermediates: bool = True, tokens=None, return_intermediates: bool = False):
    """The full layer for all tokens, or for the subset `tokens` (each token's
    output depends on no other token, so the restriction is the definition
    applied to fewer rows).  X, s1, s2 are float64 values; output float64 values
    rounded to dt.

    Rounding points of the whole layer: H and act are rounded to dt (they are
    the 16-bit operands the second mixed-type GEMM consumes: A is fp16/bf16 by
    the operator's definition, Table III), the result `out` is rounded to dt.
    The down projection Y is NOT rounded inside the layer: it goes into the
    weighted combine at full precision and the sum is rounded once.  (The paper
    does not state rounding points.  Rounding Y first would put a 16-bit ulp of
    |Y| ~ 64..128, i.e. 0.03..0.06, times the routing weight into `out`, which
    is larger than the 2e-2 absolute acceptance bound whenever two correct
    implementations round a near-tie differently; the staged grouped_gemm entry
    point still rounds its own output.)  round_intermediates=False also keeps H
    and act in float64."""
    X = np.asarray(X, dtype=np.float64)
    ids = np.asarray(topk_ids)
    w = np.asarray(topk_weights)
    if tokens is not None:
        tokens = np.asarray(tokens, dtype=np.int64)
        X, ids, w = X[tokens], ids[tokens], w[tokens]
    T, topk = ids.shape
    E = qw1.shape[0]
    mid = dt if round_intermediates else None
    slot_expert = ids.reshape(-1)
    valid = (slot_expert >= 0) & (slot_expert < E)
    H = grouped_gemm(X, topk, qw1, s1, z1, slot_expert, group, mid, fill=0.0)
    act = silu_mul(H, mid)
    Y = grouped_gemm(act, 1, qw2, s2, z2, slot_expert, group, None, fill=0.0)
    out = combine(Y, w, dt, slot_valid=valid)
    if return_intermediates:
        return out, {"H": H, "act": act, "Y": Y}
    return out
