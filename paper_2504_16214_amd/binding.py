"""ctypes binding of libmoe_w4a16.so.  Argument marshalling only: torch tensors supply device
pointers and the current HIP stream; all arithmetic happens in the library's kernels."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # imported before the library so it binds to the HIP runtime torch already loaded

MOE_F16, MOE_BF16 = 0, 1
_STATUS = {1: "INVALID_ARGUMENT", 2: "UNSUPPORTED_SHAPE", 3: "WORKSPACE_TOO_SMALL", 4: "HIP_ERROR"}
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[ctypes.CDLL] = None

EXPORTS = [
    "moe_last_error", "moe_align_capacity", "moe_align_by_expert", "moe_w4a16_grouped_gemm",
    "moe_silu_mul", "moe_combine", "moe_w4a16_layer_workspace_bytes", "moe_w4a16_layer",
    "moe_set_stage_events", "moe_set_tile_override", "moe_set_scale_path", "moe_set_tiles_per_workgroup", "moe_set_reduction_splits", "moe_layer_block_m",
    "moe_w4a16_dense_gemm", "moe_route_topk", "moe_probe_stream_read", "moe_probe_mfma",
    "moe_w4a16_routed_layer_workspace_bytes", "moe_w4a16_routed_layer",
    "moe_repack_qweight", "moe_w4a16_layer_prepacked", "moe_import_awq",
    "fp8_blockwise_gemm_workspace_bytes", "fp8_blockwise_gemm", "fp8_moe_grouped_gemm", "fp8_set_plan_override",
    "fp8_probe_mfma", "moe_set_block_m_override", "moe_last_gemm_plan",
    "moe_w4a16_layer_noalloc", "moe_layer_block_m_for", "moe_set_wide_tiles",
    "fp8_quantize_rows", "fp8_silu_mul_quantize", "fp8_moe_layer_workspace_bytes", "fp8_moe_layer",
    "fp8_set_layer_block_m", "moe_route_align", "moe_combine_masked",
    "moe_probe_issue_mix",
]


class MoEError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


def library_path() -> str:
    """The in-tree library, or the file MOE_W4A16_LIBRARY names (e.g. the build with the sanitized
    host layer); there is no search and no fallback."""
    return os.environ.get("MOE_W4A16_LIBRARY") or os.path.join(_HERE, "libmoe_w4a16.so")


def load_library() -> ctypes.CDLL:
    """Load the in-tree HIP library; fail loudly if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2504_16214_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.moe_last_error.restype = ctypes.c_char_p
    lib.moe_last_error.argtypes = []
    lib.moe_align_capacity.restype = sz
    lib.moe_align_capacity.argtypes = [i32] * 4
    lib.moe_align_by_expert.restype = i32
    lib.moe_align_by_expert.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.moe_w4a16_grouped_gemm.restype = i32
    lib.moe_w4a16_grouped_gemm.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.moe_w4a16_dense_gemm.restype = i32
    lib.moe_w4a16_dense_gemm.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp]
    lib.moe_route_topk.restype = i32
    lib.moe_route_topk.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
    lib.moe_probe_stream_read.restype = i32
    lib.moe_probe_stream_read.argtypes = [vp, sz, vp, vp]
    lib.moe_probe_issue_mix.restype = i32
    lib.moe_probe_issue_mix.argtypes = [vp, i32, i32, i32, vp]
    lib.moe_probe_mfma.restype = i32
    lib.moe_probe_mfma.argtypes = [vp, i32, vp]
    lib.moe_w4a16_routed_layer_workspace_bytes.restype = sz
    lib.moe_w4a16_routed_layer_workspace_bytes.argtypes = [i32] * 6
    lib.moe_w4a16_routed_layer.restype = i32
    lib.moe_w4a16_routed_layer.argtypes = [vp] * 10 + [i32] * 7 + [vp, sz, vp]
    lib.moe_repack_qweight.restype = i32
    lib.moe_repack_qweight.argtypes = [vp, i32, i32, i32, i32, vp, vp]
    lib.fp8_blockwise_gemm_workspace_bytes.restype = sz
    lib.fp8_blockwise_gemm_workspace_bytes.argtypes = [i32, i32, i32]
    lib.fp8_blockwise_gemm.restype = i32
    lib.fp8_blockwise_gemm.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, sz, vp]
    lib.fp8_moe_grouped_gemm.restype = i32
    lib.fp8_moe_grouped_gemm.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.fp8_set_plan_override.restype = i32
    lib.fp8_set_plan_override.argtypes = [i32, i32, i32, i32]
    lib.fp8_probe_mfma.restype = i32
    lib.fp8_probe_mfma.argtypes = [vp, i32, vp]
    lib.moe_import_awq.restype = i32
    lib.moe_import_awq.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.moe_w4a16_layer_prepacked.restype = i32
    lib.moe_w4a16_layer_prepacked.argtypes = [vp] * 10 + [i32] * 7 + [vp, sz, vp]
    lib.moe_silu_mul.restype = i32
    lib.moe_silu_mul.argtypes = [vp, vp, i32, i32, i32, vp]
    lib.moe_combine_masked.restype = i32
    lib.moe_combine_masked.argtypes = [vp, vp, vp, i32, vp, i32, i32, i32, i32, vp]
    lib.moe_combine.restype = i32
    lib.moe_combine.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp]
    lib.moe_w4a16_layer_workspace_bytes.restype = sz
    lib.moe_w4a16_layer_workspace_bytes.argtypes = [i32] * 6
    lib.moe_w4a16_layer.restype = i32
    lib.moe_w4a16_layer.argtypes = [vp] * 10 + [i32] * 7 + [vp, sz, vp]
    lib.moe_set_stage_events.restype = i32
    lib.moe_set_stage_events.argtypes = [ctypes.POINTER(vp), i32]
    lib.moe_set_tile_override.restype = i32
    lib.moe_set_tile_override.argtypes = [i32, i32]
    lib.moe_set_scale_path.restype = i32
    lib.moe_set_scale_path.argtypes = [i32]
    lib.moe_set_tiles_per_workgroup.restype = i32
    lib.moe_set_tiles_per_workgroup.argtypes = [i32]
    lib.moe_set_reduction_splits.restype = i32
    lib.moe_set_reduction_splits.argtypes = [i32]
    lib.moe_layer_block_m.restype = i32
    lib.moe_layer_block_m.argtypes = [i32, i32, i32]
    lib.moe_w4a16_layer_noalloc.restype = i32
    lib.moe_w4a16_layer_noalloc.argtypes = [vp] * 10 + [i32] * 7 + [vp]
    lib.moe_route_align.restype = i32
    lib.moe_route_align.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.fp8_quantize_rows.restype = i32
    lib.fp8_quantize_rows.argtypes = [vp, i32, i32, i32, vp, vp, vp]
    lib.fp8_silu_mul_quantize.restype = i32
    lib.fp8_silu_mul_quantize.argtypes = [vp, i32, i32, i32, vp, vp, vp]
    lib.fp8_moe_layer_workspace_bytes.restype = sz
    lib.fp8_moe_layer_workspace_bytes.argtypes = [i32] * 5
    lib.fp8_moe_layer.restype = i32
    lib.fp8_moe_layer.argtypes = [vp] * 8 + [i32] * 6 + [vp, sz, vp]
    lib.fp8_set_layer_block_m.restype = i32
    lib.fp8_set_layer_block_m.argtypes = [i32]
    lib.moe_layer_block_m_for.restype = i32
    lib.moe_layer_block_m_for.argtypes = [i32] * 6
    lib.moe_set_wide_tiles.restype = i32
    lib.moe_set_wide_tiles.argtypes = [i32]
    lib.moe_set_block_m_override.restype = i32
    lib.moe_set_block_m_override.argtypes = [i32]
    lib.moe_last_gemm_plan.restype = i32
    lib.moe_last_gemm_plan.argtypes = [ctypes.POINTER(ctypes.c_int)]
    _LIB = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        raise MoEError(status, load_library().moe_last_error().decode())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return t.data_ptr()


def _expect(t, name: str, dtype=None, shape=None, min_numel=None) -> None:
    """Argument checks the C ABI cannot make (it sees raw pointers): raise ValueError before any
    launch on a wrong element type, a wrong shape or a buffer that is too small.  A dimension given
    as None is not checked."""
    if t is None:
        raise ValueError(f"{name}: a tensor is required")
    if dtype is not None:
        allowed = dtype if isinstance(dtype, (tuple, list)) else (dtype,)
        if t.dtype not in allowed:
            raise ValueError(f"{name}: dtype {t.dtype}, expected {' or '.join(str(d) for d in allowed)}")
    if shape is not None:
        if t.dim() != len(shape) or any(w is not None and int(g) != int(w) for g, w in zip(t.shape, shape)):
            raise ValueError(f"{name}: shape {tuple(t.shape)}, expected {tuple('*' if w is None else w for w in shape)}")
    if min_numel is not None and t.numel() < min_numel:
        raise ValueError(f"{name}: {t.numel()} elements, at least {min_numel} needed")


_F16 = (torch.float16, torch.bfloat16)


def _expect_weights(qweight, scales, zeros, group_size: int, act_dtype, what: str):
    """qweight [E, rows, red/8] int32 with scales / zeros [E, rows, red/group]."""
    _expect(qweight, f"{what} qweight", torch.int32)
    if qweight.dim() != 3:
        raise ValueError(f"{what} qweight: expected [E, rows, K/8], got shape {tuple(qweight.shape)}")
    E, rows, kw = qweight.shape
    if group_size < 1 or (kw * 8) % group_size != 0:
        return          # the library reports unsupported group sizes with its own status and message
    G = kw * 8 // group_size
    _expect(scales, f"{what} scales", act_dtype, (E, rows, G))
    _expect(zeros, f"{what} zeros", torch.uint8, (E, rows, G))


def _expect_layer(X, topk_ids, topk_weights, qw1, s1, z1, qw2, s2, z2, out, group_size):
    _expect(X, "X", _F16)
    if X.dim() != 2:
        raise ValueError(f"X: expected [T, K], got shape {tuple(X.shape)}")
    T, K = X.shape
    _expect_weights(qw1, s1, z1, group_size, X.dtype, "W1")
    E, N2, kw1 = qw1.shape
    if kw1 * 8 != K or N2 % 2 != 0:
        raise ValueError(f"W1 qweight: shape {tuple(qw1.shape)} does not match X [T, {K}] (expected [E, 2N, {K // 8}])")
    _expect_weights(qw2, s2, z2, group_size, X.dtype, "W2")
    if tuple(qw2.shape) != (E, K, N2 // 2 // 8):
        raise ValueError(f"W2 qweight: shape {tuple(qw2.shape)}, expected {(E, K, N2 // 2 // 8)}")
    if topk_ids is not None:
        _expect(topk_ids, "topk_ids", torch.int32, (T, None))
        _expect(topk_weights, "topk_weights", torch.float32, tuple(topk_ids.shape))
    _expect(out, "out", X.dtype, (T, K))


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return MOE_F16
    if t.dtype == torch.bfloat16:
        return MOE_BF16
    raise ValueError(f"fp16 or bf16 tensor expected, got {t.dtype}")


def moe_last_error() -> str:
    return load_library().moe_last_error().decode()


def moe_align_capacity(T: int, topk: int, E: int, block_m: int) -> int:
    return int(load_library().moe_align_capacity(T, topk, E, block_m))


def moe_layer_block_m(T: int, E: int, topk: int) -> int:
    return int(load_library().moe_layer_block_m(T, E, topk))


def moe_align_by_expert(topk_ids, E, block_m, expert_counts, expert_offsets, sorted_slot_ids,
                        block_expert_ids, num_padded, stream=None) -> None:
    """topk_ids [T, topk] int32; outputs are preallocated int32 device tensors."""
    _expect(topk_ids, "topk_ids", torch.int32)
    if topk_ids.dim() != 2:
        raise ValueError(f"topk_ids: expected [T, topk], got shape {tuple(topk_ids.shape)}")
    T, topk = topk_ids.shape
    cap = moe_align_capacity(T, topk, E, block_m)
    _expect(expert_counts, "expert_counts", torch.int32, min_numel=E)
    _expect(expert_offsets, "expert_offsets", torch.int32, min_numel=E + 1)
    _expect(sorted_slot_ids, "sorted_slot_ids", torch.int32, min_numel=cap)
    _expect(block_expert_ids, "block_expert_ids", torch.int32, min_numel=cap // max(block_m, 1))
    _expect(num_padded, "num_padded", torch.int32, min_numel=1)
    _check(load_library().moe_align_by_expert(_ptr(topk_ids), T, topk, E, block_m, _ptr(expert_counts),
                                              _ptr(expert_offsets), _ptr(sorted_slot_ids),
                                              _ptr(block_expert_ids), _ptr(num_padded), _stream(stream)))


def moe_w4a16_grouped_gemm(A, row_div, qweight, scales, zeros, sorted_slot_ids, block_expert_ids,
                           num_padded, num_slots, group_size, block_m, C, stream=None) -> None:
    _expect(A, "A", _F16)
    _expect_weights(qweight, scales, zeros, group_size, A.dtype, "W")
    E, N_out, kw = qweight.shape
    if A.dim() != 2 or A.shape[1] != kw * 8 or A.shape[0] * row_div < num_slots:
        raise ValueError(f"A: shape {tuple(A.shape)}, expected [>= ceil({num_slots} / {row_div}), {kw * 8}]")
    _expect(C, "C", (A.dtype,), (None, N_out), min_numel=num_slots * N_out)
    if block_m in (16, 32, 64, 128, 256):
        cap = moe_align_capacity(num_slots, 1, E, block_m)        # depends on T * topk only
        _expect(sorted_slot_ids, "sorted_slot_ids", torch.int32, min_numel=cap)
        _expect(block_expert_ids, "block_expert_ids", torch.int32, min_numel=cap // block_m)
    _expect(num_padded, "num_padded", torch.int32, min_numel=1)
    _check(load_library().moe_w4a16_grouped_gemm(
        _ptr(A), row_div, _ptr(qweight), _ptr(scales), _ptr(zeros), _ptr(sorted_slot_ids),
        _ptr(block_expert_ids), _ptr(num_padded), num_slots, E, N_out, kw * 8, group_size, block_m,
        _dt(A), _ptr(C), _stream(stream)))


def moe_w4a16_dense_gemm(A, qweight, scales, zeros, group_size, C, stream=None) -> None:
    """A [M, K] fp16/bf16, qweight [N, K/8] int32, scales [N, K/g], zeros [N, K/g] uint8, C [M, N]."""
    _expect(A, "A", _F16)
    _expect_weights(qweight[None], scales[None], zeros[None], group_size, A.dtype, "W")
    N_out, kw = qweight.shape
    _expect(A, "A", shape=(None, kw * 8))
    _expect(C, "C", (A.dtype,), (A.shape[0], N_out))
    _check(load_library().moe_w4a16_dense_gemm(_ptr(A), _ptr(qweight), _ptr(scales), _ptr(zeros), A.shape[0],
                                               N_out, kw * 8, group_size, _dt(A), _ptr(C), _stream(stream)))


def moe_route_topk(logits, bias, topk_ids, topk_weights, stream=None) -> None:
    """logits [T, E] float32, bias [E] float32 or None; outputs [T, topk] int32 / float32."""
    _expect(logits, "logits", torch.float32)
    T, E = logits.shape
    if bias is not None:
        _expect(bias, "bias", torch.float32, (E,))
    _expect(topk_ids, "topk_ids", torch.int32, (T, None))
    _expect(topk_weights, "topk_weights", torch.float32, tuple(topk_ids.shape))
    _check(load_library().moe_route_topk(_ptr(logits), _ptr(bias), T, E, topk_ids.shape[1], _ptr(topk_ids),
                                         _ptr(topk_weights), _stream(stream)))


def moe_route_align(logits, bias, block_m, topk_ids, topk_weights, expert_counts, expert_offsets, sorted_slot_ids,
                    block_expert_ids, num_padded, stream=None) -> None:
    """Router + bucketing: logits [T, E] float32 (+ bias [E] or None) -> topk_ids / topk_weights [T, topk] and
    the five tables of moe_align_by_expert (all preallocated)."""
    T, E = logits.shape
    _check(load_library().moe_route_align(_ptr(logits), _ptr(bias), T, E, topk_ids.shape[1], block_m, _ptr(topk_ids),
                                          _ptr(topk_weights), _ptr(expert_counts), _ptr(expert_offsets),
                                          _ptr(sorted_slot_ids), _ptr(block_expert_ids), _ptr(num_padded),
                                          _stream(stream)))


def moe_probe_stream_read(src, sink, stream=None) -> None:
    _check(load_library().moe_probe_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink),
                                                _stream(stream)))


def moe_probe_mfma(sink, iters: int, stream=None) -> None:
    _check(load_library().moe_probe_mfma(_ptr(sink), iters, _stream(stream)))


def moe_probe_issue_mix(sink, iters: int, valu_per_mfma: int, lds_reads_per_8_mfma: int, stream=None) -> None:
    _check(load_library().moe_probe_issue_mix(_ptr(sink), iters, valu_per_mfma, lds_reads_per_8_mfma, _stream(stream)))


def moe_silu_mul(H, act, stream=None) -> None:
    _expect(H, "H", _F16)
    S, N2 = H.shape
    _expect(act, "act", (H.dtype,), (S, N2 // 2))
    _check(load_library().moe_silu_mul(_ptr(H), _ptr(act), S, N2 // 2, _dt(H), _stream(stream)))


def moe_combine(Y, topk_weights, out, stream=None) -> None:
    _expect(topk_weights, "topk_weights", torch.float32)
    T, topk = topk_weights.shape
    _expect(Y, "Y", _F16, (T * topk, None))
    _expect(out, "out", (Y.dtype,), (T, Y.shape[1]))
    _check(load_library().moe_combine(_ptr(Y), _ptr(topk_weights), _ptr(out), T, topk, Y.shape[1], _dt(Y),
                                      _stream(stream)))


def moe_combine_masked(Y, topk_weights, topk_ids, E: int, out, stream=None) -> None:
    """moe_combine in which slots whose expert id lies outside [0, E) contribute zero."""
    _expect(topk_weights, "topk_weights", torch.float32)
    T, topk = topk_weights.shape
    _expect(topk_ids, "topk_ids", torch.int32, (T, topk))
    _expect(Y, "Y", _F16, (T * topk, None))
    _expect(out, "out", (Y.dtype,), (T, Y.shape[1]))
    _check(load_library().moe_combine_masked(_ptr(Y), _ptr(topk_weights), _ptr(topk_ids), E, _ptr(out), T, topk,
                                             Y.shape[1], _dt(Y), _stream(stream)))


def moe_w4a16_layer_workspace_bytes(T, K, N, E, topk, dt) -> int:
    return int(load_library().moe_w4a16_layer_workspace_bytes(T, K, N, E, topk, dt))


def moe_w4a16_layer(X, topk_ids, topk_weights, qw1, s1, z1, qw2, s2, z2, out, group_size, workspace,
                    stream=None) -> None:
    _expect_layer(X, topk_ids, topk_weights, qw1, s1, z1, qw2, s2, z2, out, group_size)
    _expect(workspace, "workspace", torch.uint8)
    T, K = X.shape
    E, N2, _ = qw1.shape
    topk = topk_ids.shape[1]
    _check(load_library().moe_w4a16_layer(
        _ptr(X), _ptr(topk_ids), _ptr(topk_weights), _ptr(qw1), _ptr(s1), _ptr(z1), _ptr(qw2), _ptr(s2),
        _ptr(z2), _ptr(out), T, K, N2 // 2, E, topk, group_size, _dt(X), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))


def moe_w4a16_layer_noalloc(X, topk_ids, topk_weights, qw1, s1, z1, qw2, s2, z2, out, group_size, stream=None) -> None:
    """moe_w4a16_layer on the library's built-in scratch array: no workspace, no allocation."""
    _expect_layer(X, topk_ids, topk_weights, qw1, s1, z1, qw2, s2, z2, out, group_size)
    T, K = X.shape
    E, N2, _ = qw1.shape
    topk = topk_ids.shape[1]
    _check(load_library().moe_w4a16_layer_noalloc(
        _ptr(X), _ptr(topk_ids), _ptr(topk_weights), _ptr(qw1), _ptr(s1), _ptr(z1), _ptr(qw2), _ptr(s2),
        _ptr(z2), _ptr(out), T, K, N2 // 2, E, topk, group_size, _dt(X), _stream(stream)))


def moe_w4a16_routed_layer_workspace_bytes(T, K, N, E, topk, dt) -> int:
    return int(load_library().moe_w4a16_routed_layer_workspace_bytes(T, K, N, E, topk, dt))


def moe_w4a16_routed_layer(X, logits, bias, qw1, s1, z1, qw2, s2, z2, out, topk, group_size, workspace,
                           stream=None) -> None:
    _expect_layer(X, None, None, qw1, s1, z1, qw2, s2, z2, out, group_size)
    _expect(logits, "logits", torch.float32, (X.shape[0], qw1.shape[0]))
    if bias is not None:
        _expect(bias, "bias", torch.float32, (qw1.shape[0],))
    _expect(workspace, "workspace", torch.uint8)
    T, K = X.shape
    E, N2, _ = qw1.shape
    _check(load_library().moe_w4a16_routed_layer(
        _ptr(X), _ptr(logits), _ptr(bias), _ptr(qw1), _ptr(s1), _ptr(z1), _ptr(qw2), _ptr(s2), _ptr(z2),
        _ptr(out), T, K, N2 // 2, E, topk, group_size, _dt(X), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))


def moe_repack_qweight(qweight, paired: bool, out, stream=None) -> None:
    """qweight [E, N_out, K/8] int32 -> out (same shape / size), operand-order layout."""
    E, N_out, kw = qweight.shape
    _check(load_library().moe_repack_qweight(_ptr(qweight), E, N_out, kw * 8, 1 if paired else 0, _ptr(out),
                                             _stream(stream)))


def moe_import_awq(awq_qweight, awq_qzeros, awq_scales, qweight, scales, zeros, stream=None) -> None:
    """AWQ tensors [E, K_in, N_out/8], [E, K_in/g, N_out/8], [E, K_in/g, N_out] -> qweight [E, N_out, K_in/8],
    scales [E, N_out, K_in/g], zeros [E, N_out, K_in/g] uint8 (all preallocated)."""
    E, K_in, nw = awq_qweight.shape
    G = awq_qzeros.shape[1]
    _check(load_library().moe_import_awq(_ptr(awq_qweight), _ptr(awq_qzeros), _ptr(awq_scales), E, K_in, nw * 8,
                                         K_in // G, _ptr(qweight), _ptr(scales), _ptr(zeros), _stream(stream)))


def moe_w4a16_layer_prepacked(X, topk_ids, topk_weights, qw1p, s1, z1, qw2p, s2, z2, out, group_size, workspace,
                              stream=None) -> None:
    T, K = X.shape
    E, N2 = s1.shape[0], s1.shape[1]      # s1 is [E, 2N, K/g]; the repacked weight tensors carry no shape
    topk = topk_ids.shape[1]
    _check(load_library().moe_w4a16_layer_prepacked(
        _ptr(X), _ptr(topk_ids), _ptr(topk_weights), _ptr(qw1p), _ptr(s1), _ptr(z1), _ptr(qw2p), _ptr(s2),
        _ptr(z2), _ptr(out), T, K, N2 // 2, E, topk, group_size, _dt(X), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))


def fp8_blockwise_gemm_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load_library().fp8_blockwise_gemm_workspace_bytes(M, N, K))


def fp8_blockwise_gemm(A, a_scale, B, b_scale, C, workspace=None, stream=None) -> None:
    """A [M, K] uint8 e4m3 codes, a_scale [M, K/128] float32, B [N, K] uint8, b_scale [ceil(N/128), K/128]
    float32, C [M, N] float16 / bfloat16 / float32 (preallocated); workspace: uint8 tensor of at least
    fp8_blockwise_gemm_workspace_bytes(M, N, K) bytes (None when that is 0)."""
    import torch
    M, K = A.shape
    N = B.shape[0]
    out_dtype = {torch.float16: 0, torch.bfloat16: 1, torch.float32: 2}[C.dtype]
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().fp8_blockwise_gemm(_ptr(A), _ptr(a_scale), _ptr(B), _ptr(b_scale), _ptr(C), M, N, K,
                                             out_dtype, None if workspace is None else _ptr(workspace), wb,
                                             _stream(stream)))


def fp8_moe_grouped_gemm(A, a_scale, row_div: int, B, b_scale, sorted_slot_ids, block_expert_ids, num_padded,
                         num_slots: int, block_m: int, C, stream=None) -> None:
    """A [rows_A, K] uint8, a_scale [rows_A, K/128] float32, B [E, N, K] uint8, b_scale [E, ceil(N/128), K/128],
    slot tables from moe_align_by_expert, C [num_slots, N] float16 / bfloat16 (preallocated)."""
    import torch
    E, N, K = B.shape
    out_dtype = {torch.float16: 0, torch.bfloat16: 1, torch.float32: 2}[C.dtype]
    _check(load_library().fp8_moe_grouped_gemm(_ptr(A), _ptr(a_scale), row_div, _ptr(B), _ptr(b_scale),
                                               _ptr(sorted_slot_ids), _ptr(block_expert_ids), _ptr(num_padded),
                                               num_slots, E, N, K, block_m, out_dtype, _ptr(C), _stream(stream)))


def fp8_quantize_rows(X, codes, scales, stream=None) -> None:
    """X [rows, K] fp16/bf16 -> codes [rows, K] uint8 (e4m3), scales [rows, K/128] float32 (preallocated)."""
    rows, K = X.shape
    _check(load_library().fp8_quantize_rows(_ptr(X), rows, K, _dt(X), _ptr(codes), _ptr(scales), _stream(stream)))


def fp8_silu_mul_quantize(H, codes, scales, stream=None) -> None:
    """H [S, 2N] fp16/bf16 -> e4m3 codes [S, N] and scales [S, N/128] of round(silu(gate) * up)."""
    S, N2 = H.shape
    _check(load_library().fp8_silu_mul_quantize(_ptr(H), S, N2 // 2, _dt(H), _ptr(codes), _ptr(scales), _stream(stream)))


def fp8_moe_layer_workspace_bytes(T: int, K: int, N: int, E: int, topk: int) -> int:
    return int(load_library().fp8_moe_layer_workspace_bytes(T, K, N, E, topk))


def fp8_moe_layer(X, topk_ids, topk_weights, w1, w1_scale, w2, w2_scale, out, workspace, stream=None) -> None:
    """X [T, K] fp16/bf16, w1 [E, 2N, K] uint8 + w1_scale [E, 2N/128, K/128] float32, w2 [E, K, N] uint8 +
    w2_scale [E, K/128, N/128], out [T, K] (preallocated), workspace uint8 tensor."""
    T, K = X.shape
    E, N2, _ = w1.shape
    topk = topk_ids.shape[1]
    _check(load_library().fp8_moe_layer(
        _ptr(X), _ptr(topk_ids), _ptr(topk_weights), _ptr(w1), _ptr(w1_scale), _ptr(w2), _ptr(w2_scale), _ptr(out),
        T, K, N2 // 2, E, topk, _dt(X), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def fp8_set_layer_block_m(block_m: int) -> None:
    _check(load_library().fp8_set_layer_block_m(block_m))


def fp8_set_plan_override(mt: int, nt: int, k_splits: int, group_m: int = 0) -> None:
    _check(load_library().fp8_set_plan_override(mt, nt, k_splits, group_m))


def fp8_probe_mfma(sink, iters: int, stream=None) -> None:
    _check(load_library().fp8_probe_mfma(_ptr(sink), iters, _stream(stream)))


def moe_set_tile_override(mt: int, nt: int) -> None:
    _check(load_library().moe_set_tile_override(mt, nt))


def moe_layer_block_m_for(T: int, K: int, N: int, E: int, topk: int, group_size: int) -> int:
    return int(load_library().moe_layer_block_m_for(T, K, N, E, topk, group_size))


def moe_set_wide_tiles(mode: int) -> None:
    _check(load_library().moe_set_wide_tiles(mode))


def moe_set_block_m_override(block_m: int) -> None:
    _check(load_library().moe_set_block_m_override(block_m))


def moe_last_gemm_plan() -> dict:
    """The tile plan of the last grouped / dense GEMM launched from this thread."""
    arr = (ctypes.c_int * 9)()
    _check(load_library().moe_last_gemm_plan(arr))
    keys = ("mt", "nt", "ks", "register_scales", "tiles_per_workgroup", "reduction_splits", "k_span", "fused", "waves")
    return dict(zip(keys, (int(v) for v in arr)))


def moe_set_scale_path(mode: int) -> None:
    _check(load_library().moe_set_scale_path(mode))


def moe_set_tiles_per_workgroup(n: int) -> None:
    _check(load_library().moe_set_tiles_per_workgroup(n))


def moe_set_reduction_splits(n: int) -> None:
    _check(load_library().moe_set_reduction_splits(n))


def moe_set_stage_events(events) -> None:
    """events: sequence of 5 raw hipEvent_t handles (ints), or None to clear."""
    lib = load_library()
    if not events:
        _check(lib.moe_set_stage_events(None, 0))
        return
    arr = (ctypes.c_void_p * len(events))(*events)
    _check(lib.moe_set_stage_events(arr, len(events)))
