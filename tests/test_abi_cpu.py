"""CPU-only checks of the C ABI: the in-tree library loads, exports every function the
header declares, and its host logic (capacity, workspace sizing, block choice, argument
validation that happens before any launch) behaves as documented.  No kernel is launched."""
from __future__ import annotations

import ctypes
import os
import re

import pytest

from oracle import moe_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", n) for n in ("moe_w4a16.h", "fp8_blockwise_gemm.h")]


@pytest.fixture(scope="module")
def binding():
    import paper_2504_16214_amd.binding as b
    if not os.path.exists(b.library_path()):
        from paper_2504_16214_amd.build import build
        build(verbose=False)
    b.load_library()
    return b


def declared_functions():
    text = "".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:moe|fp8)_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_five_entry_points():
    names = declared_functions()
    for n in ("moe_align_by_expert", "moe_w4a16_grouped_gemm", "moe_silu_mul", "moe_combine", "moe_w4a16_layer"):
        assert n in names


def test_library_exports_every_declared_symbol(binding):
    lib = ctypes.CDLL(binding.library_path())
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in the header but not exported"
    assert sorted(binding.EXPORTS) == declared_functions()


@pytest.mark.parametrize("T,topk,E,bm", [(16, 2, 8, 16), (128, 8, 256, 16), (4096, 8, 256, 128), (1, 1, 1, 256),
                                         (0, 2, 4, 16), (3, 2, 1000, 64)])
def test_capacity_matches_oracle(binding, T, topk, E, bm):
    assert binding.moe_align_capacity(T, topk, E, bm) == O.align_capacity(T, topk, E, bm)


def test_capacity_rejects_bad_block(binding):
    assert binding.moe_align_capacity(4, 2, 8, 24) == 0


def test_workspace_covers_tables_and_intermediates(binding):
    T, K, N, E, topk = 128, 7168, 2048, 256, 8
    need = binding.moe_w4a16_layer_workspace_bytes(T, K, N, E, topk, 0)
    S = T * topk
    assert need >= S * N * 2 + S * K * 4 + O.align_capacity(T, topk, E, 128) * 4
    assert need < 2 * (S * N * 2 + S * K * 4) + (1 << 22)
    assert binding.moe_w4a16_layer_workspace_bytes(-1, K, N, E, topk, 0) == 0
    # an empty batch still has a (table-only) workspace size
    assert 0 < binding.moe_w4a16_layer_workspace_bytes(0, K, N, E, topk, 0) < (1 << 20)
    # few experts, few rows, long reduction: room for several partial planes of the down projection
    T, K, N, E, topk = 64, 4096, 14336, 8, 2
    S = T * topk
    need = binding.moe_w4a16_layer_workspace_bytes(T, K, N, E, topk, 0)
    assert S * N * 2 + 2 * S * K * 4 <= need <= S * N * 2 + 8 * S * K * 4 + (1 << 20)


def test_layer_block_choice_tracks_rows_per_expert(binding):
    assert binding.moe_layer_block_m(128, 256, 8) == 16      # about 4 rows per expert
    assert binding.moe_layer_block_m(64, 8, 2) == 32         # 16 rows per expert
    assert binding.moe_layer_block_m(4096, 256, 8) == 64     # 128 rows per expert
    # with the layer's shapes known: the eight-wave tile (group 128, K and N multiples of 1024)
    # takes 128-slot blocks from 29 rows per expert on; other shapes keep 64-slot blocks
    f = binding.moe_layer_block_m_for
    assert f(128, 7168, 2048, 256, 8, 128) == 16
    assert f(896, 7168, 2048, 256, 8, 128) == 32             # 28 rows per expert
    assert f(1024, 7168, 2048, 256, 8, 128) == 128           # 32 rows per expert
    assert f(4096, 7168, 2048, 256, 8, 128) == 128
    assert f(1024, 2048, 1408, 64, 6, 64) == 64              # group 64: no eight-wave tile


def test_validation_before_launch_returns_status(binding):
    lib = binding.load_library()
    assert lib.moe_silu_mul(None, None, -1, 8, 0, None) == 1
    assert b"S >= 0" in lib.moe_last_error()
    assert lib.moe_combine(None, None, None, 4, 0, 8, 0, None) == 1
    assert lib.moe_align_by_expert(None, 4, 2, 2000, 16, None, None, None, None, None, None) == 2
    assert lib.moe_align_by_expert(None, 4, 2, 8, 17, None, None, None, None, None, None) == 1
    # grouped GEMM: shape checks come before any pointer is touched
    args = [None, 1, None, None, None, None, None, None]
    assert lib.moe_w4a16_grouped_gemm(*args, 8, 4, 64, 256, 48, 16, 0, None, None) == 2      # group % 32
    assert lib.moe_w4a16_grouped_gemm(*args, 8, 4, 64, 200, 64, 16, 0, None, None) == 2      # K_in % group
    assert lib.moe_w4a16_grouped_gemm(*args, 8, 4, 60, 256, 64, 16, 0, None, None) == 2      # N_out % 16
    assert lib.moe_w4a16_grouped_gemm(*args, 8, 4, 64, 256, 64, 16, 5, None, None) == 1      # dtype
    assert lib.moe_w4a16_grouped_gemm(*args, 8, 4, 64, 256, 64, 16, 0, None, None) == 1      # null pointers
    assert lib.moe_w4a16_grouped_gemm(*args, 0, 4, 64, 256, 64, 16, 0, None, None) == 0      # no slots: no-op
    assert lib.moe_w4a16_layer(*([None] * 10), 0, 256, 128, 4, 2, 128, 0, None, 0, None) == 0  # T == 0
    assert lib.moe_w4a16_layer(*([None] * 10), 4, 256, 128, 4, 2, 128, 0, None, 0, None) == 1  # null pointers
    assert lib.moe_set_stage_events(None, 0) == 0
    assert lib.moe_set_tile_override(0, 0) == 0


def test_fp8_gemm_host_logic(binding):
    """Workspace sizing and every check that happens before a launch (no kernel runs: the dummy
    pointers are never dereferenced)."""
    lib = binding.load_library()
    wsb = binding.fp8_blockwise_gemm_workspace_bytes
    assert wsb(4096, 51200, 5120) == 0                        # enough workgroups: no split reduction
    assert wsb(32, 51200, 5120) == 0
    need = wsb(16, 5120, 25600)                               # few workgroups, long reduction: float32 planes
    plane = 16 * 5120 * 4
    assert need % plane == 0 and 2 <= need // plane <= 16
    assert wsb(16, 5120, 200) == 0 and wsb(16, 100, 256) == 0 and wsb(0, 128, 256) == 0
    p = 0x10000                                               # aligned, never touched
    call = lib.fp8_blockwise_gemm
    assert call(p, p, p, p, 2 * p, 4, 128, 200, 1, None, 0, None) == 2          # K % 128
    assert call(p, p, p, p, 2 * p, 4, 100, 256, 1, None, 0, None) == 2          # N % 64
    assert call(p, p, p, p, 2 * p, 4, 128, 256, 3, None, 0, None) == 1          # output type
    assert call(None, p, p, p, 2 * p, 4, 128, 256, 1, None, 0, None) == 1       # null pointer
    assert call(p + 4, p, p, p, 2 * p, 4, 128, 256, 1, None, 0, None) == 1      # alignment
    assert call(p, p, p, p, p, 4, 128, 256, 1, None, 0, None) == 1              # C aliases A
    assert call(None, None, None, None, None, 0, 128, 256, 1, None, 0, None) == 0   # M == 0: no-op
    assert call(p, p, p, p, 2 * p, 70000, 64, 65536, 1, None, 0, None) == 2     # M * K >= 2^32
    assert b"2^32" in lib.moe_last_error()
    assert call(p, p, p, p, 2 * p, 16, 5120, 25600, 1, None, 0, None) == 3      # split reduction without workspace
    assert lib.fp8_set_plan_override(3, 0, 0, 0) == 0
    try:
        assert call(p, p, p, p, 2 * p, 4, 128, 256, 1, None, 0, None) == 2      # no 48-row tile
        assert wsb(4, 128, 256) == 0
    finally:
        assert lib.fp8_set_plan_override(0, 0, 0, 0) == 0
    assert lib.fp8_set_plan_override(-1, 0, 0, 0) == 1
    assert lib.fp8_probe_mfma(None, 4, None) == 1


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2504_16214_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".def")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower().replace("no cpu fallback", ""), f
    assert "oracle" not in open(os.path.join(ROOT, "moe_workloads", "__init__.py")).read().replace(
        "CPU oracle and the HIP path alike", "")
    assert "oracle" not in open(os.path.join(ROOT, "moe_workloads", "fp8.py")).read().replace(
        "The oracle and the HIP path read", "")


# ------------------------------------------------------------------ binding-side argument checks
def _layer_args(torch, T=4, K=256, N=128, E=3, topk=2, g=128, dt=None):
    dt = dt or torch.float16
    return dict(
        X=torch.zeros(T, K, dtype=dt), topk_ids=torch.zeros(T, topk, dtype=torch.int32),
        topk_weights=torch.zeros(T, topk, dtype=torch.float32),
        qw1=torch.zeros(E, 2 * N, K // 8, dtype=torch.int32), s1=torch.zeros(E, 2 * N, K // g, dtype=dt),
        z1=torch.zeros(E, 2 * N, K // g, dtype=torch.uint8),
        qw2=torch.zeros(E, K, N // 8, dtype=torch.int32), s2=torch.zeros(E, K, N // g, dtype=dt),
        z2=torch.zeros(E, K, N // g, dtype=torch.uint8), out=torch.zeros(T, K, dtype=dt))


@pytest.mark.parametrize("field,make_bad,needle", [
    ("topk_ids", lambda t, torch: t.to(torch.int64), "topk_ids: dtype"),              # what torch.topk returns
    ("topk_weights", lambda t, torch: t.to(torch.float64), "topk_weights: dtype"),
    ("z1", lambda t, torch: t.to(torch.int32), "W1 zeros: dtype"),
    ("s1", lambda t, torch: t[:, :, :1].contiguous(), "W1 scales: shape"),             # wrong group_size for the scale shape
    ("s2", lambda t, torch: t.to(torch.float32), "W2 scales: dtype"),
    ("out", lambda t, torch: t[:2].contiguous(), "out: shape"),                         # undersized result
    ("qw2", lambda t, torch: t[:, :, :4].contiguous(), "W2"),
])
def test_binding_rejects_wrong_dtypes_and_shapes_before_any_launch(binding, field, make_bad, needle):
    import torch
    a = _layer_args(torch)
    a[field] = make_bad(a[field], torch)
    ws = torch.zeros(1 << 20, dtype=torch.uint8)
    with pytest.raises(ValueError) as e:          # raised on CPU tensors: no pointer is ever taken
        binding.moe_w4a16_layer(a["X"], a["topk_ids"], a["topk_weights"], a["qw1"], a["s1"], a["z1"], a["qw2"],
                                a["s2"], a["z2"], a["out"], 128, ws)
    assert needle in str(e.value), str(e.value)


def test_binding_rejects_short_tables_and_mismatched_outputs(binding):
    import torch
    T, topk, E, bm = 8, 2, 4, 16
    ids = torch.zeros(T, topk, dtype=torch.int32)
    cap = binding.moe_align_capacity(T, topk, E, bm)
    ok = dict(expert_counts=torch.zeros(E, dtype=torch.int32), expert_offsets=torch.zeros(E + 1, dtype=torch.int32),
              sorted_slot_ids=torch.zeros(cap, dtype=torch.int32), block_expert_ids=torch.zeros(cap // bm, dtype=torch.int32),
              num_padded=torch.zeros(1, dtype=torch.int32))
    with pytest.raises(ValueError) as e:
        binding.moe_align_by_expert(ids, E, bm, ok["expert_counts"], ok["expert_offsets"],
                                    torch.zeros(cap - 1, dtype=torch.int32), ok["block_expert_ids"], ok["num_padded"])
    assert "sorted_slot_ids" in str(e.value)
    A = torch.zeros(T, 256, dtype=torch.float16)
    qw = torch.zeros(E, 64, 32, dtype=torch.int32)
    s = torch.zeros(E, 64, 2, dtype=torch.float16)
    z = torch.zeros(E, 64, 2, dtype=torch.uint8)
    with pytest.raises(ValueError) as e:          # C with the wrong number of columns
        binding.moe_w4a16_grouped_gemm(A, topk, qw, s, z, ok["sorted_slot_ids"], ok["block_expert_ids"],
                                       ok["num_padded"], T * topk, 128, bm, torch.zeros(T * topk, 32, dtype=torch.float16))
    assert "C:" in str(e.value)
    with pytest.raises(ValueError) as e:          # bf16 scales with fp16 activations
        binding.moe_w4a16_grouped_gemm(A, topk, qw, s.to(torch.bfloat16), z, ok["sorted_slot_ids"],
                                       ok["block_expert_ids"], ok["num_padded"], T * topk, 128, bm,
                                       torch.zeros(T * topk, 64, dtype=torch.float16))
    assert "scales: dtype" in str(e.value)
    with pytest.raises(ValueError):
        binding.moe_silu_mul(torch.zeros(4, 64, dtype=torch.float16), torch.zeros(4, 16, dtype=torch.float16))
    with pytest.raises(ValueError):
        binding.moe_combine(torch.zeros(8, 64, dtype=torch.float16), torch.zeros(4, 2, dtype=torch.float64),
                            torch.zeros(4, 64, dtype=torch.float16))
