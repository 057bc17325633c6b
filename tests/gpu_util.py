"""Helpers for the GPU parity tests: move seeded workloads to the device, run the HIP
entry points through the binding, bring results back as float64."""
from __future__ import annotations

import numpy as np
import torch

import paper_2504_16214_amd as M
from oracle import moe_oracle as O

TORCH_DT = {"f16": torch.float16, "bf16": torch.bfloat16}

# Acceptance bound of the benchmark statement: |gpu - oracle| <= 2e-2 + 1e-2 * |oracle|
ATOL, RTOL = 2e-2, 1e-2


def bits_to_dev(bits: np.ndarray, dt: str) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(TORCH_DT[dt])


def vals_to_dev(vals: np.ndarray, dt: str) -> torch.Tensor:
    """float64 values already representable in dt -> device tensor."""
    return bits_to_dev(O.encode_bits(vals, dt), dt)


def dev_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def i32(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


class DevInputs:
    def __init__(self, inp):
        c = inp.cfg
        self.cfg = c
        self.X = bits_to_dev(inp.x_bits, c.dtype)
        self.ids = i32(inp.topk_ids)
        self.w = torch.from_numpy(inp.topk_weights).cuda()
        self.qw1 = torch.from_numpy(inp.qw1).cuda()
        self.s1 = bits_to_dev(inp.s1_bits, c.dtype)
        self.z1 = torch.from_numpy(inp.z1).cuda()
        self.qw2 = torch.from_numpy(inp.qw2).cuda()
        self.s2 = bits_to_dev(inp.s2_bits, c.dtype)
        self.z2 = torch.from_numpy(inp.z2).cuda()


def run_align(ids_dev: torch.Tensor, E: int, block_m: int):
    T, topk = ids_dev.shape
    cap = M.moe_align_capacity(T, topk, E, block_m)
    out = {
        "expert_counts": torch.full((E,), -7, dtype=torch.int32, device="cuda"),
        "expert_offsets": torch.full((E + 1,), -7, dtype=torch.int32, device="cuda"),
        "sorted_slot_ids": torch.full((max(cap, 1),), -7, dtype=torch.int32, device="cuda"),
        "block_expert_ids": torch.full((max(cap // block_m, 1),), -7, dtype=torch.int32, device="cuda"),
        "num_padded": torch.full((1,), -7, dtype=torch.int32, device="cuda"),
    }
    M.moe_align_by_expert(ids_dev, E, block_m, out["expert_counts"], out["expert_offsets"],
                          out["sorted_slot_ids"], out["block_expert_ids"], out["num_padded"])
    torch.cuda.synchronize()
    out["capacity"] = cap
    return out


def assert_align_equal(got: dict, want: dict, block_m: int):
    cap = got["capacity"]
    np.testing.assert_array_equal(got["expert_counts"].cpu().numpy(), want["expert_counts"])
    np.testing.assert_array_equal(got["expert_offsets"].cpu().numpy(), want["expert_offsets"])
    np.testing.assert_array_equal(got["num_padded"].cpu().numpy(), want["num_padded"])
    assert cap == want["sorted_slot_ids"].size
    np.testing.assert_array_equal(got["sorted_slot_ids"].cpu().numpy()[:cap], want["sorted_slot_ids"])
    np.testing.assert_array_equal(got["block_expert_ids"].cpu().numpy()[:cap // block_m],
                                  want["block_expert_ids"])


def assert_close(got: np.ndarray, want: np.ndarray, what: str = ""):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = np.abs(got - want)
    bound = ATOL + RTOL * np.abs(want)
    bad = err > bound
    if bad.any():
        idx = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} outside |d| <= {ATOL} + {RTOL}|ref|; worst at "
                             f"{idx}: got {got[idx]!r} want {want[idx]!r}")
    return float((err / bound).max()) if err.size else 0.0


def run_layer(d: DevInputs, out=None):
    c = d.cfg
    dtc = M.MOE_F16 if c.dtype == "f16" else M.MOE_BF16
    nbytes = M.moe_w4a16_layer_workspace_bytes(c.T, c.K, c.N, c.E, c.topk, dtc)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    if out is None:
        out = torch.full((c.T, c.K), float("nan"), dtype=TORCH_DT[c.dtype], device="cuda")
    M.moe_w4a16_layer(d.X, d.ids, d.w, d.qw1, d.s1, d.z1, d.qw2, d.s2, d.z2, out, c.group, ws)
    torch.cuda.synchronize()
    return out
