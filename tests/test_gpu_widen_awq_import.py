"""GPU parity of the AWQ checkpoint import: a pure rearrangement of nibbles, bytes and 16-bit
patterns, so every output is compared bit for bit with the oracle's import of the same seeded
random words (any 32-bit word is a valid AWQ word).  One case continues into the dense GEMM: the
product on imported tensors against the oracle's product on the oracle-imported tensors."""
from __future__ import annotations

import sys

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2504_16214_amd as M
    import gpu_util as U


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def awq_words(E, K, N, g, seed):
    rng = np.random.default_rng(seed)
    aq = rng.integers(0, 2 ** 32, size=(E, K, N // 8), dtype=np.uint32).view(np.int32)
    az = rng.integers(0, 2 ** 32, size=(E, K // g, N // 8), dtype=np.uint32).view(np.int32)
    asb = rng.integers(0, 2 ** 16, size=(E, K // g, N), dtype=np.uint16)       # raw 16-bit patterns
    return aq, az, asb


def run_import(aq, az, asb):
    E, K, nw = aq.shape
    G, N = az.shape[1], nw * 8
    q = torch.full((E, N, K // 8), -1, dtype=torch.int32, device="cuda")
    s = torch.full((E, N, G), -1, dtype=torch.int16, device="cuda")
    z = torch.full((E, N, G), 255, dtype=torch.uint8, device="cuda")
    M.moe_import_awq(torch.from_numpy(aq).cuda(), torch.from_numpy(az).cuda(),
                     torch.from_numpy(asb.view(np.int16)).cuda(), q, s, z)
    torch.cuda.synchronize()
    return q.cpu().numpy(), s.cpu().numpy().view(np.uint16), z.cpu().numpy()


@pytest.mark.parametrize("E,K,N,g", [
    (1, 8, 8, 8),            # one word
    (3, 40, 24, 8),          # K/8 = 5 words per row (scalar stores), ragged column block
    (2, 96, 200, 32),        # columns past the first 64, 12 words per row
    (2, 1024, 512, 128),     # several workgroups along both axes
    (5, 136, 72, 136),       # one group, 17 words per row: scalar stores, last lane group partly filled
    (2, 160, 72, 32),        # 20 words per row: vector stores, second block along the reduction partly empty
])
def test_import_matches_oracle_bitwise(E, K, N, g):
    say(f"awq import E={E} K={K} N={N} g={g}")
    aq, az, asb = awq_words(E, K, N, g, seed=1000 + K + N)
    q, s, z = run_import(aq, az, asb)
    wq, ws, wz = O.import_awq(aq, az, asb)
    assert np.array_equal(q, wq)
    assert np.array_equal(s, ws)
    assert np.array_equal(z, wz)


def test_import_unaligned_output_base():
    """An output tensor that starts 4 bytes past a 16-byte boundary takes the scalar-store path."""
    E, K, N, g = 2, 128, 64, 64
    say(f"awq import, output base offset by one word E={E} K={K} N={N}")
    aq, az, asb = awq_words(E, K, N, g, seed=77)
    buf = torch.full((E * N * (K // 8) + 1,), -1, dtype=torch.int32, device="cuda")
    q = buf[1:].view(E, N, K // 8)
    s = torch.empty((E, N, K // g), dtype=torch.int16, device="cuda")
    z = torch.empty((E, N, K // g), dtype=torch.uint8, device="cuda")
    M.moe_import_awq(torch.from_numpy(aq).cuda(), torch.from_numpy(az).cuda(),
                     torch.from_numpy(asb.view(np.int16)).cuda(), q, s, z)
    torch.cuda.synchronize()
    assert int(buf[0]) == -1
    assert np.array_equal(q.cpu().numpy(), O.import_awq(aq, az, asb)[0])


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_imported_weights_feed_the_dense_gemm(dtype):
    E, K, N, g, rows = 1, 1024, 256, 128, 19
    say(f"awq import -> dense gemm K={K} N={N} {dtype}")
    rng = np.random.default_rng(5)
    aq, az, _ = awq_words(E, K, N, g, seed=6)
    scales = O.rnd(rng.uniform(0.005, 0.02, size=(E, K // g, N)), dtype)
    asb = O.encode_bits(scales, dtype)
    x = O.rnd(rng.standard_normal((rows, K)), dtype)
    tdt = U.TORCH_DT[dtype]
    q = torch.empty((E, N, K // 8), dtype=torch.int32, device="cuda")
    s = torch.empty((E, N, K // g), dtype=tdt, device="cuda")
    z = torch.empty((E, N, K // g), dtype=torch.uint8, device="cuda")
    M.moe_import_awq(torch.from_numpy(aq).cuda(), torch.from_numpy(az).cuda(), U.bits_to_dev(asb, dtype), q, s, z)
    C = torch.full((rows, N), float("nan"), dtype=tdt, device="cuda")
    M.moe_w4a16_dense_gemm(U.bits_to_dev(O.encode_bits(x, dtype), dtype), q[0], s[0], z[0], g, C)
    torch.cuda.synchronize()
    wq, ws, wz = O.import_awq(aq, az, scales)
    want = O.dense_gemm(x, wq[0], ws[0], wz[0], g, dtype)
    U.assert_close(U.dev_to_f64(C), want, "dense gemm on imported weights")


def test_import_error_paths():
    say("awq import error paths")
    aq, az, asb = awq_words(1, 16, 16, 8, seed=3)
    dq, dz, ds = torch.from_numpy(aq).cuda(), torch.from_numpy(az).cuda(), torch.from_numpy(asb.view(np.int16)).cuda()
    q = torch.empty((1, 16, 2), dtype=torch.int32, device="cuda")
    s = torch.empty((1, 16, 2), dtype=torch.int16, device="cuda")
    z = torch.empty((1, 16, 2), dtype=torch.uint8, device="cuda")
    lib = M.load_library()
    ptr = lambda t: t.data_ptr()
    # K_in not a multiple of the group size
    assert lib.moe_import_awq(ptr(dq), ptr(dz), ptr(ds), 1, 16, 16, 5, ptr(q), ptr(s), ptr(z), None) == 2
    # N_out not a multiple of 8
    assert lib.moe_import_awq(ptr(dq), ptr(dz), ptr(ds), 1, 16, 12, 8, ptr(q), ptr(s), ptr(z), None) == 2
    # in place
    assert lib.moe_import_awq(ptr(dq), ptr(dz), ptr(ds), 1, 16, 16, 8, ptr(dq), ptr(s), ptr(z), None) == 1
    # null
    assert lib.moe_import_awq(None, ptr(dz), ptr(ds), 1, 16, 16, 8, ptr(q), ptr(s), ptr(z), None) == 1
    assert "null" in M.moe_last_error()
