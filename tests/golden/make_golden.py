"""Writes tests/golden/small_layer_<dtype>.json and tests/golden/small_fp8_gemm.json from the CPU
oracles alone.

The paper (Section VII-B, "Mixed-type MoE") prints no worked numeric example
for this operator, so these fixtures are not paper values: they freeze what the
pinned oracle computes for a small seeded workload, as a regression guard for
the oracle and as a second parity target for the HIP path.  Run from the repo
root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from moe_workloads import MoEConfig, make_inputs  # noqa: E402
from oracle import moe_oracle as O  # noqa: E402
from oracle import fp8_oracle as F  # noqa: E402
from moe_workloads.fp8 import Fp8GemmConfig, make_fp8_inputs  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def main():
    for dt in ("f16", "bf16"):
        cfg = MoEConfig("golden_small", T=5, K=64, N=32, E=4, topk=2, group=32, dtype=dt, seed=1234)
        inp = make_inputs(cfg)
        X, s1, s2 = (O.decode_bits(b, dt) for b in (inp.x_bits, inp.s1_bits, inp.s2_bits))
        out, mid = O.layer(X, inp.topk_ids, inp.topk_weights, inp.qw1, s1, inp.z1, inp.qw2, s2, inp.z2,
                           cfg.group, dt, return_intermediates=True)
        al = O.align_by_expert(inp.topk_ids, cfg.E, 16)
        doc = {
            "source": "oracle/moe_oracle.py via tests/golden/make_golden.py (not a paper value)",
            "config": dict(T=cfg.T, K=cfg.K, N=cfg.N, E=cfg.E, topk=cfg.topk, group=cfg.group,
                           dtype=dt, seed=cfg.seed, block_m=16),
            "topk_ids": inp.topk_ids.tolist(),
            "out_bits": O.encode_bits(out, dt).tolist(),
            "H_bits_row0": O.encode_bits(mid["H"][0], dt).tolist(),
            "align": {k: v.tolist() for k, v in al.items()},
        }
        with open(os.path.join(HERE, f"small_layer_{dt}.json"), "w") as f:
            json.dump(doc, f, separators=(",", ":"))
            f.write("\n")
    # blockwise-scaled FP8 GEMM (the paper names the operator, Table II, and prints no example)
    cfg = Fp8GemmConfig("golden_fp8", M=5, N=128, K=256, seed=4321)
    inp = make_fp8_inputs(cfg)
    out = F.blockwise_gemm(inp.a_codes, inp.a_scale, inp.b_codes, inp.b_scale, "bf16")
    doc = {
        "source": "oracle/fp8_oracle.py via tests/golden/make_golden.py (not a paper value)",
        "config": dict(M=cfg.M, N=cfg.N, K=cfg.K, seed=cfg.seed, out="bf16"),
        "a_codes_row0": inp.a_codes[0].tolist(),
        "a_scale": [[float(v).hex() for v in r] for r in inp.a_scale],
        "b_scale": [[float(v).hex() for v in r] for r in inp.b_scale],
        "out_bits": O.encode_bits(out, "bf16").tolist(),
    }
    with open(os.path.join(HERE, "small_fp8_gemm.json"), "w") as f:
        json.dump(doc, f, separators=(",", ":"))
        f.write("\n")


if __name__ == "__main__":
    main()
