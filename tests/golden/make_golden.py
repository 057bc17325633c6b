"""Writes tests/golden/small_layer_<dtype>.json from the CPU oracle alone.

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


if __name__ == "__main__":
    main()
