"""Writes tests/golden/tiny_seed0.json from the CPU oracle alone.

The paper prints no numeric values for the MoE operator (Sec. 4.5 describes it in
prose only), so there is no paper-printed fixture; this file freezes what the
oracle computes on the tiny seeded workload so that an accidental change to the
oracle or to the input generator is noticed.  It calls only `oracle/` and the
input generator.

    python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import moe_oracle as orc                      # noqa: E402
from paper_2602_19128_amd import synthetic as syn         # noqa: E402


def main():
    inp = syn.make_inputs(syn.WORKLOADS["tiny"], seed=0)
    p = orc.problem_from_inputs(inp)
    out, ids, w, margin = orc.forward(p)
    offsets, sorted_pair, inv = orc.permute(ids, p.E)
    doc = {
        "workload": "tiny", "seed": 0,
        "source": "oracle/moe_oracle.c on paper_2602_19128_amd.synthetic inputs (CPU generator)",
        "ids": ids.tolist(),
        "w": [[float(f"{v:.12e}") for v in row] for row in w],
        "min_margin": float(margin.min()),
        "offsets": offsets.tolist(),
        "sorted_pair": sorted_pair.tolist(),
        "out_row0_first8": [float(f"{v:.12e}") for v in out[0, :8]],
        "out_abs_sum": float(f"{np.abs(out).sum():.12e}"),
        "out_max_abs": float(f"{np.abs(out).max():.12e}"),
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_seed0.json")
    with open(path, "w") as f:
        json.dump(doc, f)
        f.write("\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
