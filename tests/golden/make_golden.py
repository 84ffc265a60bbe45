"""Writes tests/golden/tiny_seed0.json and tests/golden/quantize_seed0.json from the CPU oracle alone.

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
        "source": "oracle/moe_oracle.c on paper_2602_19128_amd.synthetic inputs (counter-based generator, the same bits on every device)",
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

    # the 1x128 activation quantiser (paper Sec. 4.3, kernel table: fp8 packing and scaling) on the
    # tiny workload's bf16 hidden states: every scale, the codes of the first block, a checksum of all
    q, scale = orc.quantize_rows_1x128(inp.x)
    qdoc = {
        "workload": "tiny", "seed": 0,
        "source": "oracle_quantize_rows_1x128 on paper_2602_19128_amd.synthetic hidden states (counter-based generator)",
        "scale_bits": scale.view(np.uint32).reshape(-1).tolist(),
        "codes_row0_block0": q[0, :128].tolist(),
        "code_sum": int(q.astype(np.int64).sum()),
        "code_weighted_sum": int((q.astype(np.int64) * (np.arange(q.size).reshape(q.shape) % 251 + 1)).sum()),
    }
    qpath = os.path.join(os.path.dirname(os.path.abspath(__file__)), "quantize_seed0.json")
    with open(qpath, "w") as f:
        json.dump(qdoc, f)
        f.write("\n")
    print("wrote", qpath)


if __name__ == "__main__":
    main()
