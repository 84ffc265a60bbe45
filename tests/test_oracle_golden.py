"""The oracle still produces the frozen tiny-workload values (see tests/golden/make_golden.py)."""
import json
import os

import numpy as np

from oracle import moe_oracle as orc
from paper_2602_19128_amd import synthetic as syn

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiny_seed0.json")


def test_tiny_seed0_matches_frozen_values():
    with open(GOLDEN) as f:
        doc = json.load(f)
    inp = syn.make_inputs(syn.WORKLOADS["tiny"], seed=0)
    p = orc.problem_from_inputs(inp)
    out, ids, w, margin = orc.forward(p)
    offsets, sorted_pair, _ = orc.permute(ids, p.E)
    assert ids.tolist() == doc["ids"]
    np.testing.assert_allclose(w, np.array(doc["w"]), rtol=1e-10)
    assert offsets.tolist() == doc["offsets"]
    assert sorted_pair.tolist() == doc["sorted_pair"]
    np.testing.assert_allclose(out[0, :8], np.array(doc["out_row0_first8"]), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(np.abs(out).sum(), doc["out_abs_sum"], rtol=1e-10)
    np.testing.assert_allclose(np.abs(out).max(), doc["out_max_abs"], rtol=1e-10)
    assert margin.min() >= 1e-6          # no tie-excused token in this fixture


def test_quantizer_matches_frozen_values():
    with open(os.path.join(os.path.dirname(GOLDEN), "quantize_seed0.json")) as f:
        doc = json.load(f)
    inp = syn.make_inputs(syn.WORKLOADS["tiny"], seed=0)
    q, scale = orc.quantize_rows_1x128(inp.x)
    assert scale.view(np.uint32).reshape(-1).tolist() == doc["scale_bits"]
    assert q[0, :128].tolist() == doc["codes_row0_block0"]
    assert int(q.astype(np.int64).sum()) == doc["code_sum"]
    weights = np.arange(q.size).reshape(q.shape) % 251 + 1
    assert int((q.astype(np.int64) * weights).sum()) == doc["code_weighted_sum"]
