"""moe_forward_static (the entry point for callers that cannot allocate: intermediates in the
library's own static device buffer) against moe_forward on a caller workspace, through the C ABI:
two calls in a row, the second on a smaller problem, every output bit compared; the layer output
is also held to the oracle's tolerance."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from paper_2602_19128_amd import binding as moe
from paper_2602_19128_amd import synthetic as syn
from parity_util import TOL_MAX, TOL_MEAN, err_stats, f64

pytestmark = pytest.mark.gpu

GROUPED = dict(scoring="sigmoid", has_bias=True, routed_scale=2.5, group_score_topn=2)


def _both(wl, seed):
    print(f"\n[static scratch] {wl}", flush=True)
    cpu = syn.make_inputs(wl, seed=seed)
    gpu = cpu.to("cuda")
    cfg = moe.MoEConfig.from_workload(wl)
    assert moe.moe_workspace_size(cfg) <= moe.STATIC_SCRATCH_BYTES
    args = (cfg, gpu.x, gpu.x_scale, gpu.router_w, gpu.bias, gpu.w1, gpu.w1_scale, gpu.w2, gpu.w2_scale)
    ref = moe.moe_forward(*args)
    out = torch.full((wl.T, wl.H), float("nan"), dtype=torch.bfloat16, device="cuda")
    moe.moe_forward_static(*args, out)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), "static-scratch call differs from moe_forward"
    exact, *_ = orc.forward(orc.problem_from_inputs(cpu))
    max_rel, mean_rel = err_stats(f64(out), exact)
    print(f"  vs oracle: max_rel={max_rel:.2e} mean_rel={mean_rel:.2e}", flush=True)
    assert max_rel <= TOL_MAX[wl.fp8] and mean_rel <= TOL_MEAN[wl.fp8]


def test_static_scratch_forward_matches_workspace_forward_twice():
    moe.moe_init()
    # a DeepSeek-shaped grouped layer with several row tiles, then a smaller fp8 layer that reuses
    # (and only partly overwrites) the same buffer
    _both(syn.Workload("static_a", T=300, H=512, I=256, E=64, top_k=6, n_group=8, topk_group=4, **GROUPED), seed=0)
    _both(syn.Workload("static_b", T=37, H=256, I=128, E=16, top_k=2, fp8=True), seed=1)
    # and the first shape again: nothing left behind by the smaller call may matter
    _both(syn.Workload("static_a", T=300, H=512, I=256, E=64, top_k=6, n_group=8, topk_group=4, **GROUPED), seed=2)
