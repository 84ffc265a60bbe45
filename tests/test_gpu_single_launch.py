"""The single-launch forward (one persistent kernel for latency-bound layers, or for their routing
and sort-scatter) against the multi-launch pipeline, through the C ABI: same bits in the output and
in every intermediate the workspace holds, which path a problem takes, repeated launches (the
barrier counters must be back at zero each time), replay from a HIP graph, and the oracle's
tolerance for the path as taken."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from paper_2602_19128_amd import binding as moe
from paper_2602_19128_amd import synthetic as syn
from parity_util import TOL_MAX, TOL_MEAN, err_stats, f64

pytestmark = pytest.mark.gpu

GROUPED = dict(scoring="sigmoid", has_bias=True, routed_scale=2.5, group_score_topn=2)
ALL, NONE = moe.SINGLE_LAUNCH_ALL, moe.SINGLE_LAUNCH_NONE

CASES = {
    # name: (workload, path expected)
    "tiny": (syn.WORKLOADS["tiny"], ALL),                                                       # few experts, one wavefront per token
    "few_split": (syn.Workload("few_split", T=37, H=1024, I=64, E=8, top_k=2), ALL),            # four wavefronts per token
    "one_token": (syn.Workload("one_token", T=1, H=128, I=64, E=8, top_k=3), ALL),
    "split_experts": (syn.Workload("split_experts", T=100, H=256, I=128, E=8, top_k=2, scoring="sigmoid", has_bias=True,
                                   hot_experts=1, hot_bias=0.5), ALL),                          # a hot expert cut into several 64-row tiles
    "tiled_64": (syn.Workload("tiled_64", T=100, H=512, I=256, E=64, top_k=6, n_group=8, topk_group=4, **GROUPED), ALL),
    "tiled_128": (syn.Workload("tiled_128", T=70, H=384, I=128, E=128, top_k=8), ALL),          # two experts per lane
    "tiled_256_sparse": (syn.Workload("tiled_256_sparse", T=33, H=256, I=128, E=256, top_k=8, n_group=8,
                                      topk_group=4, **GROUPED), ALL),                           # empty experts, four per lane
    "local": (syn.Workload("local", T=90, H=256, I=128, E=32, top_k=4, local_offset=8, local_experts=16), ALL),
    "decode_like": (syn.Workload("decode_like", T=64, H=512, I=1024, E=128, top_k=8, n_group=8, topk_group=4,
                                 **GROUPED), NONE),                                             # wide GEMM workgroups
    "few_tall": (syn.Workload("few_tall", T=200, H=256, I=128, E=4, top_k=2), NONE),            # 128-row tiles
    "many_pairs": (syn.Workload("many_pairs", T=300, H=256, I=64, E=40, top_k=4), NONE),        # more than 1024 pairs
    "fp8": (syn.Workload("fp8", T=50, H=256, I=256, E=8, top_k=2, fp8=True), NONE),
}


def _forward(cfg, gpu, ws, out):
    moe.moe_forward(cfg, gpu.x, gpu.x_scale, gpu.router_w, gpu.bias, gpu.w1, gpu.w1_scale, gpu.w2, gpu.w2_scale,
                    out=out, workspace=ws)


@pytest.mark.parametrize("name", list(CASES))
def test_single_launch_gives_the_bits_of_the_pipeline(name):
    wl, expect = CASES[name]
    print(f"\n[single launch] {wl}", flush=True)
    cpu = syn.make_inputs(wl, seed=0)
    gpu = cpu.to("cuda")
    cfg = moe.MoEConfig.from_workload(wl)
    n = moe.moe_workspace_size(cfg)
    assert moe.moe_single_launch_mode(cfg) == NONE           # off unless asked for
    ws0 = torch.zeros((n,), dtype=torch.uint8, device="cuda")
    out0 = torch.empty((wl.T, wl.H), dtype=torch.bfloat16, device="cuda")
    _forward(cfg, gpu, ws0, out0)
    torch.cuda.synchronize()
    ws1 = torch.zeros((n,), dtype=torch.uint8, device="cuda")
    out1 = torch.full((wl.T, wl.H), float("nan"), dtype=torch.bfloat16, device="cuda")
    try:
        moe.moe_single_launch(True)
        assert moe.moe_single_launch_mode(cfg) == expect
        for rep in range(3):                                 # the counters are back at zero after every launch
            _forward(cfg, gpu, ws1, out1)
            torch.cuda.synchronize()
            assert torch.equal(out0.view(torch.int16), out1.view(torch.int16)), f"output differs (launch {rep})"
            # ids, weights, offsets, permutation, tile list, schedule, act, y: the workspaces hold the same bytes
            assert torch.equal(ws0, ws1), f"workspace contents differ (launch {rep})"
    finally:
        moe.moe_single_launch(False)
    assert moe.moe_single_launch_timeouts() == 0
    ref, *_ = orc.forward(orc.problem_from_inputs(cpu))
    max_rel, mean_rel = err_stats(f64(out1), ref)
    print(f"  path={expect} vs oracle: max_rel={max_rel:.2e} mean_rel={mean_rel:.2e}", flush=True)
    assert max_rel <= TOL_MAX[wl.fp8] and mean_rel <= TOL_MEAN[wl.fp8]


@pytest.mark.parametrize("name", ["tiny", "tiled_64"])
def test_single_launch_replays_from_a_graph(name):
    """The launch owns no host state and clears its barrier counters itself, so it can be captured
    and replayed; every replay, with eager launches in between, gives the eager bits."""
    wl, _ = CASES[name]
    gpu = syn.make_inputs(wl, seed=1).to("cuda")
    cfg = moe.MoEConfig.from_workload(wl)
    ws = torch.empty((moe.moe_workspace_size(cfg),), dtype=torch.uint8, device="cuda")
    out = torch.empty((wl.T, wl.H), dtype=torch.bfloat16, device="cuda")
    _forward(cfg, gpu, ws, out)                              # the pipeline's bits
    torch.cuda.synchronize()
    eager = out.clone()
    try:
        moe.moe_single_launch(True)
        assert moe.moe_single_launch_mode(cfg) == ALL
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            _forward(cfg, gpu, ws, out)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            _forward(cfg, gpu, ws, out)
        for rep in range(4):
            out.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {rep} differs"
            _forward(cfg, gpu, ws, out)                      # eager work between the replays
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), eager.view(torch.int16))
    finally:
        moe.moe_single_launch(False)
    assert moe.moe_single_launch_timeouts() == 0
