"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times
(one moe_forward call on a preallocated workspace).

The oracle cannot run these sizes in full, so: routing and the sort-scatter are
compared for every token (they need no expert weights); both grouped GEMMs are
compared on rows taken from EVERY tile of the schedule the launch really ran
(first row, last row and two seeded rows of each tile, every column of those rows,
so that each tile height, each ragged last row block, each tile of a split expert
and every column slab is looked at); and the layer output is compared on a seeded
sample of tokens the oracle computes one by one.  Tensors are drawn on the GPU
and copied to the host for the oracle.
"""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from paper_2602_19128_amd import binding as moe
from paper_2602_19128_amd import synthetic as syn
from parity_util import (TOL_MAX, TOL_MEAN, check_tiles, choice_keys, compare_routing, err_stats, f64,
                         local_permute)

pytestmark = pytest.mark.gpu

SAMPLE_TOKENS = 96
ROWS_PER_TILE = 4           # first, last and two seeded rows of every tile


def _check_workload(gpu, host_w, sample_tokens=SAMPLE_TOKENS):
    wl = gpu.wl
    print(f"\n[full-size] {wl}", flush=True)
    cfg = moe.MoEConfig.from_workload(wl)
    out = torch.empty((wl.T, wl.H), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty((moe.moe_workspace_size(cfg),), dtype=torch.uint8, device="cuda")
    moe.moe_forward(cfg, gpu.x, gpu.x_scale, gpu.router_w, gpu.bias, gpu.w1, gpu.w1_scale, gpu.w2, gpu.w2_scale,
                    out=out, workspace=ws)
    torch.cuda.synchronize()
    first = out.clone()
    moe.moe_forward(cfg, gpu.x, gpu.x_scale, gpu.router_w, gpu.bias, gpu.w1, gpu.w1_scale, gpu.w2, gpu.w2_scale,
                    out=out, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(first.view(torch.int16), out.view(torch.int16)), "not run-to-run identical"
    assert torch.isfinite(out.float()).all()

    # routing + sort-scatter for every token
    host = syn.MoEInputs(wl, gpu.x.cpu(), host_w.router_w, None if gpu.bias is None else gpu.bias.cpu(),
                         host_w.w1, host_w.w2, None if gpu.x_scale is None else gpu.x_scale.cpu(),
                         host_w.w1_scale, host_w.w2_scale)
    p = orc.problem_from_inputs(host)
    z = orc.router_logits(p)
    ids_r, w_r, margin = orc.route(p, z)
    ids_g, w_g = moe.moe_route(cfg, gpu.x, gpu.x_scale, gpu.router_w, gpu.bias)
    other, swapped, same_set = compare_routing(ids_g, w_g, ids_r, w_r, margin, wl.routed_scale, wl.E,
                                               choice_keys(p, z))
    off_g, sp_g, inv_g, tiles, sched = moe.moe_permute(cfg, ids_g)
    torch.cuda.synchronize()
    off_r, sp_r, inv_r, kept = local_permute(ids_g.cpu().numpy(), wl.E, wl.local_offset, wl.local_experts)   # oracle on the GPU's own routing
    assert np.array_equal(off_g.cpu().numpy(), off_r)
    assert np.array_equal(sp_g.cpu().numpy()[:kept], sp_r) and np.array_equal(inv_g.cpu().numpy(), inv_r)
    check_tiles(tiles, sched, off_r, moe.moe_tile_rows(cfg))
    load = np.diff(off_r)
    print(f"  routing: tie-excused tokens={other} swapped slots={swapped} of {wl.T}; "
          f"active experts={(load > 0).sum()} max/mean load={load.max() / load.mean():.2f}", flush=True)

    # both GEMMs on rows of every tile of this schedule, every column of those rows
    n_tiles = int(sched.cpu()[0])
    rec = tiles.cpu().numpy()[:n_tiles]
    rng_t = np.random.default_rng(1)
    rows = []
    for _, row0, nrows, _first, _count, *_pad in rec:
        inner = rng_t.integers(0, nrows, size=ROWS_PER_TILE - 2)
        rows += [row0, row0 + nrows - 1] + [row0 + int(r) for r in inner]
    rows = np.unique(np.asarray(rows, dtype=np.int64))
    pair = sp_r[rows]                                        # sorted row -> pair id
    tok = (pair // wl.top_k).astype(np.int32)
    exp = (ids_g.cpu().numpy().reshape(-1)[pair] - wl.local_offset).astype(np.int32)
    x_g, xs_g = (gpu.x, gpu.x_scale)
    if wl.quantize_x:
        x_g, xs_g = moe.moe_quantize_act(cfg, gpu.x)
    act_g, asc_g = moe.moe_grouped_gemm_swiglu(cfg, x_g, xs_g, gpu.w1, gpu.w1_scale, sp_g, tiles, sched)
    y_g = moe.moe_grouped_gemm_down(cfg, act_g, asc_g, gpu.w2, gpu.w2_scale, tiles, sched)
    torch.cuda.synchronize()
    pick = torch.from_numpy(rows).cuda()
    act_rows = f64(act_g[pick])
    if asc_g is not None:
        act_rows = act_rows * np.repeat(f64(asc_g[pick]), 128, axis=1)
    act_ref = orc.swiglu_rows(p, tok, exp)
    a_max, a_mean = err_stats(act_rows, act_ref)
    y_ref = orc.down_rows(p, exp, act_rows)                  # from the activations the GPU consumed
    y_max, y_mean = err_stats(f64(y_g[pick]), y_ref)
    heights = sorted(set(int(-(-r // 16)) for r in rec[:, 2]))
    print(f"  staged GEMMs: {len(rows)} rows of {n_tiles} tiles ({len(set(rec[:, 0]))} experts, "
          f"{int((rec[:, 4] > 1).sum())} tiles of split experts, row blocks per tile {heights[0]}..{heights[-1]}): "
          f"act max_rel={a_max:.2e} mean_rel={a_mean:.2e}; y max_rel={y_max:.2e} mean_rel={y_mean:.2e}", flush=True)
    if wl.fp8:
        assert a_max <= 2 ** -4 + 1e-3 and a_mean <= 3.5e-2  # e4m3 re-quantisation of act (3 mantissa bits)
    else:
        assert a_max <= 6e-3 and a_mean <= 3e-3              # one bf16 rounding of an fp32 accumulation
    assert y_max <= 6e-3 and y_mean <= 3e-3
    del act_g, asc_g, y_g

    # layer output on sampled tokens
    rng = np.random.default_rng(0)
    cand = np.arange(wl.T)
    if wl.local_experts > 0:      # tokens with at least one expert held here (the others are exactly zero)
        local = (ids_r >= wl.local_offset) & (ids_r < wl.local_offset + wl.local_experts)
        assert not f64(out[torch.from_numpy(np.nonzero(~local.any(axis=1) & same_set)[0]).cuda()]).any()
        cand = np.nonzero(local.any(axis=1))[0]
    sample = np.sort(rng.choice(cand, size=min(sample_tokens, len(cand)), replace=False)).astype(np.int32)
    ref, ids_s, w_s, margin_s = orc.forward_tokens(p, sample)
    keep = same_set[sample]
    got = f64(out[torch.from_numpy(sample.astype(np.int64)).cuda()])
    max_rel, mean_rel = err_stats(got[keep], ref[keep])
    print(f"  output on {keep.sum()} sampled tokens: max_rel={max_rel:.2e} mean_rel={mean_rel:.2e}", flush=True)
    assert keep.sum() >= len(sample) // 2
    assert max_rel <= TOL_MAX[wl.fp8] and mean_rel <= TOL_MEAN[wl.fp8]


def test_mixtral_prefill_full_size():
    gpu = syn.make_inputs(syn.WORKLOADS["mixtral_prefill"], seed=0, device="cuda")
    _check_workload(gpu, gpu.to("cpu"))


@pytest.fixture(scope="module")
def dsv3():
    gpu = syn.make_inputs(syn.WORKLOADS["dsv3_prefill"], seed=0, device="cuda")
    print("\n[full-size] copying DeepSeek-V3-shaped weights to the host for the oracle", flush=True)
    return gpu, gpu.to("cpu")


@pytest.mark.parametrize("name", ["dsv3_decode", "dsv3_prefill", "dsv3_prefill_skew"])
def test_dsv3_full_size(dsv3, name):
    base, host_w = dsv3
    gpu = base if name == "dsv3_prefill" else syn.make_inputs(syn.WORKLOADS[name], seed=0, device="cuda",
                                                               weights_from=base)
    _check_workload(gpu, host_w)


def test_fp8_prefill_full_size():
    gpu = syn.make_inputs(syn.WORKLOADS["fp8_prefill"], seed=0, device="cuda")
    _check_workload(gpu, gpu.to("cpu"))


@pytest.fixture(scope="module")
def local32():
    gpu = syn.make_inputs(syn.WORKLOADS["fp8_local32"], seed=0, device="cuda")
    return gpu, gpu.to("cpu")


def test_fp8_local_experts_full_size(local32):
    """One device's share of the DeepSeek-V3-shaped layer: 32 local experts of 256."""
    _check_workload(*local32)


def test_fp8_local_experts_quantise_on_the_path_full_size(local32):
    """The same share fed bf16 hidden states: the layer quantises them itself (1x128 blocks), the
    router scores the bf16 values.  The quantiser is also compared bit for bit on sampled rows."""
    base, host_w = local32
    wl = syn.WORKLOADS["fp8_local32_qx"]
    gpu = syn.make_inputs(wl, seed=0, device="cuda", weights_from=base)
    assert gpu.x.dtype == torch.bfloat16 and gpu.x_scale is None
    cfg = moe.MoEConfig.from_workload(wl)
    xq, xs = moe.moe_quantize_act(cfg, gpu.x)
    torch.cuda.synchronize()
    rows = np.sort(np.random.default_rng(1).choice(wl.T, size=96, replace=False))
    q_ref, s_ref = orc.quantize_rows_1x128(gpu.x[torch.from_numpy(rows).cuda()].cpu())
    assert np.array_equal(xs.cpu().numpy()[rows].view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(xq.cpu().view(torch.uint8).numpy()[rows], q_ref)
    _check_workload(gpu, host_w)
