"""GPU parity: every step of the HIP path against the CPU oracle, through the C ABI.

Small cases span several row tiles with ragged tails and exercise each tile
height the library picks; the oracle runs them in full.  Staged steps are fed
oracle-verified inputs so that one step's rounding cannot hide in the next.
"""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from paper_2602_19128_amd import binding as moe
from paper_2602_19128_amd import synthetic as syn
from parity_util import (TOL_MAX, TOL_MEAN, check_tiles, compare_routing, err_stats, f64, oracle_all)

pytestmark = pytest.mark.gpu

GROUPED = dict(scoring="sigmoid", has_bias=True, routed_scale=2.5, group_score_topn=2)

CASES = {
    # name: workload                                                        (tile height picked)
    "tiny": syn.WORKLOADS["tiny"],                                                      # 32
    "ragged64": syn.Workload("ragged64", T=203, H=256, I=192, E=8, top_k=2),            # 64
    "ragged128": syn.Workload("ragged128", T=301, H=320, I=128, E=4, top_k=2),          # 128
    "sparse32": syn.Workload("sparse32", T=33, H=256, I=128, E=64, top_k=6),            # 32, empty experts
    "grouped": syn.Workload("grouped", T=70, H=256, I=128, E=16, top_k=4, n_group=4,
                            topk_group=2, **GROUPED),
    "dsv3_like": syn.Workload("dsv3_like", T=96, H=512, I=128, E=256, top_k=8, n_group=8,
                              topk_group=4, **GROUPED),
    "one_token": syn.Workload("one_token", T=1, H=128, I=64, E=8, top_k=3),
    "one_expert": syn.Workload("one_expert", T=40, H=128, I=64, E=1, top_k=1),
    "all_experts": syn.Workload("all_experts", T=24, H=128, I=64, E=4, top_k=4),
    # fp8 e4m3 payload with 1x128 / 128x128 fp32 block scales
    "fp8_small": syn.Workload("fp8_small", T=150, H=256, I=256, E=8, top_k=2, fp8=True),
    "fp8_grouped": syn.Workload("fp8_grouped", T=96, H=512, I=256, E=256, top_k=8, n_group=8,
                                topk_group=4, fp8=True, **GROUPED),
    "fp8_tall": syn.Workload("fp8_tall", T=700, H=384, I=128, E=4, top_k=2, fp8=True),   # several 256-row tiles
    # local-expert mode: only a slice of the experts has weights here, the other pairs are dropped
    "local_bf16": syn.Workload("local_bf16", T=90, H=256, I=128, E=16, top_k=4, local_offset=4, local_experts=8),
    "local_fp8": syn.Workload("local_fp8", T=120, H=256, I=256, E=32, top_k=6, n_group=4, topk_group=2, fp8=True,
                              local_offset=16, local_experts=8, **GROUPED),
    # enough tokens for the matrix-core router (ragged token tile, expert count not a multiple of 16)
    "many_tokens": syn.Workload("many_tokens", T=600, H=256, I=64, E=40, top_k=4),
    "many_tokens_fp8": syn.Workload("many_tokens_fp8", T=530, H=384, I=128, E=64, top_k=6, n_group=4, topk_group=3,
                                    fp8=True, **GROUPED),
    # fp8 layers that receive bf16 hidden states and quantise them on the path (1x128 blocks)
    "qx_small": syn.Workload("qx_small", T=150, H=256, I=256, E=8, top_k=2, fp8=True, quantize_x=True),
    "qx_grouped_local": syn.Workload("qx_grouped_local", T=530, H=384, I=128, E=64, top_k=6, n_group=4, topk_group=3,
                                     fp8=True, quantize_x=True, local_offset=16, local_experts=32, **GROUPED),
    # few experts and few tokens: the one-launch router splits H over four wavefronts per token
    "few_split": syn.Workload("few_split", T=37, H=1024, I=64, E=8, top_k=2),
    "few_split_fp8": syn.Workload("few_split_fp8", T=21, H=1152, I=128, E=12, top_k=3, fp8=True, **GROUPED),
    # low tiles (32 rows) and enough of them that the down GEMM takes four weight blocks per wavefront
    "low_tiles": syn.Workload("low_tiles", T=256, H=2048, I=128, E=256, top_k=8),
    "low_tiles_ragged": syn.Workload("low_tiles_ragged", T=256, H=1600, I=64, E=256, top_k=8),   # 3 slabs of 512 columns + 64
    "low_tiles_fp8": syn.Workload("low_tiles_fp8", T=250, H=2048, I=128, E=256, top_k=8, n_group=8, topk_group=4,
                                  fp8=True, **GROUPED),
    # matrix-core router with several K steps per workgroup (5: the rotation of its three register
    # sets ends mid-cycle), two expert tiles with a ragged second one, an expert count that is no
    # multiple of 4 (element-wise stores and loads of the partial logits), a ragged token tile
    "router_deep": syn.Workload("router_deep", T=1300, H=1920, I=64, E=330, top_k=4),
    "router_deep_fp8": syn.Workload("router_deep_fp8", T=1300, H=1920, I=128, E=132, top_k=4, fp8=True),
    # the limits of the interface: 512 experts (8 per lane in the router) and 64 experts per token
    "max_experts": syn.Workload("max_experts", T=40, H=128, I=64, E=512, top_k=64),
    # fp8 contractions longer than 64 scale blocks (a slab's weight scales fill a second register per
    # lane): 66 blocks along H, and 96 along I with a row stride that is a multiple of 4 KiB (the K
    # loops of neighbouring workgroups then start at different columns)
    "fp8_deep_h": syn.Workload("fp8_deep_h", T=24, H=8448, I=128, E=4, top_k=2, fp8=True),
    "fp8_deep_i": syn.Workload("fp8_deep_i", T=24, H=128, I=12288, E=4, top_k=2, fp8=True),
    # the wide (8-wavefront) bf16 workgroups of the benchmark shapes, reached by making one GEMM
    # dimension long while the oracle's work stays small:
    #   gate/up, 128-row tiles, one tile per work range, a ragged last round handed out as half-width items
    "wide128_gateup_halves": syn.Workload("wide128_gateup_halves", T=300, H=128, I=9216, E=8, top_k=2),
    #   gate/up, 256-row tiles, every expert cut into two tiles
    "wide256_gateup_split": syn.Workload("wide256_gateup_split", T=700, H=128, I=16384, E=4, top_k=2),
    #   down projection, 256-row tiles, every expert cut into two tiles (which share their weights through L2)
    "wide256_down_split": syn.Workload("wide256_down_split", T=700, H=32768, I=128, E=4, top_k=2),
    #   few experts, tall tiles and a long K: inside the forward the down projection cuts K in halves (fp32
    #   partial sums, added by the combine); 2.5 column slabs of 256, ragged tiles, an odd step count per half
    "down_k_halves": syn.Workload("down_k_halves", T=300, H=640, I=4224, E=4, top_k=2),
    #   more than 64 tiles of up to 16 row blocks: both GEMMs wide, work cut into equal parts and
    #   walked alternating between tall and short tiles
    "wide256_zigzag": syn.Workload("wide256_zigzag", T=2800, H=1024, I=512, E=128, top_k=8),
}


@pytest.fixture(scope="module", params=list(CASES))
def case(request):
    wl = CASES[request.param]
    print(f"\n[case] {wl}", flush=True)
    gpu = syn.make_inputs(wl, seed=0, device="cuda")         # (the generator gives the same bits on either device)
    cpu = gpu.to("cpu")
    return wl, cpu, gpu, oracle_all(cpu)


def test_route(case):
    wl, cpu, gpu, (p, ids, w, margin, *_rest, keys) = case
    cfg = moe.MoEConfig.from_workload(wl)
    ids_g, w_g = moe.moe_route(cfg, gpu.x, gpu.x_scale, gpu.router_w, gpu.bias)
    torch.cuda.synchronize()
    other, swapped, _ = compare_routing(ids_g, w_g, ids, w, margin, wl.routed_scale, wl.E, keys)
    print(f"route {wl.name}: other-set tokens={other} swapped-slot tokens={swapped} (margin<1e-6 only)")
    s = w_g.sum(dim=1).cpu().numpy()
    np.testing.assert_allclose(s, wl.routed_scale, rtol=1e-5)           # renormalised weights


def test_permute(case):
    wl, cpu, gpu, (p, ids, w, margin, offsets, sorted_pair, inv, _k) = case
    cfg = moe.MoEConfig.from_workload(wl)
    ids_d = torch.from_numpy(ids).cuda()
    off_g, sp_g, inv_g, tiles, sched = moe.moe_permute(cfg, ids_d)
    torch.cuda.synchronize()
    assert np.array_equal(off_g.cpu().numpy(), offsets)
    assert np.array_equal(sp_g.cpu().numpy()[: len(sorted_pair)], sorted_pair)      # rows of the kept pairs
    assert np.array_equal(inv_g.cpu().numpy(), inv)
    n = check_tiles(tiles, sched, offsets, moe.moe_tile_rows(cfg))
    assert n <= moe.moe_max_tiles(cfg)


def _staged(case):
    wl, cpu, gpu, (p, ids, w, margin, offsets, sorted_pair, inv, _k) = case
    cfg = moe.MoEConfig.from_workload(wl)
    ids_d = torch.from_numpy(ids).cuda()
    off_g, sp_g, inv_g, tiles, sched = moe.moe_permute(cfg, ids_d)
    tok = sorted_pair // wl.top_k                            # one entry per kept pair, in sorted-row order
    exp = ids.reshape(-1)[sorted_pair] - wl.local_offset     # index into the (local) weight arrays
    return wl, cfg, gpu, p, ids, w, sp_g, inv_g, tiles, sched, tok, exp, inv


def _gemm_x(gpu, p):
    """Hidden states as the gate/up GEMM reads them.  When the layer quantises bf16 input itself the
    staged GEMM is fed the oracle's quantisation (the GPU's own is checked in test_quantize_act)."""
    if not gpu.wl.quantize_x:
        return gpu.x, gpu.x_scale
    xq = torch.from_numpy(p._x.reshape(gpu.wl.T, gpu.wl.H)).view(torch.float8_e4m3fn).cuda()
    return xq, torch.from_numpy(p._xs.reshape(gpu.wl.T, -1)).cuda()


def _act_f64(act, scale):
    """Activations as the GPU stored them (bf16, or fp8 payload x 1x128 scale) in float64."""
    a = f64(act)
    if scale is not None:
        a = a * np.repeat(f64(scale), 128, axis=1)
    return a


def test_gemm_swiglu(case):
    wl, cfg, gpu, p, ids, w, sp_g, inv_g, tiles, sched, tok, exp, inv = _staged(case)
    act_g, sc_g = moe.moe_grouped_gemm_swiglu(cfg, *_gemm_x(gpu, p), gpu.w1, gpu.w1_scale, sp_g, tiles, sched)
    torch.cuda.synchronize()
    ref = orc.swiglu_rows(p, tok, exp)
    n = len(tok)                                             # rows beyond the kept pairs are never written
    act_g, sc_g = act_g[:n], (None if sc_g is None else sc_g[:n])
    max_rel, mean_rel = err_stats(_act_f64(act_g, sc_g), ref)
    print(f"swiglu {wl.name}: max_rel={max_rel:.2e} mean_rel={mean_rel:.2e}")
    if wl.fp8:
        # re-quantised to e4m3 (3 mantissa bits) per 1x128 block with scale = amax/448
        assert max_rel <= 2 ** -4 + 1e-3 and mean_rel <= 3.5e-2
        q = act_g.float().abs().reshape(n, -1, 128).amax(dim=-1)
        amax_ref = torch.from_numpy(np.abs(ref).reshape(n, -1, 128).max(axis=-1)).cuda()
        assert ((q == 448) | (amax_ref == 0)).all(), "every non-zero block must use the full e4m3 range"
        np.testing.assert_allclose(sc_g.cpu().numpy(), np.maximum(amax_ref.cpu().numpy(), 1e-30) / 448, rtol=1e-2)
    else:
        assert max_rel <= 6e-3 and mean_rel <= 3e-3      # one bf16 rounding of an fp32 accumulation


def test_gemm_down(case):
    wl, cfg, gpu, p, ids, w, sp_g, inv_g, tiles, sched, tok, exp, inv = _staged(case)
    act_g, sc_g = moe.moe_grouped_gemm_swiglu(cfg, *_gemm_x(gpu, p), gpu.w1, gpu.w1_scale, sp_g, tiles, sched)
    y_g = moe.moe_grouped_gemm_down(cfg, act_g, sc_g, gpu.w2, gpu.w2_scale, tiles, sched)
    torch.cuda.synchronize()
    n = len(tok)
    ref = orc.down_rows(p, exp, _act_f64(act_g[:n], None if sc_g is None else sc_g[:n]))   # from the very activations the GPU consumed
    max_rel, mean_rel = err_stats(f64(y_g[:n]), ref)
    print(f"down {wl.name}: max_rel={max_rel:.2e} mean_rel={mean_rel:.2e}")
    assert max_rel <= 6e-3 and mean_rel <= 3e-3


def test_combine(case):
    wl, cfg, gpu, p, ids, w, sp_g, inv_g, tiles, sched, tok, exp, inv = _staged(case)
    g = torch.Generator().manual_seed(1)
    y = torch.randn((cfg.P, wl.H), generator=g).bfloat16()
    w32 = torch.from_numpy(w.astype(np.float32))
    out_g = moe.moe_combine(cfg, y.cuda(), w32.cuda(), inv_g)
    torch.cuda.synchronize()
    ref = orc.combine(w32.numpy().astype(np.float64), inv, f64(y))
    got = f64(out_g)
    # fp32 sum of k products, one rounding to bf16: within half a bf16 ulp of the exact sum plus
    # the fp32 rounding of the k terms (which matters where the terms cancel)
    mag = orc.combine(np.abs(w32.numpy()).astype(np.float64), inv, np.abs(f64(y)))
    assert (np.abs(got - ref) <= np.abs(ref) * 2.0 ** -8 + mag * 2.0 ** -21 + 1e-30).all()
    ref_bits = torch.from_numpy(ref).to(torch.bfloat16)
    assert (ref_bits.view(torch.int16) != out_g.cpu().view(torch.int16)).float().mean() < 1e-3


def test_forward(case):
    wl, cpu, gpu, (p, ids, w, margin, *_rest, keys) = case
    out_g = moe.forward_inputs(gpu)
    torch.cuda.synchronize()
    out2 = moe.forward_inputs(gpu)
    torch.cuda.synchronize()
    assert torch.equal(out_g.view(torch.int16), out2.view(torch.int16)), "forward is not run-to-run identical"
    ref, ids_r, w_r, margin_r = orc.forward(p)
    cfg = moe.MoEConfig.from_workload(wl)
    ids_g, w_g = moe.moe_route(cfg, gpu.x, gpu.x_scale, gpu.router_w, gpu.bias)
    other, swapped, same_set = compare_routing(ids_g, w_g, ids_r, w_r, margin_r, wl.routed_scale, wl.E, keys)
    got = f64(out_g)
    assert np.isfinite(got).all()
    max_rel, mean_rel = err_stats(got[same_set], ref[same_set])
    print(f"forward {wl.name}: max_rel={max_rel:.2e} mean_rel={mean_rel:.2e} tie-excused tokens={other}")
    assert max_rel <= TOL_MAX[wl.fp8] and mean_rel <= TOL_MEAN[wl.fp8]


@pytest.mark.parametrize("T, H, scale", [(1, 128, 1.0), (37, 384, 30.0), (300, 7168, 1.0), (64, 2048, 1e-3)])
def test_quantize_act_is_bit_exact(T, H, scale):
    """The 1x128 activation quantiser against the oracle: same code bytes, same scale bits."""
    g = torch.Generator().manual_seed(T * 1000 + H)
    x = (torch.randn((T, H), generator=g) * scale).bfloat16()
    x[0, :128] = 0                                           # an all-zero block (scale 1, codes 0)
    if T > 1:
        x[1, :128] = x[1, :128].abs()                        # a block without negative values
        x[T - 1, H - 128:] = torch.arange(128).bfloat16() * -0.25    # exact small multiples, largest last
        x[T // 2, 5] = -0.0
    cfg = moe.MoEConfig(T=T, H=H, I=128, E=8, top_k=2, dtype=1)
    print(f"\n[quantize] T={T} H={H} scale={scale}", flush=True)
    xq, xs = moe.moe_quantize_act(cfg, x.cuda())
    torch.cuda.synchronize()
    q_ref, s_ref = orc.quantize_rows_1x128(x)
    assert np.array_equal(xs.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(xq.cpu().view(torch.uint8).numpy(), q_ref)


@pytest.mark.parametrize("name", ["grouped", "fp8_grouped", "local_fp8", "qx_small"])
def test_generator_gives_the_same_bits_on_cpu_and_gpu(name):
    """The seeded inputs are a pure function of (seed, tensor, index), computed with integer
    operations: a draw on the GPU equals a draw on the CPU bit for bit (block-quantised payloads and
    scales included), so it does not matter where a test or the benchmark draws them."""
    wl = CASES[name]
    a, b = syn.make_inputs(wl, seed=5), syn.make_inputs(wl, seed=5, device="cuda").to("cpu")
    for field in ("x", "router_w", "bias", "w1", "w2", "x_scale", "w1_scale", "w2_scale"):
        u, v = getattr(a, field), getattr(b, field)
        assert (u is None) == (v is None), field
        if u is not None:
            assert u.dtype == v.dtype and torch.equal(u.view(torch.uint8), v.view(torch.uint8)), field


def test_local_share_without_any_pair():
    """A device whose experts nobody chose: empty schedule, both GEMMs launch with nothing to do,
    and the combine writes exact zeros."""
    wl = syn.Workload("nolocal", T=40, H=256, I=128, E=16, top_k=2, local_offset=12, local_experts=4)
    cfg = moe.MoEConfig.from_workload(wl)
    gpu = syn.make_inputs(wl, seed=3).to("cuda")
    rng = np.random.default_rng(3)
    ids = rng.integers(0, 12, size=(wl.T, wl.top_k)).astype(np.int32)        # experts 0..11 only
    off, sp, inv, tiles, sched = moe.moe_permute(cfg, torch.from_numpy(ids).cuda())
    act, _ = moe.moe_grouped_gemm_swiglu(cfg, gpu.x, None, gpu.w1, None, sp, tiles, sched)
    y = moe.moe_grouped_gemm_down(cfg, act, None, gpu.w2, None, tiles, sched)
    w = torch.rand((wl.T, wl.top_k), device="cuda")
    out = moe.moe_combine(cfg, y, w, inv)
    torch.cuda.synchronize()
    assert off.cpu().tolist() == [0] * 5 and sched.cpu().tolist()[:10] == [0] * 10
    assert (inv.cpu().numpy() == -1).all()
    assert not out.view(torch.int16).cpu().numpy().any()


def test_forward_zero_tokens_and_errors():
    wl = syn.Workload("empty", T=0, H=128, I=64, E=8, top_k=2)
    cfg = moe.MoEConfig.from_workload(wl)
    ids = torch.empty((0, 2), dtype=torch.int32, device="cuda")
    off, sp, inv, tiles, sched = moe.moe_permute(cfg, ids)
    torch.cuda.synchronize()
    assert off.cpu().tolist() == [0] * 9 and sched.cpu().tolist()[:10] == [0] * 10
    # workspace one byte short is refused before anything is enqueued
    wl = syn.WORKLOADS["tiny"]
    gpu = syn.make_inputs(wl, seed=0).to("cuda")
    cfg = moe.MoEConfig.from_workload(wl)
    small = torch.empty((moe.moe_workspace_size(cfg) - 256,), dtype=torch.uint8, device="cuda")
    with pytest.raises(moe.MoEError, match="workspace"):
        moe.moe_forward(cfg, gpu.x, None, gpu.router_w, None, gpu.w1, None, gpu.w2, None, workspace=small)


def test_permute_drops_out_of_range_ids_and_handles_one_hot_expert():
    wl = syn.Workload("drop", T=50, H=128, I=64, E=8, top_k=2)
    cfg = moe.MoEConfig.from_workload(wl)
    rng = np.random.default_rng(0)
    ids = rng.integers(0, 8, size=(50, 2)).astype(np.int32)
    ids[::7, 1] = -1
    ids[3::11, 0] = 8
    off, sp, inv, tiles, sched = moe.moe_permute(cfg, torch.from_numpy(ids).cuda())
    torch.cuda.synchronize()
    flat = ids.reshape(-1)
    keep = (flat >= 0) & (flat < 8)
    off_r, sp_r, inv_r = orc.permute(flat[keep].reshape(-1, 1), 8)      # oracle on the kept pairs
    kept_pairs = np.nonzero(keep)[0]
    assert np.array_equal(off.cpu().numpy(), off_r)
    assert np.array_equal(sp.cpu().numpy()[: keep.sum()], kept_pairs[sp_r])
    inv_g = inv.cpu().numpy()
    assert (inv_g[~keep] == -1).all() and np.array_equal(inv_g[keep], inv_r)
    # every pair on one expert: maximum rows for a single segment
    ids = np.full((50, 2), 5, dtype=np.int32)
    off, sp, inv, tiles, sched = moe.moe_permute(cfg, torch.from_numpy(ids).cuda())
    torch.cuda.synchronize()
    off_r, sp_r, inv_r = orc.permute(ids, 8)
    assert np.array_equal(off.cpu().numpy(), off_r) and np.array_equal(sp.cpu().numpy(), sp_r)
    check_tiles(tiles, sched, off_r, moe.moe_tile_rows(cfg))


@pytest.mark.parametrize("T, k, E, lo, n", [(2500, 8, 256, 0, 0), (3001, 6, 64, 16, 24), (9000, 8, 512, 0, 0),
                                            (2049, 1, 3, 0, 0)])
def test_permute_many_pairs_over_several_workgroups(T, k, E, lo, n):
    """Enough pairs that the sort-scatter runs as several independent workgroups: ragged last
    slice, ids outside the (local) expert range, experts without tokens, a heavily loaded expert."""
    wl = syn.Workload("many_pairs", T=T, H=128, I=64, E=E, top_k=k, local_offset=lo, local_experts=n)
    cfg = moe.MoEConfig.from_workload(wl)
    rng = np.random.default_rng(T + E)
    ids = rng.integers(0, E, size=(T, k)).astype(np.int32)
    ids[rng.random((T, k)) < 0.3] = min(5, E - 1)            # one expert far above the others
    if E > 8:
        ids[ids == 7] = 6                                    # an expert nobody chose
    ids[::97, 0] = -1
    ids[5::131, k - 1] = E
    print(f"\n[permute] T={T} k={k} E={E} local=({lo},{n})", flush=True)
    off, sp, inv, tiles, sched = moe.moe_permute(cfg, torch.from_numpy(ids).cuda())
    torch.cuda.synchronize()
    first, count = (lo, n) if n > 0 else (0, E)
    flat = ids.reshape(-1)
    keep = (flat >= first) & (flat < first + count)
    off_r, sp_r, inv_r = orc.permute((flat[keep] - first).reshape(-1, 1), count)   # oracle on the kept pairs
    kept_pairs = np.nonzero(keep)[0]
    assert np.array_equal(off.cpu().numpy(), off_r)
    assert np.array_equal(sp.cpu().numpy()[: keep.sum()], kept_pairs[sp_r])
    inv_g = inv.cpu().numpy()
    assert (inv_g[~keep] == -1).all() and np.array_equal(inv_g[keep], inv_r)
    check_tiles(tiles, sched, off_r, moe.moe_tile_rows(cfg))


def test_forward_with_k_in_halves_agrees_with_the_staged_steps_and_replays_from_a_graph():
    """Inside the forward the down projection of `down_k_halves` cuts K in two and the combine adds the
    partial sums; the stand-alone steps reduce over the whole of K.  The two differ only in the order of
    the fp32 sum: almost every output element has the same bits, the rest are a bf16 rounding apart.
    The forward's five launches, captured once, replay to the eager bits."""
    wl = CASES["down_k_halves"]
    gpu = syn.make_inputs(wl, seed=3, device="cuda")
    cfg = moe.MoEConfig.from_workload(wl)
    assert moe.moe_gemm_plan(cfg, "down")["k_split"] == 2
    ws = torch.empty((moe.moe_workspace_size(cfg),), dtype=torch.uint8, device="cuda")
    out = torch.empty((wl.T, wl.H), dtype=torch.bfloat16, device="cuda")
    moe.forward_inputs(gpu, out=out, workspace=ws)
    torch.cuda.synchronize()
    eager = out.clone()
    # the same layer step by step
    ids, w = moe.moe_route(cfg, gpu.x, gpu.x_scale, gpu.router_w, gpu.bias)
    off, sp, inv, tiles, sched = moe.moe_permute(cfg, ids)
    act, act_scale = moe.moe_grouped_gemm_swiglu(cfg, gpu.x, gpu.x_scale, gpu.w1, gpu.w1_scale, sp, tiles, sched)
    y = moe.moe_grouped_gemm_down(cfg, act, act_scale, gpu.w2, gpu.w2_scale, tiles, sched)
    staged = moe.moe_combine(cfg, y, w, inv)
    torch.cuda.synchronize()
    a, b = f64(eager), f64(staged)
    same = (eager.view(torch.int16) == staged.view(torch.int16)).float().mean().item()
    print(f"  forward (K in halves) vs staged steps: {same:.4f} of the elements bit-equal, max diff {np.abs(a - b).max():.3e}")
    assert same > 0.9
    assert (np.abs(a - b) <= np.abs(b) * 2.0 ** -6 + np.abs(b).max() * 2.0 ** -7).all()
    # graph replay, with eager work between the replays
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        moe.forward_inputs(gpu, out=out, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        moe.forward_inputs(gpu, out=out, workspace=ws)
    for rep in range(3):
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {rep} differs"
        moe.forward_inputs(gpu, out=out, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16))
