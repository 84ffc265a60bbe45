"""Pins of the CPU oracle against things other than itself (no GPU needed).

The paper prints no numeric values for the MoE operator, so each oracle
function is tied to what mathematics fixes instead: brute force on tiny
inputs, closed forms, special cases that collapse to a float64 library matmul,
library conversions of every bf16 / e4m3 code, and invariants.
"""
import itertools

import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from paper_2602_19128_amd import synthetic as syn


def _wl(**kw):
    base = dict(name="t", T=8, H=64, I=32, E=8, top_k=2)
    base.update(kw)
    return syn.Workload(**base)


def _f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


# ---------------------------------------------------------------- decoding


def test_bf16_decode_all_codes_match_library():
    codes = np.arange(65536, dtype=np.uint16)
    lib = torch.from_numpy(codes.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    mine = np.array([orc.bf16_to_f64(int(c)) for c in codes])
    nan = np.isnan(lib)
    assert np.array_equal(np.isnan(mine), nan)
    assert np.array_equal(mine[~nan], lib[~nan])


def test_e4m3_decode_all_codes_match_library():
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    mine = np.array([orc.e4m3_to_f64(int(c)) for c in codes])
    nan = np.isnan(lib)
    assert nan.sum() == 2                      # S.1111.111 only; no infinities
    assert np.array_equal(np.isnan(mine), nan)
    assert np.array_equal(mine[~nan], lib[~nan])
    assert mine[0x7E] == 448.0 and mine[0x01] == 2.0 ** -9


# ---------------------------------------------------------------- router logits


@pytest.mark.parametrize("fp8", [False, True])
def test_logits_equal_float64_library_matmul(fp8):
    wl = _wl(T=5, H=384, I=128, E=6, top_k=2, fp8=fp8)
    inp = syn.make_inputs(wl, seed=3)
    p = orc.problem_from_inputs(inp)
    z = orc.router_logits(p)
    x = _f64(inp.x)
    if fp8:
        x = x * np.repeat(_f64(inp.x_scale), 128, axis=1)
    ref = x @ _f64(inp.router_w).T
    assert z.shape == (5, 6)
    np.testing.assert_allclose(z, ref, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- routing


def _route_only(z, *, top_k, scoring="softmax", n_group=1, topk_group=1, topn=2, bias=None,
                scale=1.0, renorm=True):
    T, E = z.shape
    p = orc.Problem(T=T, H=1, I=1, E=E, top_k=top_k, scoring=scoring, renormalize=renorm,
                    n_group=n_group, topk_group=topk_group, group_score_topn=topn,
                    routed_scale=scale, bias=bias)
    return orc.route(p, z)


def _brute_force_choice(c, k, eligible):
    """argmax over all k-subsets of eligible experts of the summed key."""
    idx = [e for e in range(len(c)) if eligible[e]]
    best = max(itertools.combinations(idx, k), key=lambda s: sum(c[e] for e in s))
    return set(best)


def test_topk_softmax_brute_force_and_closed_form():
    rng = np.random.default_rng(0)
    z = rng.normal(size=(40, 9))
    for k in (1, 2, 4, 9):
        ids, w, margin = _route_only(z, top_k=k)
        s = np.exp(z - z.max(1, keepdims=True))
        s /= s.sum(1, keepdims=True)
        for t in range(z.shape[0]):
            assert len(set(ids[t])) == k
            assert set(ids[t]) == _brute_force_choice(s[t], k, [True] * 9)
            # reported in descending key order
            assert all(s[t, ids[t, j]] >= s[t, ids[t, j + 1]] for j in range(k - 1))
            # closed form: renormalised softmax == softmax over the selected logits
            zs = z[t, ids[t]]
            cf = np.exp(zs - zs.max())
            cf /= cf.sum()
            np.testing.assert_allclose(w[t], cf, rtol=1e-13)
            assert abs(w[t].sum() - 1.0) < 1e-14
            # every left-out key <= smallest chosen key; margin is that gap
            rest = np.delete(s[t], ids[t])
            if rest.size:
                assert rest.max() <= s[t, ids[t]].min()
                assert margin[t] == pytest.approx(s[t, ids[t]].min() - rest.max(), abs=1e-15)
            else:
                assert margin[t] == np.inf


def test_softmax_without_renormalisation_keeps_full_softmax_mass():
    rng = np.random.default_rng(1)
    z = rng.normal(size=(6, 7))
    ids, w, _ = _route_only(z, top_k=3, renorm=False, scale=1.0)
    s = np.exp(z) / np.exp(z).sum(1, keepdims=True)
    for t in range(6):
        np.testing.assert_allclose(w[t], s[t, ids[t]], rtol=1e-13)


def test_ties_go_to_lower_index():
    z = np.zeros((1, 8))
    ids, w, margin = _route_only(z, top_k=3)
    assert ids.tolist() == [[0, 1, 2]]
    assert margin[0] == 0.0
    z = np.array([[0.0, 1.0, 1.0, -1.0, 1.0, 0.5]])
    ids, _, _ = _route_only(z, top_k=2)
    assert ids.tolist() == [[1, 2]]
    # groups: equal block scores -> lower block index kept
    z = np.array([[0.3, 0.1, 0.3, 0.1, 0.3, 0.1, 0.3, 0.1]])
    ids, _, margin = _route_only(z, top_k=2, scoring="sigmoid", n_group=4, topk_group=2, topn=2)
    assert sorted(ids[0].tolist()) == [0, 2] and ids[0, 0] == 0
    assert margin[0] == 0.0


def _sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def test_group_routing_brute_force_small():
    rng = np.random.default_rng(2)
    E, G, kg, topn, k = 8, 4, 2, 2, 3
    gsz = E // G
    z = rng.normal(size=(60, E))
    bias = rng.uniform(-0.1, 0.1, size=E).astype(np.float32)
    ids, w, margin = _route_only(z, top_k=k, scoring="sigmoid", n_group=G, topk_group=kg, topn=topn,
                                 bias=bias, scale=2.5)
    s = _sigmoid(z)
    c = s + bias.astype(np.float64)
    for t in range(z.shape[0]):
        # block score by brute force: best sum over all `topn`-subsets of the block
        gs = [max(sum(c[t, g * gsz + j] for j in sub)
                  for sub in itertools.combinations(range(gsz), topn)) for g in range(G)]
        kept = max(itertools.combinations(range(G), kg), key=lambda gg: sum(gs[g] for g in gg))
        eligible = [(e // gsz) in kept for e in range(E)]
        assert set(ids[t]) == _brute_force_choice(c[t], k, eligible)
        assert len({e // gsz for e in ids[t]}) <= kg
        # weights: unbiased sigmoid, renormalised, times the routed scale
        sel = s[t, ids[t]]
        np.testing.assert_allclose(w[t], 2.5 * sel / sel.sum(), rtol=1e-13)
        assert abs(w[t].sum() - 2.5) < 1e-13
        # margin = min(expert gap, block gap)
        dropped = [gs[g] for g in range(G) if g not in kept]
        gap_g = min(gs[g] for g in kept) - max(dropped)
        rest = [c[t, e] for e in range(E) if eligible[e] and e not in set(ids[t])]
        gap_e = min(c[t, e] for e in ids[t]) - max(rest)
        assert margin[t] == pytest.approx(min(gap_g, gap_e), abs=1e-15)


def test_group_routing_reductions():
    rng = np.random.default_rng(3)
    E, k = 32, 4
    z = rng.normal(size=(50, E))
    bias = rng.uniform(-0.1, 0.1, size=E).astype(np.float32)
    plain = _route_only(z, top_k=k, scoring="sigmoid", bias=bias)
    one_group = _route_only(z, top_k=k, scoring="sigmoid", bias=bias, n_group=1, topk_group=1)
    all_groups = _route_only(z, top_k=k, scoring="sigmoid", bias=bias, n_group=4, topk_group=4)
    for other in (one_group, all_groups):
        assert np.array_equal(plain[0], other[0])
        np.testing.assert_array_equal(plain[1], other[1])
    # no bias, scale 1: w = s / sum s over the chosen ones
    ids, w, _ = _route_only(z, top_k=k, scoring="sigmoid", n_group=4, topk_group=2)
    s = _sigmoid(z)
    for t in range(z.shape[0]):
        sel = s[t, ids[t]]
        np.testing.assert_allclose(w[t], sel / sel.sum(), rtol=1e-13)
        assert len({e // 8 for e in ids[t]}) <= 2
    # bias changes the choice but never the weight formula
    big = np.zeros(E, dtype=np.float32)
    big[5] = 10.0
    ids, w, _ = _route_only(z, top_k=k, scoring="sigmoid", bias=big, renorm=False)
    assert (ids[:, 0] == 5).all()
    np.testing.assert_allclose(w[:, 0], s[:, 5], rtol=1e-13)


def test_group_score_uses_topn_not_max_or_sum():
    # block 0: one large key; block 1: two medium keys.  top-1 keeps block 0,
    # top-2 keeps block 1, the plain block sum would keep block 2.
    c = np.array([[0.90, 0.01, 0.01, 0.01, 0.55, 0.55, 0.01, 0.01, 0.40, 0.40, 0.40, 0.40]])
    z = np.log(c / (1 - c))
    for topn, want in ((1, 0), (2, 1), (4, 2)):
        ids, _, _ = _route_only(z, top_k=1, scoring="sigmoid", n_group=3, topk_group=1, topn=topn)
        assert ids[0, 0] // 4 == want


# ---------------------------------------------------------------- permutation


def test_permute_is_the_stable_sort_by_expert():
    rng = np.random.default_rng(4)
    T, k, E = 37, 3, 11
    ids = rng.integers(0, E, size=(T, k)).astype(np.int32)
    ids[:, 0] = np.where(ids[:, 0] == 7, 6, ids[:, 0])       # leave expert 7 sparse
    offsets, sorted_pair, inv = orc.permute(ids, E)
    flat = ids.reshape(-1)
    P = flat.size
    assert offsets[0] == 0 and offsets[E] == P
    assert np.array_equal(np.diff(offsets), np.bincount(flat, minlength=E))
    assert np.array_equal(sorted_pair, np.argsort(flat, kind="stable"))
    assert np.array_equal(inv[sorted_pair], np.arange(P))
    assert np.array_equal(sorted_pair[inv], np.arange(P))
    for e in range(E):
        seg = sorted_pair[offsets[e]:offsets[e + 1]]
        assert (flat[seg] == e).all()
        assert (np.diff(seg) > 0).all()
    data = rng.normal(size=(P, 4))
    assert np.array_equal(data[sorted_pair][inv], data)          # gather then scatter back


def test_permute_empty_experts_and_single_expert():
    ids = np.full((5, 2), 3, dtype=np.int32)
    offsets, sorted_pair, inv = orc.permute(ids, 6)
    assert offsets.tolist() == [0, 0, 0, 0, 10, 10, 10]
    assert sorted_pair.tolist() == list(range(10)) and inv.tolist() == list(range(10))


# ---------------------------------------------------------------- expert FFN


def _silu(v):
    return v / (1.0 + np.exp(-v))


def _dense_mlp(x, w1, w2, I):
    g = x @ w1[:I].T
    u = x @ w1[I:].T
    return (_silu(g) * u) @ w2.T


def test_single_expert_is_a_dense_swiglu_mlp():
    wl = _wl(T=7, H=96, I=40, E=1, top_k=1)
    inp = syn.make_inputs(wl, seed=5)
    p = orc.problem_from_inputs(inp)
    out, ids, w, margin = orc.forward(p)
    assert (ids == 0).all() and np.allclose(w, 1.0) and np.isinf(margin).all()
    ref = _dense_mlp(_f64(inp.x), _f64(inp.w1[0]), _f64(inp.w2[0]), wl.I)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    # gate and up are not interchangeable: the swapped reading must differ
    w1 = _f64(inp.w1[0])
    swapped = _dense_mlp(_f64(inp.x), np.concatenate([w1[wl.I:], w1[:wl.I]]), _f64(inp.w2[0]), wl.I)
    assert np.abs(swapped - ref).max() > 1e-3


def test_all_experts_selected_is_the_weighted_dense_sum():
    wl = _wl(T=6, H=64, I=24, E=4, top_k=4)
    inp = syn.make_inputs(wl, seed=6)
    p = orc.problem_from_inputs(inp)
    out, ids, w, _ = orc.forward(p)
    x = _f64(inp.x)
    z = x @ _f64(inp.router_w).T
    s = np.exp(z - z.max(1, keepdims=True))
    s /= s.sum(1, keepdims=True)
    ref = np.zeros_like(out)
    for e in range(4):
        ref += s[:, e:e + 1] * _dense_mlp(x, _f64(inp.w1[e]), _f64(inp.w2[e]), wl.I)
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-13)
    assert all(sorted(r) == [0, 1, 2, 3] for r in ids.tolist())


def test_staged_steps_compose_to_the_definition():
    wl = _wl(T=9, H=64, I=48, E=5, top_k=2)
    inp = syn.make_inputs(wl, seed=7)
    p = orc.problem_from_inputs(inp)
    out, ids, w, _ = orc.forward(p)
    z = orc.router_logits(p)
    ids2, w2, _ = orc.route(p, z)
    assert np.array_equal(ids, ids2) and np.array_equal(w, w2)
    offsets, sorted_pair, inv = orc.permute(ids, wl.E)
    tok = sorted_pair // wl.top_k
    exp = ids.reshape(-1)[sorted_pair]
    assert np.array_equal(exp, np.repeat(np.arange(wl.E), np.diff(offsets)))
    act = orc.swiglu_rows(p, tok, exp)
    y = orc.down_rows(p, exp, act)
    staged = orc.combine(w, inv, y)
    np.testing.assert_allclose(staged, out, rtol=1e-13, atol=1e-15)
    # each staged piece against the float64 library for one expert's rows
    e = int(exp[0])
    rows = np.nonzero(exp == e)[0]
    x = _f64(inp.x)[tok[rows]]
    w1 = _f64(inp.w1[e])
    np.testing.assert_allclose(act[rows], _silu(x @ w1[:wl.I].T) * (x @ w1[wl.I:].T), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(y[rows], act[rows] @ _f64(inp.w2[e]).T, rtol=1e-12, atol=1e-14)


def test_combine_definition_and_slot_order():
    rng = np.random.default_rng(8)
    T, k, H = 5, 3, 7
    w = rng.normal(size=(T, k))
    y = rng.normal(size=(T * k, H))
    inv = rng.permutation(T * k).astype(np.int32)
    out = orc.combine(w, inv, y)
    ref = np.einsum("tj,tjh->th", w, y[inv].reshape(T, k, H))
    np.testing.assert_allclose(out, ref, rtol=1e-13, atol=1e-15)


def test_invariants_linearity_zero_duplicates_and_token_order():
    wl = _wl(T=10, H=64, I=32, E=6, top_k=2)
    inp = syn.make_inputs(wl, seed=9)
    p = orc.problem_from_inputs(inp)
    out, ids, w, _ = orc.forward(p)
    # W2 * 2 is exact in bf16 -> output doubles exactly
    inp2 = syn.MoEInputs(wl, inp.x, inp.router_w, inp.bias, inp.w1, inp.w2 * 2)
    out2, _, _, _ = orc.forward(orc.problem_from_inputs(inp2))
    assert np.array_equal(out2, 2.0 * out)
    # x = 0 -> output 0
    inp0 = syn.MoEInputs(wl, torch.zeros_like(inp.x), inp.router_w, inp.bias, inp.w1, inp.w2)
    out0, _, _, _ = orc.forward(orc.problem_from_inputs(inp0))
    assert (out0 == 0).all()
    # duplicated tokens give identical rows; permuting tokens permutes rows bit-exactly
    perm = torch.tensor([3, 3, 0, 9, 1, 1, 7, 2, 5, 4])
    inpp = syn.MoEInputs(wl, inp.x[perm].contiguous(), inp.router_w, inp.bias, inp.w1, inp.w2)
    outp, idsp, _, _ = orc.forward(orc.problem_from_inputs(inpp))
    assert np.array_equal(outp, out[perm.numpy()])
    assert np.array_equal(idsp, ids[perm.numpy()])


# ---------------------------------------------------------------- fp8 block scales


def test_fp8_with_unit_scales_equals_bf16_on_representable_values():
    wl = _wl(T=4, H=128, I=128, E=3, top_k=2)
    g = torch.Generator().manual_seed(10)
    small = lambda *s: torch.randint(-3, 4, s, generator=g).float()      # exact in e4m3 and bf16
    x, w1, w2 = small(4, 128), small(3, 256, 128) / 16, small(3, 128, 128) / 16
    rw = torch.randn(3, 128, generator=g) / 11
    bf = syn.MoEInputs(wl, x.bfloat16(), rw, None, w1.bfloat16(), w2.bfloat16())
    wl8 = wl.replace(fp8=True)
    f8 = syn.MoEInputs(wl8, x.to(torch.float8_e4m3fn), rw, None, w1.to(torch.float8_e4m3fn),
                       w2.to(torch.float8_e4m3fn), torch.ones(4, 1), torch.ones(3, 2, 1), torch.ones(3, 1, 1))
    a = orc.forward(orc.problem_from_inputs(bf))
    b = orc.forward(orc.problem_from_inputs(f8))
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_fp8_block_scales_index_the_right_blocks():
    # non-square scale grids: H/128 = 3, I/128 = 1 -> a transposed scale index would read wrong blocks
    wl = _wl(T=6, H=384, I=128, E=2, top_k=1, fp8=True)
    inp = syn.make_inputs(wl, seed=11)
    p = orc.problem_from_inputs(inp)
    out, ids, w, _ = orc.forward(p)
    x = _f64(inp.x) * np.repeat(_f64(inp.x_scale), 128, axis=1)
    ref = np.zeros_like(out)
    for t in range(wl.T):
        e = int(ids[t, 0])
        w1 = _f64(inp.w1[e]) * np.kron(_f64(inp.w1_scale[e]), np.ones((128, 128)))
        w2 = _f64(inp.w2[e]) * np.kron(_f64(inp.w2_scale[e]), np.ones((128, 128)))
        ref[t] = w[t, 0] * _dense_mlp(x[t:t + 1], w1, w2, wl.I)[0]
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-14)


def test_fp8_quantised_inputs_are_close_to_their_source():
    g = torch.Generator().manual_seed(12)
    v = torch.randn(256, 256, generator=g)
    q, s = syn.quantize_blocks_128x128(v)
    deq = q.float() * torch.kron(s, torch.ones(128, 128))
    rel = ((deq - v).abs() / v.abs().clamp_min(1e-3 * v.abs().max())).max().item()
    assert rel <= 2 ** -4 + 1e-6
    q, s = syn.quantize_rows_1x128(v)
    deq = q.float() * s.repeat_interleave(128, dim=1)
    assert ((deq - v).abs() <= v.abs() * 2 ** -4 + s.repeat_interleave(128, dim=1) * 2 ** -10 + 1e-12).all()
    assert q.float().abs().max() <= 448


# ---------------------------------------------------------------- local-expert mode


@pytest.mark.parametrize("fp8", [False, True])
def test_local_shares_partition_the_layer(fp8):
    """Disjoint local ranges that cover every expert add up to the full layer, a range that
    holds none of a token's experts gives exactly zero, the full range changes nothing."""
    wl = _wl(T=9, H=128, I=128, E=8, top_k=3, fp8=fp8)
    full = syn.make_inputs(wl, seed=5)
    p = orc.problem_from_inputs(full)
    ref, ids, w, margin = orc.forward(p)
    total = np.zeros_like(ref)
    for lo, n in [(0, 3), (3, 1), (4, 4)]:
        share = full.local_share(lo, n)
        out, ids_s, w_s, _ = orc.forward(orc.problem_from_inputs(share))
        assert np.array_equal(ids_s, ids) and np.array_equal(w_s, w)        # routing is that of the full layer
        total += out
        untouched = ~((ids >= lo) & (ids < lo + n)).any(axis=1)
        assert (out[untouched] == 0).all()
        # brute force over the token's chosen experts with the full weights
        for t in range(wl.T):
            acc = np.zeros(wl.H)
            for j in range(wl.top_k):
                e = int(ids[t, j])
                if lo <= e < lo + n:
                    act = orc.swiglu_rows(p, [t], [e])
                    acc += w[t, j] * orc.down_rows(p, [e], act)[0]
            np.testing.assert_allclose(out[t], acc, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(total, ref, rtol=1e-12, atol=1e-13)
    same, *_ = orc.forward(orc.problem_from_inputs(full.local_share(0, wl.E)))
    assert np.array_equal(same, ref)


def test_combine_skips_pairs_without_a_row():
    rng = np.random.default_rng(2)
    T, k, H = 5, 3, 4
    w = rng.normal(size=(T, k))
    y = rng.normal(size=(T * k, H))
    inv = rng.permutation(T * k).astype(np.int32)
    dropped = np.array([1, 4, 5, 13])
    inv_d = inv.copy(); inv_d[dropped] = -1
    w_zero = w.copy().reshape(-1); w_zero[dropped] = 0.0
    np.testing.assert_allclose(orc.combine(w, inv_d, y), orc.combine(w_zero.reshape(T, k), inv, y), rtol=0, atol=0)


# ---------------------------------------------------------------- activation quantisation on the path


def _lib_e4m3_codes(v32: torch.Tensor) -> np.ndarray:
    """Library conversion (clamped to the finite range first) -> code bytes."""
    return v32.clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def test_e4m3_encode_matches_library_cast_including_ties_and_saturation():
    g = torch.Generator().manual_seed(20)
    pos = np.array([orc.e4m3_to_f64(c) for c in range(0x7f)])                 # every finite magnitude, ascending
    mid = (pos[:-1] + pos[1:]) / 2                                              # exact ties (representable in binary32)
    vals = np.concatenate([pos, mid, np.nextafter(mid.astype(np.float32), np.float32(0)),
                           np.nextafter(mid.astype(np.float32), np.float32(1e9)),
                           [448.0, 449.0, 464.0, 1e4, 3e38, 1e-9, 2.0 ** -10, 2.0 ** -9 * 0.999],
                           (torch.randn(4000, generator=g) * 60).numpy(),
                           (torch.randn(2000, generator=g) * 0.02).numpy()]).astype(np.float32)
    vals = np.concatenate([vals, -vals])
    mine = np.array([orc.f32_to_e4m3(float(v)) for v in vals], dtype=np.uint8)
    lib = _lib_e4m3_codes(torch.from_numpy(vals))
    zero = (mine & 0x7f) == 0                                                   # +0 / -0 carry the sign of the input
    assert np.array_equal(mine & 0x7f, lib & 0x7f)
    assert np.array_equal(mine[~zero], lib[~zero])
    # ties go to the even mantissa, beyond 448 saturates, decode(encode(code value)) is the identity
    assert orc.f32_to_e4m3(float(mid[8])) % 2 == 0 and orc.f32_to_e4m3(1e30) == 0x7e
    assert all(orc.f32_to_e4m3(float(pos[c])) == c for c in range(0x7f))


def test_quantize_rows_matches_library_division_and_cast():
    g = torch.Generator().manual_seed(21)
    x = (torch.randn(5, 384, generator=g) * torch.tensor([1e-3, 1.0, 30.0]).repeat_interleave(128)).bfloat16()
    x[3, 128:256] = 0                                                           # an all-zero block
    q, s = orc.quantize_rows_1x128(x)
    b = x.float().reshape(5, 3, 128)
    amax = b.abs().amax(-1)
    s_lib = torch.where(amax > 0, amax / 448.0, torch.ones_like(amax))          # binary32 division
    q_lib = _lib_e4m3_codes(b / s_lib[..., None]).reshape(5, 384)
    assert np.array_equal(s.view(np.uint32), s_lib.numpy().view(np.uint32))
    zero = (q & 0x7f) == 0
    assert np.array_equal(q & 0x7f, q_lib & 0x7f) and np.array_equal(q[~zero], q_lib[~zero])
    assert (s[3, 1] == 1.0) and (q[3, 128:256] & 0x7f == 0).all()
    # every block's largest magnitude lands on the largest code, with its sign
    xf = x.float().numpy().reshape(5, 3, 128)
    qb = q.reshape(5, 3, 128)
    for r in range(5):
        for blk in range(3):
            if (r, blk) == (3, 1):
                continue
            j = int(np.abs(xf[r, blk]).argmax())
            assert qb[r, blk, j] == (0x7e | (0x80 if xf[r, blk, j] < 0 else 0))


def test_quantize_rows_is_exact_on_representable_blocks_and_bounded_elsewhere():
    g = torch.Generator().manual_seed(22)
    codes = torch.randint(0, 0x7f, (4, 256), generator=g).to(torch.uint8)
    codes[:, 7] = 0x7e
    codes[:, 128 + 9] = 0x7e                                                    # amax of each block = 448 * 2^-5
    sign = torch.randint(0, 2, (4, 256), generator=g).to(torch.uint8) << 7
    val = (codes | sign).view(torch.float8_e4m3fn).float() * 2.0 ** -5          # exact in bf16 (4 significant bits)
    q, s = orc.quantize_rows_1x128(val.bfloat16())
    assert (s == 2.0 ** -5).all()
    deq = np.array([orc.e4m3_to_f64(int(c)) for c in q.reshape(-1)]).reshape(4, 256) * 2.0 ** -5
    assert np.array_equal(deq, val.double().numpy())
    # generic values: relative error of one e4m3 rounding, plus half a subnormal step near zero
    x = (torch.randn(6, 512, generator=g) * 3).bfloat16()
    q, s = orc.quantize_rows_1x128(x)
    deq = np.array([orc.e4m3_to_f64(int(c)) for c in q.reshape(-1)]).reshape(6, 512) * np.repeat(s.astype(np.float64), 128, axis=1)
    xv = x.double().numpy()
    assert (np.abs(deq - xv) <= np.abs(xv) * 2.0 ** -4 + np.repeat(s, 128, axis=1) * 2.0 ** -10).all()
    # negating the input flips exactly the sign bits
    qn, sn = orc.quantize_rows_1x128(-x)
    assert np.array_equal(sn, s) and np.array_equal(qn ^ 0x80, q)


def test_quantize_on_the_path_routes_on_bf16_and_feeds_quantised_rows_to_the_experts():
    wl = _wl(T=6, H=256, I=128, E=4, top_k=2, fp8=True, quantize_x=True, scoring="sigmoid")
    inp = syn.make_inputs(wl, seed=23)
    assert inp.x.dtype == torch.bfloat16 and inp.x_scale is None
    p = orc.problem_from_inputs(inp)
    out, ids, w, _ = orc.forward(p)
    # router: float64 library matmul of the bf16 hidden states as they arrived
    z = orc.router_logits(p)
    np.testing.assert_allclose(z, _f64(inp.x) @ _f64(inp.router_w).T, rtol=1e-12, atol=1e-13)
    ids2, w2, _ = orc.route(p, z)
    assert np.array_equal(ids, ids2) and np.array_equal(w, w2)
    # experts: dense MLP on the dequantised library quantisation of x
    b = inp.x.float().reshape(wl.T, 2, 128)
    sc = b.abs().amax(-1) / 448.0
    xq = (b / sc[..., None]).clamp(-448, 448).to(torch.float8_e4m3fn).double() * sc[..., None].double()
    xq = xq.reshape(wl.T, wl.H).numpy()
    ref = np.zeros_like(out)
    for t in range(wl.T):
        for j in range(wl.top_k):
            e = int(ids[t, j])
            w1 = _f64(inp.w1[e]) * np.kron(_f64(inp.w1_scale[e]), np.ones((128, 128)))
            w2m = _f64(inp.w2[e]) * np.kron(_f64(inp.w2_scale[e]), np.ones((128, 128)))
            ref[t] += w[t, j] * _dense_mlp(xq[t:t + 1], w1, w2m, wl.I)[0]
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-13)
    # and it differs from routing on the quantised hidden states only through the logits
    p_q = orc.Problem(**{**{f: getattr(p, f) for f in ("T", "H", "I", "E", "top_k", "scoring", "renormalize", "n_group",
                                                        "topk_group", "group_score_topn", "routed_scale", "fp8", "x",
                                                        "x_scale", "router_w", "bias", "w1", "w1_scale", "w2", "w2_scale")}})
    assert not np.array_equal(orc.router_logits(p_q), z)
