"""Shared comparison helpers of the GPU parity tests (GPU library vs CPU oracle)."""
from __future__ import annotations

import numpy as np
import torch

from oracle import moe_oracle as orc

# Tolerances of the layer output (bf16 path / fp8 path), relative to max|ref| and as
# mean relative error sum|err| / sum|ref|.
TOL_MAX = {False: 2e-2, True: 6e-2}
TOL_MEAN = {False: 5e-3, True: 3e-2}
TIE_MARGIN = 1e-6           # routing decisions closer than this may legitimately differ


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def err_stats(got: np.ndarray, ref: np.ndarray):
    err = np.abs(got - ref)
    peak = float(np.abs(ref).max()) if ref.size else 0.0
    max_rel = float(err.max() / peak) if ref.size and peak > 0 else 0.0
    mean_rel = float(err.sum() / np.abs(ref).sum()) if ref.size and np.abs(ref).sum() > 0 else 0.0
    return max_rel, mean_rel


def compare_routing(ids_gpu, w_gpu, ids_ref, w_ref, margin, routed_scale=1.0, n_experts=None, key_ref=None):
    """Expert ids must match the oracle bit for bit, in order.  Two exceptions, both
    counted and returned: a token whose decision margin in the oracle is below
    TIE_MARGIN may pick a different expert set, and two chosen experts whose keys
    are that close may swap slots (same set, weights equal per expert).
    Weights must agree to fp32 accuracy.
    Returns (tokens_with_other_set, tokens_with_swapped_slots, same_set_mask)."""
    ids_gpu = ids_gpu.cpu().numpy()
    w_gpu = w_gpu.cpu().numpy().astype(np.float64)
    T, k = ids_ref.shape
    atol = 2e-6 * max(1.0, routed_scale)
    if n_experts is not None:
        assert ((ids_gpu >= 0) & (ids_gpu < n_experts)).all(), "expert id out of range"
    exact = (ids_gpu == ids_ref).all(axis=1)
    same_set = np.array([sorted(ids_gpu[t]) == sorted(ids_ref[t]) for t in range(T)], dtype=bool)
    for t in range(T):
        assert len(set(ids_gpu[t].tolist())) == k, f"token {t}: experts not distinct"
    bad = ~same_set & (margin >= TIE_MARGIN)
    if bad.any():
        t = int(np.nonzero(bad)[0][0])
        raise AssertionError(f"{int(bad.sum())} tokens routed differently with margin >= {TIE_MARGIN}: "
                             f"first t={t} gpu={ids_gpu[t]} ref={ids_ref[t]} margin={margin[t]}")
    for t in np.nonzero(same_set & ~exact)[0]:
        slot = {int(e): j for j, e in enumerate(ids_ref[t])}
        perm = [slot[int(e)] for e in ids_gpu[t]]
        np.testing.assert_allclose(w_gpu[t], w_ref[t][perm], rtol=2e-5, atol=atol)
        if key_ref is not None:           # the experts that changed slot must have near-equal keys
            moved = [int(ids_ref[t][j]) for j in range(k) if perm[j] != j]
            spread = key_ref[t][moved].max() - key_ref[t][moved].min()
            assert spread < 2 * TIE_MARGIN, f"token {t}: slots swapped between unequal experts"
    if exact.any():
        np.testing.assert_allclose(w_gpu[exact], w_ref[exact], rtol=2e-5, atol=atol)
    return int((~same_set).sum()), int((same_set & ~exact).sum()), same_set


def check_tiles(tiles, sched, offsets_ref, tile_rows):
    """The tile list covers every non-empty expert segment exactly once, cut as documented, and is a
    valid schedule: an expert's records are consecutive and lie in one work range, experts are dealt
    to the eight ranges in snake order of their row count (largest first, equal counts by index), and
    every range lists its experts in that order."""
    hdr = sched.cpu().numpy()
    n = int(hdr[0])
    rec = tiles.cpu().numpy()[:n]
    E = len(offsets_ref) - 1
    rows_of = np.diff(np.asarray(offsets_ref, dtype=np.int64))
    want = {}                              # expert -> list of (row0, rows)
    for e in range(E):
        lo, hi = int(offsets_ref[e]), int(offsets_ref[e + 1])
        cnt = -(-(hi - lo) // tile_rows)
        part = -(-(-(-(hi - lo) // cnt) if cnt else 0) // 16) * 16    # equal parts, whole 16-row blocks
        cuts = []
        for i in range(cnt):
            r0 = lo + i * part
            assert hi - r0 > 0
            cuts.append((r0, min(part, hi - r0)))
        if cuts:
            want[e] = cuts
    assert n == sum(len(c) for c in want.values()), f"{n} tiles, expected {sum(len(c) for c in want.values())}"
    # the ranges tile [0, n) in order
    starts = hdr[1:10].astype(np.int64)
    assert starts[0] == 0 and starts[8] == n and (np.diff(starts) >= 0).all(), f"bad work ranges {starts}"
    # snake dealing of the experts ranked by rows (stable: equal rows keep index order)
    order = sorted(want, key=lambda e: (-rows_of[e], e))
    expect = [[] for _ in range(8)]
    for rank, e in enumerate(order):
        rnd, pos = divmod(rank, 8)
        expect[7 - pos if rnd % 2 else pos].append(e)
    at = 0
    for r in range(8):
        assert at == starts[r], f"range {r} starts at {starts[r]}, expected {at}"
        for e in expect[r]:
            cuts = want[e]
            got = rec[at:at + len(cuts)]
            assert (got[:, 0] == e).all() and (got[:, 3] == at).all() and (got[:, 4] == len(cuts)).all(), \
                f"records of expert {e} at {at}: {got[:, :5]}"
            assert [tuple(x) for x in got[:, 1:3]] == cuts, f"expert {e}: cuts {got[:, 1:3]} expected {cuts}"
            at += len(cuts)
    assert at == n
    return n


def choice_keys(p, z):
    """Choice key of every expert from the oracle's logits (only used to judge slot swaps)."""
    if p.scoring == "softmax":
        s = np.exp(z - z.max(axis=1, keepdims=True))
        s /= s.sum(axis=1, keepdims=True)
    else:
        s = 1.0 / (1.0 + np.exp(-z))
    if p.bias is not None:
        s = s + p._b.astype(np.float64)[None, :]
    return s


def local_permute(ids, E, local_offset=0, local_count=0):
    """Oracle sort-scatter of the pairs whose expert is held locally (all of them unless
    local-expert mode is on): offsets [EL+1], sorted_pair [kept], inv [P] with -1 for the
    pairs that were dropped, and the number of kept pairs."""
    flat = np.asarray(ids, dtype=np.int32).reshape(-1)
    if local_count <= 0:
        local_offset, local_count = 0, E
    keep = (flat >= local_offset) & (flat < local_offset + local_count)
    kept_pairs = np.nonzero(keep)[0].astype(np.int32)
    off, sp, inv_k = orc.permute((flat[keep] - local_offset).reshape(-1, 1), local_count)
    inv = np.full(flat.shape, -1, dtype=np.int32)
    inv[keep] = inv_k
    return off, kept_pairs[sp], inv, int(keep.sum())


def oracle_all(inp):
    """Oracle routing for every token + the permutation of that routing."""
    p = orc.problem_from_inputs(inp)
    z = orc.router_logits(p)
    ids, w, margin = orc.route(p, z)
    offsets, sorted_pair, inv, _ = local_permute(ids, p.E, p.local_offset, p.local_count)
    return p, ids, w, margin, offsets, sorted_pair, inv, choice_keys(p, z)
