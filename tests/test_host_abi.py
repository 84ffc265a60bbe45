"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol include/moe.h declares, and refuses bad problem statements before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_2602_19128_amd import binding as moe
from paper_2602_19128_amd import synthetic as syn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(moe.LIB_PATH):
        from paper_2602_19128_amd import build
        build.build(verbose=False)
    return moe.load()


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert set(names) == set(moe.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_nothing_but_the_c_abi_is_exported(lib):
    """The dynamic symbol table holds the declared entry points and nothing else of ours (the
    toolchain's own per-translation-unit markers aside)."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", moe.LIB_PATH], capture_output=True, text=True, check=True).stdout
    syms = [line.split()[-1] for line in out.splitlines() if line.strip()]
    ours = [s for s in syms if not s.startswith("__hip_")]
    assert sorted(ours) == sorted(moe.EXPORTS), sorted(set(ours) ^ set(moe.EXPORTS))


def test_config_struct_matches_header():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    body = re.search(r"typedef struct moe_config \{(.*?)\} moe_config;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        decl = decl.strip()
        if decl:
            fields += [f.strip() for f in decl.split(None, 1)[1].split(",")]
    assert fields == [f[0] for f in moe.MoEConfig._fields_]
    assert C.sizeof(moe.MoEConfig) == 4 * len(fields)
    assert moe.TILE_INTS * 4 == 32


def test_size_queries_and_tile_heights(lib):
    for name, wl in syn.WORKLOADS.items():
        if wl.fp8:
            continue
        cfg = moe.MoEConfig.from_workload(wl)
        rows = moe.moe_tile_rows(cfg)
        assert rows in (16, 32, 64, 128, 256)
        P = wl.T * wl.top_k
        assert moe.moe_max_tiles(cfg) >= -(-P // rows)
        ws = moe.moe_workspace_size(cfg)
        assert ws % 256 == 0 and ws >= P * wl.I * 2 + P * wl.H * 2
        # partial logits [splits, T, E] fp32; layers with at most 16 experts route in one kernel without scratch
        assert moe.moe_route_workspace_size(cfg) >= (wl.T * wl.E * 4 if wl.E > 16 else 1)


@pytest.mark.parametrize("change, code", [
    (dict(top_k=9), -1),                 # top_k > E
    (dict(H=100), -2),                   # H not a multiple of 64
    (dict(E=1024, top_k=2), -2),         # too many experts
    (dict(scoring=7), -1),
    (dict(n_group=3), -1),               # E % n_group != 0
    (dict(n_group=4, topk_group=5), -1),
    (dict(n_group=4, topk_group=1, group_score_topn=2, top_k=3), -1),   # top_k > eligible experts
    (dict(n_group=4, topk_group=2, group_score_topn=3), -1),            # topn > group size
    (dict(local_expert_offset=4, num_local_experts=5), -1),             # local range past the last expert
    (dict(local_expert_offset=2, num_local_experts=0), -1),             # offset without a local count
    (dict(num_local_experts=-1), -1),
    (dict(quantize_x=1), -1),                                           # quantise-on-the-path needs an fp8 layer
    (dict(quantize_x=2, dtype=1), -1),
    (dict(dtype=1, H=16384 + 128), -2),                                 # fp8: more than 128 scale blocks along H
    (dict(dtype=1, I=16384 + 128), -2),
])
def test_bad_problem_statements_are_refused(lib, change, code):
    cfg = moe.MoEConfig(T=16, H=256, I=128, E=8, top_k=2, scoring=0, renormalize=1, n_group=1,
                        topk_group=1, group_score_topn=2, dtype=0, routed_scale=1.0)
    for k, v in change.items():
        setattr(cfg, k, v)
    assert moe.moe_workspace_size(cfg) == 0
    one = C.c_void_p(256)                # never dereferenced: validation fails first
    rc = lib.moe_forward(C.byref(cfg), one, None, one, None, one, None, one, None, one, one, C.c_size_t(1 << 40), None)
    assert rc == code
    rc = lib.moe_route(C.byref(cfg), one, None, one, None, one, one, one, C.c_size_t(1 << 40), None)
    assert rc == code


def test_null_pointers_and_small_workspace_are_refused(lib):
    cfg = moe.MoEConfig.from_workload(syn.WORKLOADS["tiny"])
    one = C.c_void_p(256)
    rc = lib.moe_forward(C.byref(cfg), None, None, one, None, one, None, one, None, one, one, C.c_size_t(1 << 40), None)
    assert rc == -1
    rc = lib.moe_forward(C.byref(cfg), one, None, one, None, one, None, one, None, one, one, C.c_size_t(16), None)
    assert rc == -3
    rc = lib.moe_forward(C.byref(cfg), one, None, one, None, one, None, one, None, one, C.c_void_p(264),
                         C.c_size_t(1 << 40), None)
    assert rc == -1                      # workspace not 256-byte aligned
    assert lib.moe_error_string(-3).startswith(b"workspace too small")
    assert lib.moe_forward(None, one, None, one, None, one, None, one, None, one, one, C.c_size_t(0), None) == -1


def test_static_scratch_entry_refuses_large_problems_without_touching_the_device(lib):
    """moe_forward_static: a problem beyond the static scratch is refused on the host, before any
    device call (so this runs without a GPU); a bad problem statement gets its usual code."""
    one = C.c_void_p(256)
    big = moe.MoEConfig.from_workload(syn.WORKLOADS["dsv3_prefill"])
    assert moe.moe_workspace_size(big) > moe.STATIC_SCRATCH_BYTES
    assert lib.moe_forward_static(C.byref(big), one, None, one, one, one, None, one, None, one, None) == -3
    for name in ("tiny", "mixtral_prefill", "dsv3_decode"):
        assert moe.moe_workspace_size(moe.MoEConfig.from_workload(syn.WORKLOADS[name])) <= moe.STATIC_SCRATCH_BYTES
    bad = moe.MoEConfig(T=16, H=100, I=128, E=8, top_k=2)
    assert lib.moe_forward_static(C.byref(bad), one, None, one, None, one, None, one, None, one, None) == -2
    none = moe.MoEConfig(T=0, H=256, I=128, E=8, top_k=2, renormalize=1)
    assert lib.moe_forward_static(C.byref(none), None, None, None, None, None, None, None, None, None, None) == 0
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    assert int(re.search(r"MOE_STATIC_SCRATCH_BYTES = (\d+) << 20", text).group(1)) << 20 == moe.STATIC_SCRATCH_BYTES


def test_parity_cases_reach_the_kernel_shapes_the_benchmarks_run(lib):
    """The launch shape of both grouped GEMMs for every benchmark workload, and the small parity
    cases that are there to reach the same kernel instantiations whole-tile (tests/test_gpu_parity.py)."""
    import test_gpu_parity as tp
    plan = lambda wl, which: moe.moe_gemm_plan(moe.MoEConfig.from_workload(wl), which)
    shape = lambda wl, which: tuple(plan(wl, which)[k] for k in ("tile_rows", "wavefronts", "blocks_per_wavefront"))
    W = syn.WORKLOADS
    # benchmark workloads
    assert shape(W["mixtral_prefill"], "gateup") == (256, 8, 2) and shape(W["mixtral_prefill"], "down") == (256, 8, 2)
    # few experts, tall tiles, long K: the forward's down projection cuts K in halves; its workspace holds both partial sums
    assert plan(W["mixtral_prefill"], "down")["k_split"] == 2 and not plan(W["mixtral_prefill"], "down")["half_items"]
    mix = W["mixtral_prefill"]
    assert moe.moe_workspace_size(moe.MoEConfig.from_workload(mix)) >= mix.T * mix.top_k * mix.H * 8
    for name in W:
        assert plan(W[name], "gateup")["k_split"] == 1 and (name == "mixtral_prefill" or plan(W[name], "down")["k_split"] == 1)
    assert plan(W["mixtral_prefill"], "gateup")["whole_ranges"] and plan(W["mixtral_prefill"], "gateup")["half_items"]
    for name in ("dsv3_prefill", "dsv3_prefill_skew"):
        assert shape(W[name], "gateup") == (256, 8, 2) and shape(W[name], "down") == (256, 8, 2)
        assert not plan(W[name], "gateup")["whole_ranges"]
    assert shape(W["dsv3_decode"], "gateup") == (16, 8, 2) and shape(W["dsv3_decode"], "down") == (16, 8, 2)
    assert shape(W["fp8_prefill"], "gateup") == (64, 8, 2) and shape(W["fp8_prefill"], "down") == (64, 8, 4)
    assert shape(W["fp8_local32"], "gateup") == (256, 8, 2) and shape(W["fp8_local32"], "down") == (256, 8, 2)
    assert plan(W["fp8_local32"], "gateup")["whole_ranges"]
    # the small cases that stand in for them
    C_ = tp.CASES
    assert shape(C_["wide128_gateup_halves"], "gateup") == (128, 8, 2)
    g = plan(C_["wide128_gateup_halves"], "gateup")
    assert g["whole_ranges"] and g["half_items"] and (C_["wide128_gateup_halves"].I // g["columns"]) % 32 in range(1, 17)
    assert shape(C_["wide256_gateup_split"], "gateup") == (256, 8, 2)       # = Mixtral / DeepSeek-shaped gate/up
    assert shape(C_["wide256_down_split"], "down") == (256, 8, 2)           # = DeepSeek-shaped down
    for which in ("gateup", "down"):
        assert shape(C_["wide256_zigzag"], which) == (256, 8, 2) and not plan(C_["wide256_zigzag"], which)["whole_ranges"]
    assert shape(C_["ragged128"], "down")[1:] == (4, 2) and shape(C_["fp8_tall"], "down") == (256, 4, 2)    # narrow
    assert plan(C_["ragged128"], "down")["k_split"] == 1 and plan(C_["fp8_tall"], "down")["k_split"] == 1
    for name in ("down_k_halves", "wide256_gateup_split", "wide128_gateup_halves"):    # K in halves, 8 wavefronts
        assert plan(C_[name], "down")["k_split"] == 2 and shape(C_[name], "down")[1:] == (8, 2)
    assert shape(C_["low_tiles"], "down") == (32, 8, 4) and shape(C_["low_tiles_fp8"], "down") == (32, 8, 4)
    assert shape(C_["fp8_tall"], "gateup") == (256, 8, 2) and shape(C_["fp8_deep_h"], "gateup")[1:] == (8, 2)
    assert lib.moe_gemm_plan(C.byref(moe.MoEConfig.from_workload(W["tiny"])), 2, (C.c_int32 * 8)()) == -1


def test_single_launch_path_is_a_property_of_the_problem_statement(lib):
    """Which problems moe_forward runs as one launch once that is switched on (host logic only; the
    GPU tests compare the paths)."""
    mode = lambda name: moe.moe_single_launch_mode(moe.MoEConfig.from_workload(syn.WORKLOADS[name]))
    assert mode("tiny") == moe.SINGLE_LAUNCH_NONE                       # off by default
    try:
        moe.moe_single_launch(True)
        assert mode("tiny") == moe.SINGLE_LAUNCH_ALL
        for name in ("dsv3_decode", "mixtral_prefill", "dsv3_prefill", "fp8_prefill", "fp8_local32"):
            assert mode(name) == moe.SINGLE_LAUNCH_NONE
    finally:
        moe.moe_single_launch(False)
    bad = moe.MoEConfig(T=16, H=100, I=128, E=8, top_k=2)
    assert lib.moe_single_launch_mode(C.byref(bad)) == -2
    assert lib.moe_single_launch_timeouts(None) == -1


def test_quantise_on_the_path_sizes_and_argument_checks(lib):
    wl = syn.WORKLOADS["fp8_prefill"]
    cfg = moe.MoEConfig.from_workload(wl)
    cfg_q = moe.MoEConfig.from_workload(syn.WORKLOADS["fp8_prefill_qx"])
    assert cfg_q.quantize_x == 1 and cfg.quantize_x == 0
    # the workspace grows by the e4m3 copy of x and its scales
    extra = moe.moe_workspace_size(cfg_q) - moe.moe_workspace_size(cfg)
    assert wl.T * wl.H + wl.T * (wl.H // 128) * 4 <= extra <= wl.T * wl.H + wl.T * (wl.H // 128) * 4 + wl.T * wl.E * 64
    one = C.c_void_p(256)
    # x_scale may be missing when the layer makes it itself, the weight scales may not
    big = C.c_size_t(1 << 40)
    assert lib.moe_forward(C.byref(cfg), one, None, one, None, one, one, one, one, one, one, big, None) == -1
    assert lib.moe_forward(C.byref(cfg_q), one, None, one, None, one, None, one, one, one, one, big, None) == -1
    assert lib.moe_forward(C.byref(cfg_q), one, None, one, None, one, one, one, one, one, one, C.c_size_t(16), None) == -3
    # moe_quantize_act: H must be a multiple of 128, pointers present; zero tokens is a no-op
    bad = moe.MoEConfig(T=4, H=192, I=128, E=8, top_k=2, dtype=1)
    assert lib.moe_quantize_act(C.byref(bad), one, one, one, None) == -2
    ok = moe.MoEConfig(T=4, H=256, I=128, E=8, top_k=2, dtype=1)
    assert lib.moe_quantize_act(C.byref(ok), None, one, one, None) == -1
    assert lib.moe_quantize_act(C.byref(ok), one, one, None, None) == -1
    none = moe.MoEConfig(T=0, H=256, I=128, E=8, top_k=2, dtype=1)
    assert lib.moe_quantize_act(C.byref(none), None, None, None, None) == 0
    assert lib.moe_quantize_act(None, one, one, one, None) == -1


def test_binding_refuses_cpu_tensors(lib):
    import torch
    wl = syn.WORKLOADS["tiny"]
    inp = syn.make_inputs(wl, seed=0)
    cfg = moe.MoEConfig.from_workload(wl)
    with pytest.raises(moe.MoEError):
        moe.moe_combine(cfg, torch.zeros(cfg.P, wl.H, dtype=torch.bfloat16), torch.zeros(wl.T, wl.top_k),
                        torch.zeros(cfg.P, dtype=torch.int32))
