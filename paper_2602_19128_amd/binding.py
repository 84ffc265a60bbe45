"""ctypes front end of libmoe_gfx950.so (the C ABI declared in include/moe.h).

Argument marshalling only: every step of the layer runs in the HIP kernels.
PyTorch supplies device memory and the current stream; there is no fallback --
if the library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmoe_gfx950.so")

EXPORTS = [
    "moe_tile_rows", "moe_max_tiles", "moe_route_workspace_size", "moe_workspace_size",
    "moe_route", "moe_quantize_act", "moe_permute", "moe_grouped_gemm_swiglu", "moe_grouped_gemm_down",
    "moe_combine", "moe_forward", "moe_forward_marked", "moe_init", "moe_forward_static",
    "moe_single_launch", "moe_single_launch_mode", "moe_single_launch_timeouts", "moe_gemm_plan",
    "moe_error_string", "moe_last_hip_error",
]
STATIC_SCRATCH_BYTES = 64 << 20   # MOE_STATIC_SCRATCH_BYTES

TILE_INTS = 8            # int32 fields of one moe_tile record
SCHED_INTS = 16          # int32 entries of the schedule header moe_permute writes (MOE_SCHED_INTS)
WORK_RANGES = 8          # MOE_WORK_RANGES


class MoEError(RuntimeError):
    pass


class MoEConfig(C.Structure):
    """Mirror of `moe_config` in include/moe.h."""
    _fields_ = [
        ("T", C.c_int32), ("H", C.c_int32), ("I", C.c_int32), ("E", C.c_int32), ("top_k", C.c_int32),
        ("scoring", C.c_int32), ("renormalize", C.c_int32), ("n_group", C.c_int32),
        ("topk_group", C.c_int32), ("group_score_topn", C.c_int32), ("dtype", C.c_int32),
        ("routed_scale", C.c_float),
        ("local_expert_offset", C.c_int32), ("num_local_experts", C.c_int32),
        ("quantize_x", C.c_int32),
    ]

    @classmethod
    def from_workload(cls, wl) -> "MoEConfig":
        return cls(wl.T, wl.H, wl.I, wl.E, wl.top_k, {"softmax": 0, "sigmoid": 1}[wl.scoring], 1,
                   wl.n_group, wl.topk_group, wl.group_score_topn, 1 if wl.fp8 else 0,
                   float(wl.routed_scale), wl.local_offset, wl.local_experts,
                   1 if getattr(wl, "quantize_x", False) else 0)

    @property
    def P(self) -> int:
        return self.T * self.top_k

    @property
    def EL(self) -> int:
        """Experts whose weights the call holds (all E unless local-expert mode is on)."""
        return self.num_local_experts if self.num_local_experts > 0 else self.E


_lib = None


def load():
    """Load the built library (build it first with `python -m paper_2602_19128_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MoEError(f"{LIB_PATH} is not built; run `python -m paper_2602_19128_amd.build`")
    lib = C.CDLL(LIB_PATH)
    cfgp, vp, i32p, f32p = C.POINTER(MoEConfig), C.c_void_p, C.c_void_p, C.c_void_p
    lib.moe_tile_rows.restype = C.c_int32
    lib.moe_tile_rows.argtypes = [cfgp]
    lib.moe_max_tiles.restype = C.c_int32
    lib.moe_max_tiles.argtypes = [cfgp]
    lib.moe_route_workspace_size.restype = C.c_size_t
    lib.moe_route_workspace_size.argtypes = [cfgp]
    lib.moe_workspace_size.restype = C.c_size_t
    lib.moe_workspace_size.argtypes = [cfgp]
    lib.moe_route.restype = C.c_int
    lib.moe_route.argtypes = [cfgp, vp, f32p, f32p, f32p, i32p, f32p, vp, C.c_size_t, vp]
    lib.moe_quantize_act.restype = C.c_int
    lib.moe_quantize_act.argtypes = [cfgp, vp, vp, f32p, vp]
    lib.moe_permute.restype = C.c_int
    lib.moe_permute.argtypes = [cfgp, i32p, i32p, i32p, i32p, vp, i32p, vp]
    lib.moe_grouped_gemm_swiglu.restype = C.c_int
    lib.moe_grouped_gemm_swiglu.argtypes = [cfgp, vp, f32p, vp, f32p, i32p, vp, i32p, vp, f32p, vp]
    lib.moe_grouped_gemm_down.restype = C.c_int
    lib.moe_grouped_gemm_down.argtypes = [cfgp, vp, f32p, vp, f32p, vp, i32p, vp, vp]
    lib.moe_combine.restype = C.c_int
    lib.moe_combine.argtypes = [cfgp, vp, f32p, i32p, vp, vp]
    lib.moe_forward.restype = C.c_int
    lib.moe_forward.argtypes = [cfgp, vp, f32p, f32p, f32p, vp, f32p, vp, f32p, vp, vp, C.c_size_t, vp]
    lib.moe_forward_marked.restype = C.c_int
    lib.moe_forward_marked.argtypes = lib.moe_forward.argtypes + [C.POINTER(C.c_void_p)]
    lib.moe_init.restype = C.c_int
    lib.moe_init.argtypes = []
    lib.moe_forward_static.restype = C.c_int
    lib.moe_forward_static.argtypes = [cfgp, vp, f32p, f32p, f32p, vp, f32p, vp, f32p, vp, vp]
    lib.moe_gemm_plan.restype = C.c_int
    lib.moe_gemm_plan.argtypes = [cfgp, C.c_int, C.POINTER(C.c_int32)]
    lib.moe_single_launch.restype = None
    lib.moe_single_launch.argtypes = [C.c_int]
    lib.moe_single_launch_mode.restype = C.c_int
    lib.moe_single_launch_mode.argtypes = [cfgp]
    lib.moe_single_launch_timeouts.restype = C.c_int
    lib.moe_single_launch_timeouts.argtypes = [C.POINTER(C.c_uint32)]
    lib.moe_error_string.restype = C.c_char_p
    lib.moe_error_string.argtypes = [C.c_int]
    lib.moe_last_hip_error.restype = C.c_int
    _lib = lib
    return lib


def _check(rc: int, what: str):
    if rc != 0:
        lib = load()
        msg = lib.moe_error_string(rc).decode()
        raise MoEError(f"{what}: {msg} (code {rc}, hip error {lib.moe_last_hip_error()})")


def _p(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise MoEError("tensors handed to the MoE library must live on the GPU")
    if not t.is_contiguous():
        raise MoEError("tensors handed to the MoE library must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _payload(cfg: MoEConfig):
    return torch.float8_e4m3fn if cfg.dtype == 1 else torch.bfloat16


def _x_arrives_as(cfg: MoEConfig):
    """dtype of the hidden states handed to moe_route / moe_forward (bf16 when the layer quantises them itself)."""
    return torch.bfloat16 if cfg.quantize_x else _payload(cfg)


def _expect(t, shape, dtype, name):
    if t is None:
        return
    if tuple(t.shape) != tuple(shape) or t.dtype != dtype:
        raise MoEError(f"{name}: expected {tuple(shape)} {dtype}, got {tuple(t.shape)} {t.dtype}")


# ---- size queries ------------------------------------------------------------

def moe_tile_rows(cfg: MoEConfig) -> int:
    return int(load().moe_tile_rows(C.byref(cfg)))


def moe_max_tiles(cfg: MoEConfig) -> int:
    return int(load().moe_max_tiles(C.byref(cfg)))


def moe_route_workspace_size(cfg: MoEConfig) -> int:
    return int(load().moe_route_workspace_size(C.byref(cfg)))


def moe_workspace_size(cfg: MoEConfig) -> int:
    return int(load().moe_workspace_size(C.byref(cfg)))


def moe_gemm_plan(cfg: MoEConfig, which: str) -> dict:
    """Launch shape of the "gateup" or "down" grouped GEMM for this problem (see include/moe.h)."""
    plan = (C.c_int32 * 8)()
    _check(load().moe_gemm_plan(C.byref(cfg), {"gateup": 0, "down": 1}[which], plan), "moe_gemm_plan")
    return {"tile_rows": plan[0], "wavefronts": plan[1], "blocks_per_wavefront": plan[2], "columns": plan[3],
            "whole_ranges": bool(plan[4]), "half_items": bool(plan[5]), "k_split": plan[6]}


def _bytes(n: int, device) -> torch.Tensor:
    return torch.empty((max(int(n), 256),), dtype=torch.uint8, device=device)


# ---- the calls ------------------------------------------------------------------

def moe_route(cfg, x, x_scale, router_w, bias, ids_out=None, w_out=None, workspace=None):
    dev = x.device
    _expect(x, (cfg.T, cfg.H), _x_arrives_as(cfg), "x")
    _expect(router_w, (cfg.E, cfg.H), torch.float32, "router_w")
    _expect(bias, (cfg.E,), torch.float32, "bias")
    _expect(x_scale, (cfg.T, cfg.H // 128), torch.float32, "x_scale")
    ids_out = torch.empty((cfg.T, cfg.top_k), dtype=torch.int32, device=dev) if ids_out is None else ids_out
    w_out = torch.empty((cfg.T, cfg.top_k), dtype=torch.float32, device=dev) if w_out is None else w_out
    workspace = _bytes(moe_route_workspace_size(cfg), dev) if workspace is None else workspace
    rc = load().moe_route(C.byref(cfg), _p(x), _p(x_scale), _p(router_w), _p(bias), _p(ids_out), _p(w_out),
                          _p(workspace), C.c_size_t(workspace.numel()), _stream())
    _check(rc, "moe_route")
    return ids_out, w_out


def moe_quantize_act(cfg, x):
    """bf16 [T,H] -> (e4m3 payload [T,H], fp32 scales [T,H/128])."""
    _expect(x, (cfg.T, cfg.H), torch.bfloat16, "x")
    xq = torch.empty((cfg.T, cfg.H), dtype=torch.float8_e4m3fn, device=x.device)
    xs = torch.empty((cfg.T, cfg.H // 128), dtype=torch.float32, device=x.device)
    rc = load().moe_quantize_act(C.byref(cfg), _p(x), _p(xq), _p(xs), _stream())
    _check(rc, "moe_quantize_act")
    return xq, xs


def moe_permute(cfg, ids):
    dev = ids.device
    _expect(ids, (cfg.T, cfg.top_k), torch.int32, "ids")
    P = cfg.P
    offsets = torch.empty((cfg.EL + 1,), dtype=torch.int32, device=dev)
    sorted_pair = torch.empty((max(P, 1),), dtype=torch.int32, device=dev)
    inv = torch.empty((max(P, 1),), dtype=torch.int32, device=dev)
    tiles = torch.zeros((max(moe_max_tiles(cfg), 1), TILE_INTS), dtype=torch.int32, device=dev)
    sched = torch.zeros((SCHED_INTS,), dtype=torch.int32, device=dev)
    rc = load().moe_permute(C.byref(cfg), _p(ids), _p(offsets), _p(sorted_pair), _p(inv), _p(tiles), _p(sched),
                            _stream())
    _check(rc, "moe_permute")
    return offsets, sorted_pair[:P], inv[:P], tiles, sched


def moe_grouped_gemm_swiglu(cfg, x, x_scale, w1, w1_scale, sorted_pair, tiles, sched):
    dev = x.device
    _expect(x, (cfg.T, cfg.H), _payload(cfg), "x")
    _expect(w1, (cfg.EL, 2 * cfg.I, cfg.H), _payload(cfg), "w1")
    act = torch.empty((cfg.P, cfg.I), dtype=_payload(cfg), device=dev)
    act_scale = torch.empty((cfg.P, cfg.I // 128), dtype=torch.float32, device=dev) if cfg.dtype == 1 else None
    rc = load().moe_grouped_gemm_swiglu(C.byref(cfg), _p(x), _p(x_scale), _p(w1), _p(w1_scale), _p(sorted_pair),
                                        _p(tiles), _p(sched), _p(act), _p(act_scale), _stream())
    _check(rc, "moe_grouped_gemm_swiglu")
    return act, act_scale


def moe_grouped_gemm_down(cfg, act, act_scale, w2, w2_scale, tiles, sched):
    dev = act.device
    _expect(act, (cfg.P, cfg.I), _payload(cfg), "act")
    _expect(w2, (cfg.EL, cfg.H, cfg.I), _payload(cfg), "w2")
    y = torch.empty((cfg.P, cfg.H), dtype=torch.bfloat16, device=dev)
    rc = load().moe_grouped_gemm_down(C.byref(cfg), _p(act), _p(act_scale), _p(w2), _p(w2_scale), _p(tiles),
                                      _p(sched), _p(y), _stream())
    _check(rc, "moe_grouped_gemm_down")
    return y


def moe_combine(cfg, y, w, inv):
    _expect(y, (cfg.P, cfg.H), torch.bfloat16, "y")
    _expect(w, (cfg.T, cfg.top_k), torch.float32, "w")
    out = torch.empty((cfg.T, cfg.H), dtype=torch.bfloat16, device=y.device)
    rc = load().moe_combine(C.byref(cfg), _p(y), _p(w), _p(inv), _p(out), _stream())
    _check(rc, "moe_combine")
    return out


FORWARD_EVENTS = 6
STEP_NAMES = ("route", "permute", "gemm_swiglu", "gemm_down", "combine")


def moe_forward(cfg, x, x_scale, router_w, bias, w1, w1_scale, w2, w2_scale, out=None, workspace=None,
                events=None):
    """`events`: optional ctypes array of FORWARD_EVENTS hipEvent_t handles (see moe_forward_marked)."""
    dev = x.device
    _expect(x, (cfg.T, cfg.H), _x_arrives_as(cfg), "x")
    _expect(router_w, (cfg.E, cfg.H), torch.float32, "router_w")
    _expect(w1, (cfg.EL, 2 * cfg.I, cfg.H), _payload(cfg), "w1")
    _expect(w2, (cfg.EL, cfg.H, cfg.I), _payload(cfg), "w2")
    out = torch.empty((cfg.T, cfg.H), dtype=torch.bfloat16, device=dev) if out is None else out
    workspace = _bytes(moe_workspace_size(cfg), dev) if workspace is None else workspace
    args = (C.byref(cfg), _p(x), _p(x_scale), _p(router_w), _p(bias), _p(w1), _p(w1_scale), _p(w2),
            _p(w2_scale), _p(out), _p(workspace), C.c_size_t(workspace.numel()), _stream())
    if events is None:
        rc = load().moe_forward(*args)
    else:
        rc = load().moe_forward_marked(*args, events)
    _check(rc, "moe_forward")
    return out


SINGLE_LAUNCH_NONE, SINGLE_LAUNCH_ALL = 0, 1


def moe_single_launch(enable: bool):
    load().moe_single_launch(1 if enable else 0)


def moe_single_launch_mode(cfg) -> int:
    rc = int(load().moe_single_launch_mode(C.byref(cfg)))
    if rc < 0:
        _check(rc, "moe_single_launch_mode")
    return rc


def moe_single_launch_timeouts() -> int:
    n = C.c_uint32(0)
    _check(load().moe_single_launch_timeouts(C.byref(n)), "moe_single_launch_timeouts")
    return int(n.value)


def moe_init():
    _check(load().moe_init(), "moe_init")


def moe_forward_static(cfg, x, x_scale, router_w, bias, w1, w1_scale, w2, w2_scale, out):
    """moe_forward on the library's own static scratch: `out` is the caller's, nothing is allocated."""
    _expect(x, (cfg.T, cfg.H), _x_arrives_as(cfg), "x")
    _expect(out, (cfg.T, cfg.H), torch.bfloat16, "out")
    rc = load().moe_forward_static(C.byref(cfg), _p(x), _p(x_scale), _p(router_w), _p(bias), _p(w1), _p(w1_scale),
                                   _p(w2), _p(w2_scale), _p(out), _stream())
    _check(rc, "moe_forward_static")
    return out


class PreparedForward:
    """moe_forward with its arguments marshalled once (for loops where the marshalling would be most
    of the host time of a call); the stream is the one current when it was prepared."""

    def __init__(self, cfg, x, x_scale, router_w, bias, w1, w1_scale, w2, w2_scale, out, workspace):
        _expect(x, (cfg.T, cfg.H), _x_arrives_as(cfg), "x")
        _expect(out, (cfg.T, cfg.H), torch.bfloat16, "out")
        self._keep = (cfg, x, x_scale, router_w, bias, w1, w1_scale, w2, w2_scale, out, workspace)
        self._fn = load().moe_forward
        self._args = (C.byref(cfg), _p(x), _p(x_scale), _p(router_w), _p(bias), _p(w1), _p(w1_scale), _p(w2),
                      _p(w2_scale), _p(out), _p(workspace), C.c_size_t(workspace.numel()), _stream())

    def __call__(self):
        rc = self._fn(*self._args)
        if rc != 0:
            _check(rc, "moe_forward")


def forward_inputs(inp, out=None, workspace=None):
    """moe_forward on a synthetic.MoEInputs bundle that already lives on the GPU."""
    cfg = MoEConfig.from_workload(inp.wl)
    return moe_forward(cfg, inp.x, inp.x_scale, inp.router_w, inp.bias, inp.w1, inp.w1_scale, inp.w2,
                       inp.w2_scale, out=out, workspace=workspace)
