"""TEST INFRASTRUCTURE -- ctypes front end of the CPU oracle in moe_oracle.c.

Only argument marshalling lives here; every number is produced by the C file.
Used by tests/, by the smoke check and by the benchmark's CPU-baseline leg;
the GPU library never imports or links it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")


def build(force: bool = False) -> str:
    """Compile moe_oracle.c with gcc (OpenMP over independent outputs only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Problem(C.Structure):
    _fields_ = [
        ("T", C.c_int32), ("H", C.c_int32), ("I", C.c_int32), ("E", C.c_int32), ("top_k", C.c_int32),
        ("scoring", C.c_int32), ("renormalize", C.c_int32), ("n_group", C.c_int32),
        ("topk_group", C.c_int32), ("group_score_topn", C.c_int32), ("dtype", C.c_int32),
        ("routed_scale", C.c_float),
        ("x", C.c_void_p), ("x_scale", C.c_void_p), ("router_w", C.c_void_p), ("bias", C.c_void_p),
        ("w1", C.c_void_p), ("w1_scale", C.c_void_p), ("w2", C.c_void_p), ("w2_scale", C.c_void_p),
        ("local_offset", C.c_int32), ("local_count", C.c_int32),
        ("x_bf16", C.c_void_p),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_bf16_to_f64.restype = C.c_double
        _lib.oracle_bf16_to_f64.argtypes = [C.c_uint16]
        _lib.oracle_e4m3_to_f64.restype = C.c_double
        _lib.oracle_e4m3_to_f64.argtypes = [C.c_uint8]
        _lib.oracle_f32_to_e4m3.restype = C.c_uint8
        _lib.oracle_f32_to_e4m3.argtypes = [C.c_float]
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _np(a, dtype=None):
    """torch tensor / array -> contiguous numpy array sharing no GPU state."""
    if a is None:
        return None
    if hasattr(a, "detach"):          # torch tensor
        import torch
        a = a.detach().cpu().contiguous()
        if a.dtype == torch.bfloat16:
            a = a.view(torch.int16).numpy().view(np.uint16)
        elif a.dtype == torch.float8_e4m3fn:
            a = a.view(torch.uint8).numpy()
        else:
            a = a.numpy()
    a = np.ascontiguousarray(a)
    if dtype is not None and a.dtype != dtype:
        a = a.astype(dtype)
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class Problem:
    """Shapes + routing rule + host arrays of one layer call."""
    T: int
    H: int
    I: int
    E: int
    top_k: int
    scoring: str = "softmax"          # "softmax" | "sigmoid"
    renormalize: bool = True
    n_group: int = 1
    topk_group: int = 1
    group_score_topn: int = 2
    routed_scale: float = 1.0
    fp8: bool = False
    x: Optional[object] = None
    x_scale: Optional[object] = None
    router_w: Optional[object] = None
    bias: Optional[object] = None
    w1: Optional[object] = None
    w1_scale: Optional[object] = None
    w2: Optional[object] = None
    w2_scale: Optional[object] = None
    local_offset: int = 0             # local-expert mode: weights hold experts [offset, offset+count)
    local_count: int = 0              # 0 = all E experts
    x_bf16: Optional[object] = None   # quantise-on-the-path mode: the bf16 hidden states the layer received
                                      # (x / x_scale then hold quantize_rows_1x128(x_bf16))

    @property
    def EL(self) -> int:
        return self.local_count if self.local_count > 0 else self.E

    def __post_init__(self):
        pay = np.uint8 if self.fp8 else np.uint16
        self._x = _np(self.x, pay)
        self._xs = _np(self.x_scale, np.float32)
        self._rw = _np(self.router_w, np.float32)
        self._b = _np(self.bias, np.float32)
        self._w1 = _np(self.w1, pay)
        self._w1s = _np(self.w1_scale, np.float32)
        self._w2 = _np(self.w2, pay)
        self._w2s = _np(self.w2_scale, np.float32)
        self._xb = _np(self.x_bf16, np.uint16)
        if self._xb is not None:
            assert self.fp8 and self._xb.size == self.T * self.H
        if self._x is not None:
            assert self._x.size == self.T * self.H
        if self._rw is not None:
            assert self._rw.size == self.E * self.H
        if self._w1 is not None:
            assert self._w1.size == self.EL * 2 * self.I * self.H
        if self._w2 is not None:
            assert self._w2.size == self.EL * self.H * self.I
        assert 0 <= self.local_offset and self.local_offset + self.local_count <= self.E
        if self.fp8:
            assert self.H % 128 == 0 and self.I % 128 == 0
        self._c = _Problem(
            self.T, self.H, self.I, self.E, self.top_k,
            {"softmax": 0, "sigmoid": 1}[self.scoring], int(self.renormalize), self.n_group,
            self.topk_group, self.group_score_topn, int(self.fp8), float(self.routed_scale),
            _ptr(self._x), _ptr(self._xs), _ptr(self._rw), _ptr(self._b),
            _ptr(self._w1), _ptr(self._w1s), _ptr(self._w2), _ptr(self._w2s),
            self.local_offset, self.local_count, _ptr(self._xb))


def problem_from_inputs(inp) -> Problem:
    """Build a Problem from an object with `.wl` (shape/routing fields) and tensors."""
    wl = inp.wl
    x, x_scale, x_bf16 = inp.x, inp.x_scale, None
    if getattr(wl, "quantize_x", False):        # the layer quantises its bf16 hidden states itself
        x_bf16 = inp.x
        x, x_scale = quantize_rows_1x128(inp.x)
    return Problem(T=wl.T, H=wl.H, I=wl.I, E=wl.E, top_k=wl.top_k, scoring=wl.scoring,
                   renormalize=True, n_group=wl.n_group, topk_group=wl.topk_group,
                   group_score_topn=wl.group_score_topn, routed_scale=wl.routed_scale, fp8=wl.fp8,
                   x=x, x_scale=x_scale, x_bf16=x_bf16, router_w=inp.router_w, bias=inp.bias,
                   w1=inp.w1, w1_scale=inp.w1_scale, w2=inp.w2, w2_scale=inp.w2_scale,
                   local_offset=getattr(wl, "local_offset", 0), local_count=getattr(wl, "local_experts", 0))


def quantize_rows_1x128(x_bf16):
    """bf16 rows [R,K] -> (e4m3 codes [R,K] uint8, scales [R,K/128] float32)."""
    x = _np(x_bf16, np.uint16)
    assert x.ndim == 2 and x.shape[1] % 128 == 0
    R, K = x.shape
    q = np.empty((R, K), dtype=np.uint8)
    scale = np.empty((R, K // 128), dtype=np.float32)
    lib().oracle_quantize_rows_1x128(C.c_int32(R), C.c_int32(K), _ptr(x), _ptr(q), _ptr(scale))
    return q, scale


def f32_to_e4m3(v: float) -> int:
    return int(lib().oracle_f32_to_e4m3(C.c_float(v)))


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def router_logits(p: Problem) -> np.ndarray:
    z = np.empty((p.T, p.E), dtype=np.float64)
    lib().oracle_router_logits(C.byref(p._c), _ptr(z))
    return z


def route(p: Problem, z: np.ndarray):
    """-> ids [T,k] int32, w [T,k] float64, margin [T] float64."""
    z = _f64(z)
    assert z.shape == (p.T, p.E)
    ids = np.empty((p.T, p.top_k), dtype=np.int32)
    w = np.empty((p.T, p.top_k), dtype=np.float64)
    margin = np.empty((p.T,), dtype=np.float64)
    lib().oracle_route(C.byref(p._c), _ptr(z), _ptr(ids), _ptr(w), _ptr(margin))
    return ids, w, margin


def permute(ids: np.ndarray, E: int):
    """-> offsets [E+1], sorted_pair [P], inv [P] (all int32)."""
    flat = _i32(ids).reshape(-1)
    P = flat.size
    offsets = np.empty((E + 1,), dtype=np.int32)
    sorted_pair = np.empty((P,), dtype=np.int32)
    inv = np.empty((P,), dtype=np.int32)
    lib().oracle_permute(C.c_int32(P), C.c_int32(E), _ptr(flat), _ptr(offsets), _ptr(sorted_pair), _ptr(inv))
    return offsets, sorted_pair, inv


def swiglu_rows(p: Problem, tok: Sequence[int], expert: Sequence[int]) -> np.ndarray:
    tok, expert = _i32(tok), _i32(expert)
    n = tok.size
    assert expert.size == n
    act = np.empty((n, p.I), dtype=np.float64)
    lib().oracle_swiglu_rows(C.byref(p._c), C.c_int32(n), _ptr(tok), _ptr(expert), _ptr(act))
    return act


def down_rows(p: Problem, expert: Sequence[int], act: np.ndarray) -> np.ndarray:
    expert, act = _i32(expert), _f64(act)
    n = expert.size
    assert act.shape == (n, p.I)
    y = np.empty((n, p.H), dtype=np.float64)
    lib().oracle_down_rows(C.byref(p._c), C.c_int32(n), _ptr(expert), _ptr(act), _ptr(y))
    return y


def combine(w: np.ndarray, inv: np.ndarray, y: np.ndarray) -> np.ndarray:
    w, inv, y = _f64(w), _i32(inv).reshape(-1), _f64(y)
    T, k = w.shape
    H = y.shape[1]
    assert inv.size == T * k and y.shape[0] == T * k
    out = np.empty((T, H), dtype=np.float64)
    lib().oracle_combine(C.c_int32(T), C.c_int32(k), C.c_int32(H), _ptr(w), _ptr(inv), _ptr(y), _ptr(out))
    return out


def forward_tokens(p: Problem, tokens: Sequence[int]):
    """Layer output for the listed tokens -> out [n,H] f64, ids [n,k], w [n,k], margin [n]."""
    tokens = _i32(tokens)
    n = tokens.size
    out = np.empty((n, p.H), dtype=np.float64)
    ids = np.empty((n, p.top_k), dtype=np.int32)
    w = np.empty((n, p.top_k), dtype=np.float64)
    margin = np.empty((n,), dtype=np.float64)
    lib().oracle_forward_tokens(C.byref(p._c), C.c_int32(n), _ptr(tokens), _ptr(out), _ptr(ids), _ptr(w),
                                _ptr(margin))
    return out, ids, w, margin


def forward(p: Problem):
    return forward_tokens(p, np.arange(p.T, dtype=np.int32))


def bf16_to_f64(code: int) -> float:
    return lib().oracle_bf16_to_f64(C.c_uint16(code))


def e4m3_to_f64(code: int) -> float:
    return lib().oracle_e4m3_to_f64(C.c_uint8(code))


def num_threads() -> int:
    return int(lib().oracle_num_threads())
