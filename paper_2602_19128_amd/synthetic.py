"""Seeded synthetic workloads for the fused MoE forward.

This module only draws random tensors and stores them in the dtypes the layer
consumes.  It holds none of the layer's arithmetic: no routing, no GEMM, no
activation.  The one numeric step here is the block quantisation that turns
generated values into the fp8 payload + fp32 scales an fp8 workload *arrives*
with.  (Workloads with `quantize_x` hand the layer bf16 hidden states instead and
the layer quantises them itself; nothing here is used for that.)

Shapes follow the MoE operator the paper analyses (Sec. 4.5: DeepSeek-V3 style,
256 experts, top-8, hidden size 7168) plus a Mixtral-shaped and a tiny case.
The paper measured on captured serving traces that are not available; these
tensors stand in for them.

Every value is a pure function of (seed, tensor id, element index): a counter-based generator
(the splitmix64 sequence, keyed per tensor) written with integer tensor operations only, so a
tensor's values depend neither on which other tensors were generated, nor on the order, nor on the
device: a draw on the GPU and a draw on the CPU give the same bits, and one device's share of the
experts holds exactly the values of that slice of the full layer.  Normal variates are the sum of
twelve 16-bit uniforms (Irwin-Hall: mean 0, variance 1, support +-6), which needs integer additions
and one exact scaling only; library normal generators differ between devices and math libraries.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, Optional

import torch

FP8_MAX = 448.0          # largest finite OCP e4m3fn magnitude
QBLOCK = 128             # block edge of the fp8 scales


@dataclass(frozen=True)
class Workload:
    """Problem statement of one MoE layer call (shapes + routing rule)."""
    name: str
    T: int                      # tokens
    H: int                      # hidden size
    I: int                      # expert intermediate size
    E: int                      # experts
    top_k: int
    scoring: str = "softmax"    # "softmax" | "sigmoid"
    n_group: int = 1            # >1: group-limited routing
    topk_group: int = 1
    group_score_topn: int = 2
    routed_scale: float = 1.0
    has_bias: bool = False
    fp8: bool = False
    hot_experts: int = 0        # skew variant: this many experts get +hot_bias
    hot_bias: float = 0.0
    local_offset: int = 0       # local-expert mode: first expert whose weights are held ...
    local_experts: int = 0      # ... and how many (0 = all E)
    quantize_x: bool = False    # fp8 only: hidden states arrive as bf16 and the layer quantises them itself

    @property
    def EL(self) -> int:
        """Experts whose weights the call holds."""
        return self.local_experts if self.local_experts > 0 else self.E

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


_DSV3 = dict(H=7168, I=2048, E=256, top_k=8, scoring="sigmoid", n_group=8,
             topk_group=4, group_score_topn=2, routed_scale=2.5, has_bias=True)

WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", T=16, H=256, I=128, E=8, top_k=2),
    "mixtral_prefill": Workload("mixtral_prefill", T=512, H=4096, I=14336, E=8, top_k=2),
    "dsv3_decode": Workload("dsv3_decode", T=64, **_DSV3),
    "dsv3_prefill": Workload("dsv3_prefill", T=4096, **_DSV3),
    "dsv3_prefill_skew": Workload("dsv3_prefill_skew", T=4096, hot_experts=16,
                                  hot_bias=0.5, **_DSV3),
    "fp8_prefill": Workload("fp8_prefill", T=1024, fp8=True, **_DSV3),
    # one device's share under 8-way expert parallelism: 32 local experts of 256 (the shape of the
    # paper's Sec. 4.5 workload); experts 96..127 are group 3 of the 8 routing groups
    "fp8_local32": Workload("fp8_local32", T=4096, fp8=True, local_offset=96, local_experts=32, **_DSV3),
    # fp8 weights, hidden states arriving in bf16: the 1x128 activation quantisation (the "fp8
    # packing and scaling" the paper's kernel table names for this operator) runs inside the layer
    "fp8_prefill_qx": Workload("fp8_prefill_qx", T=1024, fp8=True, quantize_x=True, **_DSV3),
    "fp8_local32_qx": Workload("fp8_local32_qx", T=4096, fp8=True, quantize_x=True, local_offset=96,
                               local_experts=32, **_DSV3),
}

# tensor ids for the per-tensor generator streams
_TID = {"x": 1, "router_w": 2, "bias": 3, "w1": 4, "w2": 5}

_M64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """A 64-bit pattern as the signed integer torch.int64 holds."""
    v &= _M64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLD, _MIX1, _MIX2 = _s64(0x9E3779B97F4A7C15), _s64(0xBF58476D1CE4E5B9), _s64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 (the >> of a signed tensor is arithmetic)."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    """The output function of splitmix64 (int64 arithmetic wraps, as the generator needs)."""
    x = (x ^ _lsr(x, 30)) * _MIX1
    x = (x ^ _lsr(x, 27)) * _MIX2
    return x ^ _lsr(x, 31)


def _mix_int(v: int) -> int:
    v &= _M64
    v = ((v ^ (v >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    v = ((v ^ (v >> 27)) * 0x94D049BB133111EB) & _M64
    return v ^ (v >> 31)


def _key(seed: int, tid: int) -> int:
    """Start state of a tensor's stream."""
    return _s64(_mix_int(_mix_int(seed * 0x9E3779B97F4A7C15 + 0x1234567) + tid * 0x9E3779B97F4A7C15))


def _words(key: int, first: int, count: int, per: int, j: int, device) -> torch.Tensor:
    """Word j (of `per`) of elements first .. first+count-1: output number per*index + j of the stream."""
    n = torch.arange(first, first + count, dtype=torch.int64, device=device) * per + (j + 1)
    return _mix(n * _GOLD + key)


_CHUNK = 1 << 27          # elements generated at a time (bounds the int64 temporaries: about 1 GiB each)


def _normal(shape, std: float, seed: int, tid: int, device, first: int = 0) -> torch.Tensor:
    """fp32 tensor of `shape`; element i of the flattened tensor is variate number first + i of stream (seed, tid)."""
    total = 1
    for d in shape:
        total *= d
    out = torch.empty((total,), dtype=torch.float32, device=device)
    key = _key(seed, tid)
    for at in range(0, total, _CHUNK):
        cnt = min(_CHUNK, total - at)
        acc = torch.zeros((cnt,), dtype=torch.int64, device=device)
        for j in range(3):                               # 3 words = 12 uniforms of 16 bits
            h = _words(key, first + at, cnt, 3, j, device)
            acc += (h & 0xFFFF) + (_lsr(h, 16) & 0xFFFF) + (_lsr(h, 32) & 0xFFFF) + _lsr(h, 48)
        # sum of 12 uniforms on {0..65535}: mean 393210, standard deviation 65536 (to 1e-10); both steps exact in fp32
        out[at:at + cnt] = (acc - 393210).to(torch.float32) * (1.0 / 65536.0)
    return (out * std).reshape(shape)


def _uniform(shape, seed: int, tid: int, device) -> torch.Tensor:
    """fp32 uniforms on [0, 1) with 24 bits (exact in fp32)."""
    total = 1
    for d in shape:
        total *= d
    h = _words(_key(seed, tid), 0, total, 1, 0, device)
    return (_lsr(h, 40).to(torch.float32) * (1.0 / 16777216.0)).reshape(shape)


def hot_expert_ids(wl: Workload):
    """Skew variant: the first `hot_experts / n_group` experts of every group."""
    if wl.hot_experts <= 0:
        return []
    per = max(1, wl.hot_experts // max(1, wl.n_group))
    gsz = wl.E // max(1, wl.n_group)
    ids = []
    for g in range(max(1, wl.n_group)):
        ids.extend(g * gsz + j for j in range(per))
    return ids[: wl.hot_experts]


def quantize_rows_1x128(v: torch.Tensor):
    """[R, K] fp32 -> (fp8 e4m3fn payload [R, K], fp32 scale [R, K/128]).

    scale = amax(block) / 448 (1 if the block is all zero); payload = v / scale
    rounded to nearest-even by the dtype conversion, clamped to +-448 first.
    """
    R, K = v.shape
    assert K % QBLOCK == 0
    b = v.reshape(R, K // QBLOCK, QBLOCK)
    amax = b.abs().amax(dim=-1)
    scale = torch.where(amax > 0, amax / torch.full_like(amax, FP8_MAX), torch.ones_like(amax))   # (a tensor divisor: the
    # division by a Python scalar is a multiplication by its reciprocal on some devices)
    q = (b / scale.unsqueeze(-1)).clamp_(-FP8_MAX, FP8_MAX).to(torch.float8_e4m3fn)
    return q.reshape(R, K).contiguous(), scale.contiguous()


def quantize_blocks_128x128(v: torch.Tensor):
    """[N, K] fp32 -> (fp8 payload [N, K], fp32 scale [N/128, K/128])."""
    N, K = v.shape
    assert N % QBLOCK == 0 and K % QBLOCK == 0
    b = v.reshape(N // QBLOCK, QBLOCK, K // QBLOCK, QBLOCK)
    amax = b.abs().amax(dim=(1, 3))
    scale = torch.where(amax > 0, amax / torch.full_like(amax, FP8_MAX), torch.ones_like(amax))   # (a tensor divisor: the
    # division by a Python scalar is a multiplication by its reciprocal on some devices)
    q = (b / scale[:, None, :, None]).clamp_(-FP8_MAX, FP8_MAX).to(torch.float8_e4m3fn)
    return q.reshape(N, K).contiguous(), scale.contiguous()


@dataclass
class MoEInputs:
    wl: Workload
    x: torch.Tensor                       # [T,H] bf16, or fp8 e4m3fn when wl.fp8
    router_w: torch.Tensor                # [E,H] fp32
    bias: Optional[torch.Tensor]          # [E] fp32 or None
    w1: torch.Tensor                      # [EL,2I,H] bf16 / fp8 ; rows [0,I) gate, [I,2I) up
    w2: torch.Tensor                      # [EL,H,I]  bf16 / fp8
    x_scale: Optional[torch.Tensor] = None    # [T,H/128] fp32
    w1_scale: Optional[torch.Tensor] = None   # [EL,2I/128,H/128] fp32
    w2_scale: Optional[torch.Tensor] = None   # [EL,H/128,I/128] fp32

    def to(self, device) -> "MoEInputs":
        mv = lambda t: None if t is None else t.to(device)
        return MoEInputs(self.wl, mv(self.x), mv(self.router_w), mv(self.bias), mv(self.w1),
                         mv(self.w2), mv(self.x_scale), mv(self.w1_scale), mv(self.w2_scale))

    def local_share(self, offset: int, count: int) -> "MoEInputs":
        """The same layer call as seen by a device that holds only experts [offset, offset+count)."""
        assert self.wl.local_experts == 0 and 0 <= offset and offset + count <= self.wl.E
        cut = lambda t: None if t is None else t[offset:offset + count].contiguous()
        wl = self.wl.replace(name=f"{self.wl.name}_local{offset}+{count}", local_offset=offset, local_experts=count)
        return MoEInputs(wl, self.x, self.router_w, self.bias, cut(self.w1), cut(self.w2), self.x_scale,
                         cut(self.w1_scale), cut(self.w2_scale))


def make_inputs(wl: Workload, seed: int = 0, device="cpu",
                weights_from: Optional[MoEInputs] = None) -> MoEInputs:
    """Draw one workload's tensors.

    `weights_from`: reuse the router and expert weights of an earlier draw with the
    same H/I/E/dtype and seed (they do not depend on T), drawing only x and bias.

    hidden ~ N(0,1); router W ~ N(0,1/H) fp32; expert weights ~ N(0,1/fan_in);
    bias ~ U(-0.1,0.1) (+hot_bias on the hot experts).  bf16 workloads round to
    bf16; fp8 workloads block-quantise (1x128 activations, 128x128 weights).
    Expert weights are drawn one expert at a time to bound the temporaries; in local-expert
    mode only the local experts are drawn, and they hold the values of the same experts of
    the full layer.
    """
    dev = torch.device(device)
    T, H, I, E = wl.T, wl.H, wl.I, wl.E
    x32 = _normal((T, H), 1.0, seed, _TID["x"], dev)
    router_w = _normal((E, H), H ** -0.5, seed, _TID["router_w"], dev)
    bias = None
    if wl.has_bias:
        bias = _uniform((E,), seed, _TID["bias"], dev) * 0.2
        bias = bias - 0.1
        hot = hot_expert_ids(wl)
        if hot:
            bias[torch.tensor(hot, device=dev)] += wl.hot_bias
    if wl.fp8 and not wl.quantize_x:
        x, x_scale = quantize_rows_1x128(x32)
    else:
        x, x_scale = x32.to(torch.bfloat16), None
    if weights_from is not None:
        o = weights_from
        assert (o.wl.H, o.wl.I, o.wl.E, o.wl.fp8, o.wl.local_offset, o.wl.local_experts) == \
            (H, I, E, wl.fp8, wl.local_offset, wl.local_experts) and o.w1.device.type == dev.type
        return MoEInputs(wl, x, o.router_w, bias, o.w1, o.w2, x_scale, o.w1_scale, o.w2_scale)
    wdt = torch.float8_e4m3fn if wl.fp8 else torch.bfloat16
    EL, lo = wl.EL, wl.local_offset
    w1 = torch.empty((EL, 2 * I, H), dtype=wdt, device=dev)
    w2 = torch.empty((EL, H, I), dtype=wdt, device=dev)
    w1_scale = w2_scale = None
    if wl.fp8:
        w1_scale = torch.empty((EL, 2 * I // QBLOCK, H // QBLOCK), dtype=torch.float32, device=dev)
        w2_scale = torch.empty((EL, H // QBLOCK, I // QBLOCK), dtype=torch.float32, device=dev)
    def draw(out, out_scale, rows, cols, std, tid):
        """Experts lo .. lo+EL-1 of the full layer's [E, rows, cols] tensor, several experts at a time."""
        per = rows * cols
        group = max(1, _CHUNK // per)
        for e0 in range(0, EL, group):
            n = min(group, EL - e0)
            v = _normal((n * rows, cols), std, seed, tid, dev, first=(lo + e0) * per)
            if wl.fp8:                                   # rows is a multiple of 128: blocks never straddle experts
                q, sc = quantize_blocks_128x128(v)
                out[e0:e0 + n] = q.view(n, rows, cols)
                out_scale[e0:e0 + n] = sc.view(n, rows // QBLOCK, cols // QBLOCK)
            else:
                out[e0:e0 + n] = v.to(torch.bfloat16).view(n, rows, cols)
            del v

    draw(w1, w1_scale, 2 * I, H, H ** -0.5, _TID["w1"])
    draw(w2, w2_scale, H, I, I ** -0.5, _TID["w2"])
    return MoEInputs(wl, x, router_w, bias, w1, w2, x_scale, w1_scale, w2_scale)
