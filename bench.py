#!/usr/bin/env python3
"""Benchmark of the fused MoE forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one whole layer forward (route, sort-scatter, gate/up GEMM + SiLU gating,
down GEMM, combine) through the C ABI on synthetic tensors that are resident in
HBM before the timed region starts.  Prints one JSON line: latency per forward,
TFLOP/s and GB/s with their fractions of the MI355X peaks, the roofline of the
dominant kernel (gate/up grouped GEMM) from HIP events recorded around it in the
timed region, and the CPU oracle timed on a bounded token sample of the same
workload.
"""
import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0                                   # MI355X HBM3E
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "fp8": 5000.0}       # dense


class HipEvents:
    """hipEvent_t handles through the HIP runtime PyTorch already loaded (plumbing only)."""

    def __init__(self):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]

    def make(self, n):
        arr = (C.c_void_p * n)()
        for i in range(n):
            ev = C.c_void_p()
            rc = self.hip.hipEventCreate(C.byref(ev))
            assert rc == 0, f"hipEventCreate failed: {rc}"
            arr[i] = ev
        return arr

    def ms(self, a, b):
        out = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(out), a, b)
        assert rc == 0, f"hipEventElapsedTime failed: {rc}"
        return float(out.value)

    def free(self, arr):
        for ev in arr:
            self.hip.hipEventDestroy(ev)


def measured_traffic(workload):
    """HBM bytes per launch of the gate/up GEMM from the committed counter summary, or None when
    the kernel source has changed since the counters were taken (or none were taken)."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "traffic.json")
    src = os.path.join(ROOT, "paper_2602_19128_amd", "csrc", "moe_gemm.hip")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        doc = json.load(f)
    sha = hashlib.sha256(open(src, "rb").read()).hexdigest()
    rec = doc.get(workload)
    if not rec or rec.get("moe_gemm_sha256") != sha:
        return None
    return {"fetch_bytes": rec["fetch_bytes"], "write_bytes": rec["write_bytes"], "unit": "bytes per launch"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="mixtral_prefill")
    ap.add_argument("--tokens", type=int, default=0,
                    help="override the workload's token count (supplementary points; not the headline config)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (a kernel of known HBM traffic, used to scale "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--graph", action="store_true",
                    help="supplementary: also time the same forward replayed from a HIP graph (the five launches "
                         "recorded once; reported as graph_replay_us, never as value)")
    ap.add_argument("--cpu-baseline-seconds", type=float, default=15.0,
                    help="CPU work budget for the oracle sample; 0 skips the CPU baseline")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures the single-GPU kernel path only: run with --gpus 1 "
              "(this library has no multi-GPU code; the layer would shard by expert parallelism, one "
              "local-expert call per device plus a reduce-scatter of the partial outputs)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_19128_amd import binding as moe
    from paper_2602_19128_amd import synthetic as syn

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    moe.load()
    wl = syn.WORKLOADS[args.workload]
    if args.tokens > 0:
        wl = wl.replace(T=args.tokens, name=f"{wl.name}_T{args.tokens}")
    dev = torch.device("cuda:0")
    inp = syn.make_inputs(wl, seed=args.seed, device=dev)
    cfg = moe.MoEConfig.from_workload(wl)
    out = torch.empty((wl.T, wl.H), dtype=torch.bfloat16, device=dev)
    ws = torch.empty((moe.moe_workspace_size(cfg),), dtype=torch.uint8, device=dev)
    call = lambda ev=None: moe.moe_forward(cfg, inp.x, inp.x_scale, inp.router_w, inp.bias, inp.w1, inp.w1_scale,
                                           inp.w2, inp.w2_scale, out=out, workspace=ws, events=ev)

    if args.copy_calibration:
        src = torch.ones((1 << 28,), dtype=torch.float32, device=dev)          # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    hip = HipEvents()
    K, W = args.steps, args.warmup
    events = [hip.make(moe.FORWARD_EVENTS) for _ in range(K)]
    for _ in range(W):
        call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        call(events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K

    # supplementary: the same call recorded into a HIP graph and replayed (launch overhead of the
    # multi-launch pipeline removed; the library neither allocates nor synchronises, so it can be captured)
    graph_us = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            call()                                       # everything one-time happens outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            call()
        ref_out = out.clone()
        for _ in range(W):
            graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(K):
            graph.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - g0) * 1e6 / K
        assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16)), "graph replay changed the output"

    step_ms = {name: 0.0 for name in moe.STEP_NAMES}
    for ev in events:
        for j, name in enumerate(moe.STEP_NAMES):
            step_ms[name] += hip.ms(ev[j], ev[j + 1]) / K
    gpu_ms = sum(hip.ms(ev[0], ev[moe.FORWARD_EVENTS - 1]) for ev in events) / K
    for ev in events:
        hip.free(ev)

    # ---- work the method itself has to do (no padding flops, no skipped experts) -------------
    ids, w = moe.moe_route(cfg, inp.x, inp.x_scale, inp.router_w, inp.bias)
    counts = torch.bincount(ids.reshape(-1).long(), minlength=wl.E).cpu().numpy()
    counts = counts[wl.local_offset: wl.local_offset + wl.EL]      # experts whose weights this call holds
    e_active = int((counts > 0).sum())
    T, H, I, E, k = wl.T, wl.H, wl.I, wl.E, wl.top_k
    P = int(counts.sum())                    # (token, slot) pairs that reach a local expert
    bw = 1 if wl.fp8 else 2                      # bytes per weight / activation payload element
    scale_w = (e_active * (2 * I // 128) * (H // 128) + e_active * (H // 128) * (I // 128)) * 4 if wl.fp8 else 0
    flops = 6.0 * H * I * P + 2.0 * T * E * H
    bx = 2 if wl.quantize_x else bw           # hidden states arrive as bf16 when the layer quantises them itself
    bytes_min = e_active * 3 * H * I * bw + scale_w + T * H * bx + E * H * 4 + T * H * 2
    sec = ms_per_step * 1e-3
    kind = "fp8" if wl.fp8 else "bf16"
    tflops = flops / sec / 1e12
    gbps = bytes_min / sec / 1e9

    # dominant kernel: gate/up grouped GEMM.  Algorithmic bytes of one launch: the active experts'
    # gate/up weights once, the hidden states once, the activations written once.
    g1_bytes = e_active * 2 * I * H * bw + T * H * bw + P * I * bw
    if wl.fp8:
        g1_bytes += e_active * (2 * I // 128) * (H // 128) * 4 + T * (H // 128) * 4 + P * (I // 128) * 4
    g1_sec = step_ms["gemm_swiglu"] * 1e-3
    g1_gbps = g1_bytes / g1_sec / 1e9
    roofline = {"kernel": "grouped_gemm_swiglu", "bound": "hbm", "achieved": round(g1_gbps, 1),
                "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": round(g1_gbps / PEAK_HBM_GBPS, 4),
                "traffic": measured_traffic(wl.name), "bytes_per_launch": int(g1_bytes), "avg_launch_us": round(g1_sec * 1e6, 2),
                "tflops": round(4.0 * H * I * P / g1_sec / 1e12, 1),
                "frac_mfma": round(4.0 * H * I * P / g1_sec / 1e12 / PEAK_MFMA_TFLOPS[kind], 4)}

    # ---- CPU oracle on a bounded token sample of the same workload ------------------------------
    cpu_baseline = None
    parity = None
    if args.cpu_baseline_seconds > 0:
        from oracle import moe_oracle as orc
        cpu = inp.to("cpu")
        prob = orc.problem_from_inputs(cpu)
        rng = np.random.default_rng(args.seed)
        order = rng.permutation(T).astype(np.int32)
        probe = min(8, T - 1)                  # a few tokens to size the sample (their cost varies in local-expert mode)
        c0 = time.perf_counter()
        ref0, *_ = orc.forward_tokens(prob, order[:probe])
        per_tok = (time.perf_counter() - c0) / probe
        n = int(max(1, min(T - probe, args.cpu_baseline_seconds / max(per_tok, 1e-9))))
        sample = order[probe:probe + n]
        c0 = time.perf_counter()
        ref, ids_r, w_r, margin_r = orc.forward_tokens(prob, sample)
        cpu_s = time.perf_counter() - c0
        cpu_baseline = {"value": round(cpu_s / n * T * 1e6, 1), "unit": "us", "cores": orc.num_threads(),
                        "kind": "oracle",
                        "sample": f"{n} of {T} tokens (every local expert each of them chose) in {cpu_s:.1f} s, scaled by T/n"}
        got = out[torch.from_numpy(sample.astype(np.int64)).to(dev)].float().cpu().numpy().astype(np.float64)
        same = np.array([sorted(a) == sorted(b) for a, b in
                         zip(ids[torch.from_numpy(sample.astype(np.int64)).to(dev)].cpu().numpy(), ids_r)])
        err = np.abs(got[same] - ref[same])
        parity = {"tokens": int(same.sum()), "tie_excused": int((~same).sum()),
                  "max_rel": float(err.max() / np.abs(ref[same]).max()),
                  "mean_rel": float(err.sum() / np.abs(ref[same]).sum())}

    line = {
        "metric": "fused_moe_forward_latency", "value": round(ms_per_step * 1e3, 2), "unit": "us",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": kind,
        "data": "synthetic", "config": {"workload": wl.name, "T": T, "H": H, "I": I, "E": E, "top_k": k,
                                        "scoring": wl.scoring, "n_group": wl.n_group, "seed": args.seed,
                                        "local_experts": [wl.local_offset, wl.EL], "routed_pairs": P,
                                        "tile_rows": moe.moe_tile_rows(cfg), "active_experts": e_active,
                                        "max_over_mean_load": round(float(counts.max() / max(counts.mean(), 1e-9)), 2)},
        "tflops": round(tflops, 1), "frac_mfma_peak": round(tflops / PEAK_MFMA_TFLOPS[kind], 4),
        "gbps": round(gbps, 1), "frac_hbm_peak": round(gbps / PEAK_HBM_GBPS, 4),
        "roofline_time_us": round(max(flops / (PEAK_MFMA_TFLOPS[kind] * 1e12), bytes_min / (PEAK_HBM_GBPS * 1e9)) * 1e6, 1),
        "gpu_event_us": round(gpu_ms * 1e3, 2),
        "graph_replay_us": None if graph_us is None else round(graph_us, 2),
        "step_us": {n_: round(v * 1e3, 2) for n_, v in step_ms.items()},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "parity_sample": parity,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
