#!/usr/bin/env python3
"""Benchmark of the fused MoE forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--only]

A step is one whole layer forward (route, sort-scatter, gate/up GEMM + SiLU gating,
down GEMM, combine) through the C ABI on synthetic tensors that are resident in
HBM before the timed region starts.  Prints ONE JSON line.  Its top level describes
the headline workload (default: the largest single-GPU configuration, the 4096-token
DeepSeek-V3-shaped prefill): latency per forward, TFLOP/s and GB/s with their
fractions of the MI355X peaks, the roofline of the dominant kernel (gate/up grouped
GEMM) from HIP events recorded around it inside the timed region, and the CPU oracle
timed on a bounded token sample of the same workload.  Unless --only is given, the
other benchmark configurations are measured in the same run (same K and W, the
DeepSeek-shaped ones on the same weights) and nested, in compact form, under
"workloads".  The run fails (exit 1) if any sampled output disagrees with the oracle
beyond the tolerances.
"""
import argparse
import ctypes as C
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0                                   # MI355X HBM3E
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "fp8": 5000.0}       # dense
TOL_MAX = {"bf16": 2e-2, "fp8": 6e-2}                    # max |err| / max |ref|
TOL_MEAN = {"bf16": 5e-3, "fp8": 3e-2}                   # sum |err| / sum |ref|

HEADLINE = "dsv3_prefill"
# measured beside the headline, in this order; entries that share H/I/E/dtype share their weights
ALSO = ["tiny", "mixtral_prefill", "dsv3_decode", "dsv3_prefill_skew", "fp8_prefill", "fp8_local32"]
# oracle budget: these run every token when that fits the time given, the others a bounded sample
ORACLE_IN_FULL = {"tiny": 5.0, "dsv3_decode": 20.0, "mixtral_prefill": 60.0}

GEMM_SOURCES = ["moe_gemm_kernel.hpp", "moe_gemm.hip", "moe_gemm_gateup_bf16.hip", "moe_gemm_gateup_fp8.hip",
                "moe_gemm_down_bf16.hip", "moe_gemm_down_fp8.hip"]


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


def gemm_source_hash():
    h = hashlib.sha256()
    for name in GEMM_SOURCES:
        with open(os.path.join(ROOT, "paper_2602_19128_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(workload):
    """HBM bytes per launch of the gate/up GEMM from the committed counter summary, or None when
    the kernel sources have changed since the counters were taken (or none were taken)."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        doc = json.load(f)
    rec = doc.get(workload)
    if not rec or rec.get("gemm_sources_sha256") != gemm_source_hash():
        return None
    return {"fetch_bytes": rec["fetch_bytes"], "write_bytes": rec["write_bytes"], "unit": "bytes per launch"}


def measure(wl, inp, host, K, W, cpu_seconds, graph, seed, log, min_warm_ms=0.0):
    """One workload: K timed forwards after W warm-up ones, the per-step HIP events, the work and
    roofline figures, and the oracle on a token sample (timed, and compared with the GPU output).
    `host`: the same tensors on the CPU for the oracle (None skips the oracle)."""
    import numpy as np
    import torch
    from paper_2602_19128_amd import binding as moe

    dev = inp.x.device
    cfg = moe.MoEConfig.from_workload(wl)
    out = torch.empty((wl.T, wl.H), dtype=torch.bfloat16, device=dev)
    ws = torch.empty((moe.moe_workspace_size(cfg),), dtype=torch.uint8, device=dev)
    call = lambda ev=None: moe.moe_forward(cfg, inp.x, inp.x_scale, inp.router_w, inp.bias, inp.w1, inp.w1_scale,
                                           inp.w2, inp.w2_scale, out=out, workspace=ws, events=ev)
    hip = HipEvents()
    events = [hip.make(moe.FORWARD_EVENTS) for _ in range(K)]
    for _ in range(W):
        call()
    torch.cuda.synchronize()
    # Nested workloads: keep warming up until the GPU has worked for `min_warm_ms` (a forward of a
    # few hundred microseconds, timed after five calls, still runs at the clocks of an idle GPU:
    # +5..9 % measured).  The headline workload gets exactly W warm-up steps.
    w0 = time.perf_counter()
    while (time.perf_counter() - w0) * 1e3 < min_warm_ms:
        for _ in range(8):
            call()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        call(events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K

    # the same K forwards without the step events (recording five events per call costs a few
    # microseconds each, which is most of a latency-bound layer), and - where the library offers it
    # for this problem - as one persistent launch instead of the pipeline
    plain = moe.PreparedForward(cfg, inp.x, inp.x_scale, inp.router_w, inp.bias, inp.w1, inp.w1_scale, inp.w2,
                                inp.w2_scale, out, ws)

    def unmarked():
        for _ in range(max(W, 20)):
            plain()
        torch.cuda.synchronize()
        u0 = time.perf_counter()
        for _ in range(K):
            plain()
        torch.cuda.synchronize()
        return (time.perf_counter() - u0) * 1e6 / K

    unmarked_us = unmarked()
    single_us = None
    moe.moe_single_launch(True)
    try:
        if moe.moe_single_launch_mode(cfg) == moe.SINGLE_LAUNCH_ALL:
            pipeline_bits = out.clone()
            single_us = unmarked()
            assert torch.equal(out.view(torch.int16), pipeline_bits.view(torch.int16)), "single launch changed the output"
    finally:
        moe.moe_single_launch(False)

    # supplementary: the same call recorded into a HIP graph and replayed (the library neither
    # allocates nor synchronises, so it can be captured)
    graph_us = None
    if graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            call()                                       # everything one-time happens outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            call()
        ref_out = out.clone()
        for _ in range(W):
            g.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(K):
            g.replay()
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
    bw = 1 if wl.fp8 else 2                  # bytes per weight / activation payload element
    scale_w = (e_active * (2 * I // 128) * (H // 128) + e_active * (H // 128) * (I // 128)) * 4 if wl.fp8 else 0
    flops = 6.0 * H * I * P + 2.0 * T * E * H
    bx = 2 if wl.quantize_x else bw           # hidden states arrive as bf16 when the layer quantises them itself
    bytes_min = e_active * 3 * H * I * bw + scale_w + T * H * bx + E * H * 4 + T * H * 2
    sec = ms_per_step * 1e-3
    kind = "fp8" if wl.fp8 else "bf16"
    tflops = flops / sec / 1e12
    gbps = bytes_min / sec / 1e9
    ideal_us = max(flops / (PEAK_MFMA_TFLOPS[kind] * 1e12), bytes_min / (PEAK_HBM_GBPS * 1e9)) * 1e6

    # dominant kernel: gate/up grouped GEMM.  Algorithmic bytes of one launch: the active experts'
    # gate/up weights once, the hidden states once, the activations written once.
    g1_bytes = e_active * 2 * I * H * bw + T * H * bw + P * I * bw
    if wl.fp8:
        g1_bytes += e_active * (2 * I // 128) * (H // 128) * 4 + T * (H // 128) * 4 + P * (I // 128) * 4
    g1_sec = step_ms["gemm_swiglu"] * 1e-3
    g1_gbps = g1_bytes / g1_sec / 1e9
    g2_bytes = e_active * H * I * bw + P * I * bw + P * H * 2 + (e_active * (H // 128) * (I // 128) * 4 + P * (I // 128) * 4 if wl.fp8 else 0)
    g2_gbps = g2_bytes / (step_ms["gemm_down"] * 1e-3) / 1e9
    roofline = {"kernel": "grouped_gemm_swiglu", "bound": "hbm", "achieved": round(g1_gbps, 1),
                "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": round(g1_gbps / PEAK_HBM_GBPS, 4),
                "traffic": measured_traffic(wl.name), "bytes_per_launch": int(g1_bytes), "avg_launch_us": round(g1_sec * 1e6, 2),
                "tflops": round(4.0 * H * I * P / g1_sec / 1e12, 1),
                "frac_mfma": round(4.0 * H * I * P / g1_sec / 1e12 / PEAK_MFMA_TFLOPS[kind], 4),
                "down_gemm": {"achieved": round(g2_gbps, 1), "frac": round(g2_gbps / PEAK_HBM_GBPS, 4),
                              "bytes_per_launch": int(g2_bytes)}}

    # ---- CPU oracle on a bounded token sample of the same workload ------------------------------
    cpu_baseline = None
    parity = None
    if host is not None and cpu_seconds > 0:
        from oracle import moe_oracle as orc
        prob = orc.problem_from_inputs(host)
        rng = np.random.default_rng(seed)
        order = rng.permutation(T).astype(np.int32)
        full_budget = ORACLE_IN_FULL.get(wl.name, 0.0)
        probe = max(1, min(4, T // 4))         # a few tokens to size the sample (their cost varies in local-expert mode)
        c0 = time.perf_counter()
        orc.forward_tokens(prob, order[:probe])
        per_tok = (time.perf_counter() - c0) / probe
        if per_tok * T <= max(full_budget, cpu_seconds):
            sample, what = order, "every token"
        else:
            n = int(max(1, min(T, cpu_seconds / max(per_tok, 1e-9))))
            sample, what = order[:n], "sampled, scaled by T/n"
        n = len(sample)
        c0 = time.perf_counter()
        ref, ids_r, w_r, margin_r = orc.forward_tokens(prob, sample)
        cpu_s = time.perf_counter() - c0
        cpu_baseline = {"value": round(cpu_s / n * T * 1e6, 1), "unit": "us", "cores": orc.num_threads(),
                        "kind": "oracle",
                        "sample": f"{n} of {T} tokens ({what}; every local expert each of them chose) in {cpu_s:.1f} s"}
        pick = torch.from_numpy(sample.astype(np.int64)).to(dev)
        got = out[pick].float().cpu().numpy().astype(np.float64)
        same = np.array([sorted(a) == sorted(b) for a, b in zip(ids[pick].cpu().numpy(), ids_r)])
        tie_ok = bool((margin_r[~same] < 1e-6).all())      # another expert set is allowed only at a tie
        err = np.abs(got[same] - ref[same])
        peak, total = float(np.abs(ref[same]).max()), float(np.abs(ref[same]).sum())
        parity = {"tokens": int(same.sum()), "tie_excused": int((~same).sum()),
                  "max_rel": float(err.max() / peak) if peak > 0 else 0.0,
                  "mean_rel": float(err.sum() / total) if total > 0 else 0.0}
        parity["ok"] = bool(tie_ok and parity["max_rel"] <= TOL_MAX[kind] and parity["mean_rel"] <= TOL_MEAN[kind])
        log(f"{wl.name}: oracle {n}/{T} tokens in {cpu_s:.1f} s, max_rel={parity['max_rel']:.2e} "
            f"mean_rel={parity['mean_rel']:.2e} ok={parity['ok']}")

    return {
        "value": round(ms_per_step * 1e3, 2), "ms_per_step": round(ms_per_step, 5), "dtype": kind,
        "config": {"workload": wl.name, "T": T, "H": H, "I": I, "E": E, "top_k": k,
                   "scoring": wl.scoring, "n_group": wl.n_group, "seed": seed,
                   "local_experts": [wl.local_offset, wl.EL], "routed_pairs": P,
                   "tile_rows": moe.moe_tile_rows(cfg), "active_experts": e_active,
                   "max_over_mean_load": round(float(counts.max() / max(counts.mean(), 1e-9)), 2)},
        "tflops": round(tflops, 1), "frac_mfma_peak": round(tflops / PEAK_MFMA_TFLOPS[kind], 4),
        "gbps": round(gbps, 1), "frac_hbm_peak": round(gbps / PEAK_HBM_GBPS, 4),
        "roofline_time_us": round(ideal_us, 1), "frac_of_roofline": round(ideal_us / (ms_per_step * 1e3), 4),
        "gpu_event_us": round(gpu_ms * 1e3, 2), "unmarked_us": round(unmarked_us, 2),
        "single_launch_us": None if single_us is None else round(single_us, 2),
        "graph_replay_us": None if graph_us is None else round(graph_us, 2),
        "step_us": {n_: round(v * 1e3, 2) for n_, v in step_ms.items()},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "parity_sample": parity,
    }


def compact(rec):
    """The nested form of a workload's record: the same measurements in fewer bytes (the whole
    line should stay a few KB).  step_us = [route, sort-scatter, gate/up GEMM, down GEMM, combine];
    gemm_hbm_frac = [gate/up, down] algorithmic bytes / launch time / 8 TB/s; parity = [tokens
    compared, tie-excused tokens, max |err| / max |ref|, sum |err| / sum |ref|, within tolerance]."""
    r = rec["roofline"]
    c = rec["config"]
    out = {"us": rec["value"], "unmarked_us": rec["unmarked_us"], "frac_of_roofline": rec["frac_of_roofline"],
           "dtype": rec["dtype"], "T": c["T"], "pairs": c["routed_pairs"], "active_experts": c["active_experts"],
           "load_max_over_mean": c["max_over_mean_load"], "tflops": rec["tflops"], "frac_mfma": rec["frac_mfma_peak"],
           "gbps": rec["gbps"], "frac_hbm": rec["frac_hbm_peak"],
           "step_us": [rec["step_us"][k] for k in ("route", "permute", "gemm_swiglu", "gemm_down", "combine")],
           "gemm_hbm_frac": [r["frac"], r["down_gemm"]["frac"]]}
    if rec["single_launch_us"] is not None:
        out["single_launch_us"] = rec["single_launch_us"]
    if rec["cpu_baseline"]:
        out["cpu_oracle_us"] = rec["cpu_baseline"]["value"]
        out["cpu_sample"] = rec["cpu_baseline"]["sample"].split(" tokens")[0].replace(" of ", "/") + \
            (" sampled" if "sampled" in rec["cpu_baseline"]["sample"] else " all")
        p = rec["parity_sample"]
        out["parity"] = [p["tokens"], p["tie_excused"], float(f"{p['max_rel']:.3g}"), float(f"{p['mean_rel']:.3g}"), p["ok"]]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=HEADLINE, help="the workload the top level of the line describes")
    ap.add_argument("--only", action="store_true", help="measure the named workload alone (no nested ones)")
    ap.add_argument("--tokens", type=int, default=0,
                    help="override the workload's token count (supplementary points; not a benchmark config; implies --only)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (a kernel of known HBM traffic, used to scale "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--graph", action="store_true",
                    help="supplementary: also time the same forward replayed from a HIP graph (reported as "
                         "graph_replay_us, never as value)")
    ap.add_argument("--cpu-baseline-seconds", type=float, default=12.0,
                    help="CPU work budget per workload for the oracle sample; 0 skips the CPU baseline")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures the single-GPU kernel path only: run with --gpus 1 "
              "(this library has no multi-GPU code; the layer would shard by expert parallelism, one "
              "local-expert call per device plus a reduce-scatter of the partial outputs)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_19128_amd import binding as moe
    from paper_2602_19128_amd import synthetic as syn

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    moe.load()
    dev = torch.device("cuda:0")
    t_start = time.perf_counter()
    log = lambda msg: print(f"[bench {time.perf_counter() - t_start:6.1f}s] {msg}", file=sys.stderr, flush=True)

    if args.copy_calibration:
        src = torch.ones((1 << 28,), dtype=torch.float32, device=dev)          # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    head = syn.WORKLOADS[args.workload]
    only = args.only or args.tokens > 0
    if args.tokens > 0:
        head = head.replace(T=args.tokens, name=f"{head.name}_T{args.tokens}")
    names = [head.name] + ([] if only else [n for n in ALSO if n != head.name])
    todo = {n: (head if n == head.name else syn.WORKLOADS[n]) for n in names}

    # workloads with the same weight shapes share one draw of the weights (they do not depend on T)
    def family(wl):
        return (wl.H, wl.I, wl.E, wl.fp8, wl.local_offset, wl.local_experts)

    records = {}
    done = set()
    for name in names:
        if name in done:
            continue
        group = [n for n in names if n not in done and family(todo[n]) == family(todo[name])]
        base = syn.make_inputs(todo[group[0]], seed=args.seed, device=dev)
        torch.cuda.synchronize()
        log(f"{group}: tensors drawn on the GPU")
        host_base = base.to("cpu") if args.cpu_baseline_seconds > 0 else None
        for n in group:
            wl = todo[n]
            inp = base if n == group[0] else syn.make_inputs(wl, seed=args.seed, device=dev, weights_from=base)
            host = None
            if host_base is not None:
                host = host_base if n == group[0] else syn.MoEInputs(
                    wl, inp.x.cpu(), host_base.router_w, None if inp.bias is None else inp.bias.cpu(), host_base.w1,
                    host_base.w2, None if inp.x_scale is None else inp.x_scale.cpu(), host_base.w1_scale, host_base.w2_scale)
            records[n] = measure(wl, inp, host, args.steps, args.warmup, args.cpu_baseline_seconds,
                                 args.graph, args.seed, log,
                                 min_warm_ms=0.0 if (n == head.name and n == HEADLINE) else 60.0)
            log(f"{n}: {records[n]['value']} us per forward")
            done.add(n)
            del inp, host
        del base, host_base
        torch.cuda.empty_cache()

    rec = records[head.name]
    line = {
        "metric": "fused_moe_forward_latency", "value": rec["value"], "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": rec["ms_per_step"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": rec["dtype"],
        "data": "synthetic",
    }
    for key in ("config", "tflops", "frac_mfma_peak", "gbps", "frac_hbm_peak", "roofline_time_us", "frac_of_roofline",
                "gpu_event_us", "unmarked_us", "single_launch_us", "graph_replay_us", "step_us", "roofline", "cpu_baseline", "parity_sample"):
        line[key] = rec[key]
    if len(names) > 1:
        line["workloads"] = {n: compact(records[n]) for n in names[1:]}
    print(json.dumps(line), flush=True)
    bad = [n for n in names if records[n]["parity_sample"] is not None and not records[n]["parity_sample"]["ok"]]
    if bad:
        print(f"bench.py: GPU output disagrees with the oracle beyond the tolerances on {bad}", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
