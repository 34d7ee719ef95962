#!/usr/bin/env python3
"""Benchmark of the MoE expert-layer forward (one step = one pass of the whole hot path, a1..a8,
over one batch of synthetic tokens already resident in HBM).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mixtral_decode]

Prints ONE JSON line: whole-layer tokens/s (mean, median and minimum step time), the roofline figure of the
dominant kernel (measured with HIP events recorded on the launch stream at the stage boundaries), the CPU
oracle timed on this machine's host cores on a bounded sample of the same workload and -- for the default
workload, the Mixtral-shaped decode layer -- a nested "prefill" object with the same measurements for the
Mixtral-shaped prefill layer (the matrix-core leg of the metric).
"""
import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16/f16 MFMA, published
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# very script (scaled by what the counters read for the 1 GiB copy below); see profiles/
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def measured_traffic(workload, kernel):
    """Bytes per launch from the committed counter summary ("workload kernel bytes" lines), or None."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 3 and parts[0] == workload and parts[1] == kernel:
                    return int(parts[2])
    except (OSError, ValueError):
        pass
    return None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="mixtral_decode")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget for the oracle's expert sample")
    ap.add_argument("--no-prefill", action="store_true",
                    help="default workload only: skip the Mixtral-shaped prefill leg of the metric")
    ap.add_argument("--prefill-steps", type=int, default=10)
    ap.add_argument("--prefill-warmup", type=int, default=3)
    ap.add_argument("--sweep-tokens", default="",
                    help="comma-separated batch sizes: instead of the benchmark line, print the step time of the "
                         "workload's layer at each of them (its first T tokens; looks for cliffs between the "
                         "decode and the prefill regime)")
    ap.add_argument("--compare-lut", action="store_true",
                    help="A4 workloads: also time the gate/up product in the lookup formulation (product tables)")
    return ap.parse_args()


def cpu_baseline(L, budget_s):
    """The oracle as it stands, on the host cores: the front end on every token, then expert FFNs
    (dense decode + matmul) for as many active experts as fit in the budget, extrapolated by count."""
    from oracle import cq_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    cfg = L.cfg
    t0 = time.perf_counter()
    R = L.R if L.R is not None else O.hadamard_matrix(cfg.H) / math.sqrt(cfg.H)   # Hadamard rotation variant
    XR = O.rotate(L.X, R)
    q, scale = O.quantize(XR, cfg.act_bits)
    logits = O.router_logits(XR, L.Wr, L.bias)
    ids, w = O.route_topk(logits, cfg.top_k)
    offsets, perm, inv = O.permute_by_expert(ids, cfg.E)
    t_front = time.perf_counter() - t0
    a = scale[:, None] * q.astype(np.float64)
    active = [e for e in range(cfg.E) if offsets[e + 1] > offsets[e]] + list(range(cfg.E, cfg.E + cfg.S))
    done, rows_done, t_exp = 0, 0, 0.0
    t1 = time.perf_counter()
    for e in active:
        toks = perm[offsets[e]:offsets[e + 1]] // cfg.top_k if e < cfg.E else np.arange(cfg.T)
        O.expert_ffn(a[toks], L.experts[e], getattr(cfg, "h_bits", 0), getattr(cfg, "group_k", 0))
        done += 1
        rows_done += len(toks)
        t_exp = time.perf_counter() - t1
        if t_exp > budget_s:
            break
    rows_total = cfg.T * (cfg.top_k + cfg.S)
    scale_by = len(active) / done   # per-expert cost (dense decode + matmul), extrapolated by expert count
    est = t_front + t_exp * scale_by
    return {
        "value": cfg.T / est, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
        "sample": f"front end (rotate, quantize, route, permute) on all {cfg.T} tokens in {t_front:.2f}s + "
                  f"expert FFN of {done} of {len(active)} active experts ({rows_done} of {rows_total} rows) in "
                  f"{t_exp:.2f}s, extrapolated x{scale_by:.2f}",
    }


def yardsticks(B, torch, info):
    """Measured ceilings next to the nominal peaks: a streaming read shaped like the product's index stream, the
    bare matrix-core loop, and the plain copy of known size that the HBM counters of a profiled run are scaled by."""
    probe = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    probe.random_(0, 255)
    for _ in range(3):
        B.cq_stream_read(probe)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        B.cq_stream_read(probe)
    e1.record()
    torch.cuda.synchronize()
    read_gbps = probe.numel() * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    B.cq_mfma_loop(info["cu_count"] * 8, 200)
    torch.cuda.synchronize()
    e0.record()
    mfma_flops = B.cq_mfma_loop(info["cu_count"] * 8, 2000)
    e1.record()
    torch.cuda.synchronize()
    mfma_tflops = mfma_flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    dst = torch.empty_like(probe)
    dst.copy_(probe)
    torch.cuda.synchronize()
    del probe, dst
    return read_gbps, mfma_tflops


def prime(B, torch, info, seconds=0.3):
    """Keeps the device busy with the matrix-core yardstick loop for about `seconds`, immediately before the
    warm-up steps: setting up a layer's inputs leaves the GPU idle for seconds, and the first 10-20 ms after
    an idle phase run at the clocks of an idle device (measured: regions of 20 decode steps after 5 warm-up
    steps went 0.184, 0.183, 0.170, 0.168 ms per step without this, 0.156, 0.157, 0.151, 0.153, 0.153 with it;
    priming with the layer itself: 0.152, 0.151, 0.151, 0.151, 0.154).  The timed region is meant to show a
    busy device."""
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        B.cq_mfma_loop(info["cu_count"] * 8, 200)
        torch.cuda.synchronize()


def sweep_tokens(B, torch, synth, info, name, sizes):
    """Step time of the named workload's layer on its first T tokens, for every T in `sizes` (back-to-back steps
    between two host synchronisations, stage times from the event-timed entry point)."""
    cfg = synth.CONFIGS[name]
    L = synth.make_layer(cfg)
    layer = B.device_layer_from_inputs(L)
    Xall = torch.from_numpy(L.X).to("cuda")
    prime(B, torch, info)
    rows = []
    for T in sizes:
        T = min(int(T), cfg.T)
        X = Xall[:T].contiguous()
        Y = torch.empty((T, cfg.H), dtype=torch.float32, device="cuda")
        for _ in range(10):
            B.cq_moe_forward(layer, X, Y)
        torch.cuda.synchronize()
        n = 100 if T <= 512 else 20
        t0 = time.perf_counter()
        for _ in range(n):
            B.cq_moe_forward(layer, X, Y)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / n
        acc = np.zeros(len(B.STAGES))
        for _ in range(20):
            _, ms = B.cq_moe_forward_timed(layer, X, Y)
            acc += [ms[k] for k in B.STAGES]
        rows.append({"tokens": T, "us_per_layer": dt * 1e6, "tokens_per_s": T / dt,
                     "stage_us": dict(zip(B.STAGES, (acc / 20 * 1e3).tolist()))})
    return rows


def measure(B, torch, synth, info, name, steps, warmup, n_stage):
    """W warm-up steps, exactly K timed steps of cq_moe_forward (inputs resident in HBM), then n_stage runs of
    the same launches with events at the stage boundaries.  Returns (result dict, layer inputs)."""
    cfg = synth.CONFIGS[name]
    t_gen = time.perf_counter()
    L = synth.make_layer(cfg)
    layer = B.device_layer_from_inputs(L)
    X = torch.from_numpy(L.X).to("cuda")
    Y = torch.empty((cfg.T, cfg.H), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    prime(B, torch, info)
    for _ in range(warmup):
        B.cq_moe_forward(layer, X, Y)
    torch.cuda.synchronize()

    def region():
        """K steps enqueued back to back, a host synchronisation on both sides; seconds by the host clock."""
        t0 = time.perf_counter()
        for _ in range(steps):
            B.cq_moe_forward(layer, X, Y)
        torch.cuda.synchronize()
        return time.perf_counter() - t0
    dt = region()                                   # THE timed region: exactly K steps, nothing else in it
    # four more regions of K steps, for the spread only (an event per step would put a marker packet and
    # its few microseconds between every two steps of a 0.15 ms layer)
    per_step = np.array([dt] + [region() for _ in range(4)]) / steps * 1e3

    acc = np.zeros((n_stage, len(B.STAGES)))
    for i in range(n_stage):
        _, ms = B.cq_moe_forward_timed(layer, X, Y)
        acc[i] = [ms[k] for k in B.STAGES]
    stage = dict(zip(B.STAGES, acc.mean(axis=0).tolist()))
    stage_median = dict(zip(B.STAGES, np.median(acc, axis=0).tolist()))
    stage_min = dict(zip(B.STAGES, acc.min(axis=0).tolist()))

    mid = B.moe_intermediates(layer, cfg.T)
    offs = mid["offsets"].cpu().numpy()
    counts = np.diff(offs)
    active = int((counts > 0).sum())
    rows = int(offs[-1])
    # packed indices + centroid tables (one 32-byte table per row, or per group of group_k weights of a row)
    g = getattr(cfg, "group_k", 0)
    gu_tables, dn_tables = synth.n_blocks(cfg.H, g) or 1, synth.n_blocks(cfg.I, g) or 1
    bits = getattr(cfg, "index_bits", 4)              # index bits per weight; a table has 2^bits bf16 entries
    gu_bytes = active * (2 * cfg.I * cfg.H * bits // 8 + 2 * cfg.I * (2 << bits) * gu_tables)
    dn_bytes = active * (cfg.H * cfg.I * bits // 8 + cfg.H * (2 << bits) * dn_tables)
    gu_flops = rows * 2.0 * (2 * cfg.I) * cfg.H
    dn_flops = rows * 2.0 * cfg.H * cfg.I
    flop_per_byte = (gu_flops + dn_flops) / (gu_bytes + dn_bytes)
    gu_s, dn_s = stage["gate_up"] * 1e-3, stage["down"] * 1e-3
    gu_med, dn_med = stage_median["gate_up"] * 1e-3, stage_median["down"] * 1e-3
    hbm_bound = flop_per_byte < MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBPS * 1e9)
    if hbm_bound:
        ach = gu_bytes / gu_s / 1e9
        # (block-wise tables are decoded by the large-tile kernel, at decode sizes by its narrow-tile variant)
        # (block-wise tables: tables of 1024 weights at decode sizes run on the streaming kernel, other block-wise
        # products on the large-tile kernel or, with at most 64 rows in all, its narrow-tile variant)
        kern = ("gemm_w2_kernel" if bits == 2 else "gemm_small_kernel" if not g or (g == 1024 and cfg.T <= 16)
                else "gemm_narrow_kernel" if rows <= 64 else "gemm_large_kernel")
        roofline = {"bound": "hbm", "kernel": f"{kern} (gate/up codebook product + SwiGLU)",
                    "achieved": ach, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBPS,
                    "frac_at_median_duration": gu_bytes / gu_med / 1e9 / HBM_PEAK_GBPS,
                    "algorithmic_bytes_per_launch": gu_bytes}
    else:
        ach = gu_flops / gu_s / 1e12
        kern = "gemm_large_kernel"
        roofline = {"bound": "mfma", "kernel": "gemm_large_kernel (gate/up codebook product + SwiGLU)",
                    "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / MFMA_BF16_PEAK_TFLOPS,
                    "frac_at_median_duration": gu_flops / gu_med / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                    "algorithmic_flops_per_launch": gu_flops}
    traffic = measured_traffic(cfg.name, kern)
    roofline.update({"avg_launch_ms": stage["gate_up"], "median_launch_ms": stage_median["gate_up"],
                     "launches_timed": n_stage, "traffic": traffic,
                     "traffic_source": (f"profiles/hbm_traffic.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                        f"script, per launch of {kern}" if traffic else None)})
    res = {
        "tokens_per_s": cfg.T * steps / dt, "ms_per_step": dt / steps * 1e3,
        "ms_per_step_median": float(np.median(per_step)), "ms_per_step_min": float(per_step.min()),
        "ms_per_step_regions": [float(v) for v in per_step],
        "steps": steps, "warmup": warmup,
        "config": {"workload": f"{cfg.name} (E={cfg.E} top-{cfg.top_k} S={cfg.S} H={cfg.H} I={cfg.I} T={cfg.T} "
                               f"A{cfg.act_bits}W{bits}, {1 << bits} bf16 centroids per "
                               + (f"group of {g} weights of a row (block-wise)" if g else "weight row")
                               + (", Hadamard rotation" if getattr(cfg, "r_hadamard", False) else "")
                               + (f", online Hadamard + A{cfg.h_bits} in front of the down projection)"
                                  if getattr(cfg, "h_bits", 0) else ")"),
                   "active_experts": active, "rows": rows,
                   "max_tokens_per_expert": int(counts.max()), "mean_tokens_per_expert": float(counts.mean())},
        "roofline": roofline,
        "stage_ms": stage, "stage_ms_median": stage_median, "stage_ms_min": stage_min,
        "weight_stream": {"gate_up_plus_down_GBps": (gu_bytes + dn_bytes) / (gu_s + dn_s) / 1e9,
                          "frac_of_hbm_peak": (gu_bytes + dn_bytes) / (gu_s + dn_s) / 1e9 / HBM_PEAK_GBPS,
                          "down_frac_of_hbm_peak": dn_bytes / dn_s / 1e9 / HBM_PEAK_GBPS},
        "mfma": {"gate_up_plus_down_TFLOPs": (gu_flops + dn_flops) / (gu_s + dn_s) / 1e12,
                 "frac_of_bf16_peak": (gu_flops + dn_flops) / (gu_s + dn_s) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                 "down_frac_of_bf16_peak": dn_flops / dn_s / 1e12 / MFMA_BF16_PEAK_TFLOPS},
        "setup_s": t_gen,
    }
    return res, L, layer, X, Y, mid, rows


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2604_10496_amd import binding as B
    from paper_2604_10496_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs the MI355X: no GPU visible and there is no CPU path", file=sys.stderr)
        sys.exit(3)
    B.load_library()
    torch.cuda.set_device(0)
    info = B.cq_device_info()
    if args.sweep_tokens:
        sizes = [int(v) for v in args.sweep_tokens.split(",") if v.strip()]
        print(json.dumps({"workload": args.workload, "sweep": sweep_tokens(B, torch, synth, info, args.workload, sizes)}))
        return
    read_gbps, mfma_tflops = yardsticks(B, torch, info)

    n_stage = 100 if synth.CONFIGS[args.workload].T <= 1024 else 20
    res, L, layer, X, Y, mid, rows = measure(B, torch, synth, info, args.workload, args.steps, args.warmup, n_stage)
    cfg = L.cfg
    out = {
        "metric": "MoE-layer tokens/s", "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "ms_per_step_median": res["ms_per_step_median"], "ms_per_step_min": res["ms_per_step_min"],
        "ms_per_step_regions": res["ms_per_step_regions"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": res["config"], "roofline": res["roofline"],
        "stage_ms": res["stage_ms"], "stage_ms_median": res["stage_ms_median"], "stage_ms_min": res["stage_ms_min"],
        "weight_stream": dict(res["weight_stream"], measured_stream_read_GBps=read_gbps),
        "mfma": dict(res["mfma"], measured_mfma_loop_TFLOPs=mfma_tflops),
        # (clocks are as found: an ordinary user cannot pin them, and nothing is spawned to read them -- the
        # measured matrix-core loop and streaming read above are the yardsticks for the state of the box)
        "device": info, "setup_s": res["setup_s"],
    }
    if args.compare_lut and cfg.act_bits == 4 and not getattr(cfg, "h_bits", 0):
        # the gate/up product of this step's sorted rows, once on the matrix cores and once by table lookup
        def timed(fn, n):
            fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(n):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / n
        argsg = (mid["scale"], mid["src_token"], mid["offsets"], rows, B.CQ_EPI_SWIGLU, B.CQ_OUT_F32)
        n_rep = 20 if rows <= 256 else 2
        mm = timed(lambda: B.cq_codebook_grouped_gemm(layer.gate_up, mid["Q"], B.CQ_A_INT8_CODES, *argsg), n_rep)
        lut_out = B.cq_codebook_grouped_gemm_lut(layer.gate_up, mid["Q"], *argsg)
        lut = timed(lambda: B.cq_codebook_grouped_gemm_lut(layer.gate_up, mid["Q"], *argsg, out=lut_out), n_rep)
        out["lut_comparison"] = {"stage": "gate/up product + SwiGLU on int8-held 4-bit codes", "rows": rows,
                                 "matrix_core_ms": mm, "lookup_ms": lut, "lookup_over_matrix_core": lut / mm}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(L, args.cpu_seconds)
    del layer, X, Y, mid, L
    torch.cuda.empty_cache()
    if args.workload == "mixtral_decode" and not args.no_prefill:
        # the third leg of the metric: matrix-core utilisation of the Mixtral-shaped prefill layer (T = 4096, A4)
        pre, _, _, _, _, _, _ = measure(B, torch, synth, info, "mixtral_prefill", args.prefill_steps, args.prefill_warmup, 10)
        out["prefill"] = {k: pre[k] for k in ("tokens_per_s", "ms_per_step", "ms_per_step_median", "ms_per_step_min", "ms_per_step_regions",
                                              "steps", "warmup", "config", "roofline", "stage_ms", "stage_ms_median",
                                              "mfma", "setup_s")}
        out["prefill"]["mfma"]["measured_mfma_loop_TFLOPs"] = mfma_tflops
    print(json.dumps(out))


if __name__ == "__main__":
    main()
