#!/usr/bin/env python3
"""Benchmark of the MoE expert-layer forward (one step = one pass of the whole hot path, a1..a8,
over one batch of synthetic tokens already resident in HBM).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mixtral_decode]

Prints ONE JSON line: whole-layer tokens/s, the roofline figure of the dominant kernel (measured
with HIP events recorded on the launch stream at the stage boundaries), and the CPU oracle timed on
this machine's host cores on a bounded sample of the same workload.
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
    cfg = synth.CONFIGS[args.workload]
    t_gen = time.perf_counter()
    L = synth.make_layer(cfg)
    layer = B.device_layer_from_inputs(L)
    X = torch.from_numpy(L.X).to("cuda")
    Y = torch.empty((cfg.T, cfg.H), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    info = B.cq_device_info()

    for _ in range(args.warmup):
        B.cq_moe_forward(layer, X, Y)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        B.cq_moe_forward(layer, X, Y)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    tokens_per_s = cfg.T * args.steps / dt

    # per-stage durations from HIP events recorded on the launch stream at the stage boundaries
    stage = {k: 0.0 for k in B.STAGES}
    n_timed = max(10, min(args.steps, 100))
    for _ in range(n_timed):
        _, ms = B.cq_moe_forward_timed(layer, X, Y)
        for k in stage:
            stage[k] += ms[k] / n_timed

    mid = B.moe_intermediates(layer, cfg.T)
    offs = mid["offsets"].cpu().numpy()
    counts = np.diff(offs)
    active = int((counts > 0).sum())
    rows = int(offs[-1])
    # packed indices + centroid tables (one 32-byte table per row, or per group of group_k weights of a row)
    g = getattr(cfg, "group_k", 0)
    gu_tables, dn_tables = synth.n_blocks(cfg.H, g) or 1, synth.n_blocks(cfg.I, g) or 1
    gu_bytes = active * (2 * cfg.I * cfg.H // 2 + 2 * cfg.I * 32 * gu_tables)
    dn_bytes = active * (cfg.H * cfg.I // 2 + cfg.H * 32 * dn_tables)
    gu_flops = rows * 2.0 * (2 * cfg.I) * cfg.H
    dn_flops = rows * 2.0 * cfg.H * cfg.I
    flop_per_byte = (gu_flops + dn_flops) / (gu_bytes + dn_bytes)
    gu_s = stage["gate_up"] * 1e-3
    dn_s = stage["down"] * 1e-3
    if flop_per_byte < MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBPS * 1e9):
        ach = gu_bytes / gu_s / 1e9
        # (block-wise tables are decoded by the large-tile kernel, at decode sizes by its narrow-tile variant)
        kern = "gemm_narrow_kernel" if g and rows <= 64 else "gemm_large_kernel" if g else "gemm_small_kernel"
        roofline = {"bound": "hbm", "kernel": f"{kern} (gate/up codebook product + SwiGLU)",
                    "achieved": ach, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBPS,
                    "traffic": measured_traffic(cfg.name, kern),
                    "algorithmic_bytes_per_launch": gu_bytes, "avg_launch_ms": stage["gate_up"]}
    else:
        ach = gu_flops / gu_s / 1e12
        roofline = {"bound": "mfma", "kernel": "gemm_large_kernel (gate/up codebook product + SwiGLU)",
                    "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / MFMA_BF16_PEAK_TFLOPS,
                    "traffic": measured_traffic(cfg.name, "gemm_large_kernel"),
                    "algorithmic_flops_per_launch": gu_flops, "avg_launch_ms": stage["gate_up"]}

    # measured streaming-read ceiling next to the nominal peak
    probe = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    probe.random_(0, 255)
    for _ in range(3):
        B.cq_stream_read(probe)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(10):
        B.cq_stream_read(probe)
    torch.cuda.synchronize()
    read_gbps = probe.numel() * 10 / (time.perf_counter() - t0) / 1e9
    # measured dense bf16 MFMA ceiling: bare matrix-core loop, 8 workgroups per CU
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    B.cq_mfma_loop(info["cu_count"] * 8, 200)
    torch.cuda.synchronize()
    e0.record()
    mfma_flops = B.cq_mfma_loop(info["cu_count"] * 8, 2000)
    e1.record()
    torch.cuda.synchronize()
    mfma_tflops = mfma_flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    # a plain copy of known size (1 GiB read + 1 GiB written): the yardstick the HBM counters of a
    # profiled run are scaled by
    dst = torch.empty_like(probe)
    dst.copy_(probe)
    torch.cuda.synchronize()
    del probe, dst

    out = {
        "metric": "MoE-layer tokens/s", "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name} (E={cfg.E} top-{cfg.top_k} S={cfg.S} H={cfg.H} I={cfg.I} T={cfg.T} "
                               f"A{cfg.act_bits}W4, 16 bf16 centroids per "
                               + (f"group of {g} weights of a row (block-wise)" if g else "weight row")
                               + (", Hadamard rotation" if getattr(cfg, "r_hadamard", False) else "")
                               + (f", online Hadamard + A{cfg.h_bits} in front of the down projection)"
                                  if getattr(cfg, "h_bits", 0) else ")"),
                   "active_experts": active, "rows": rows,
                   "max_tokens_per_expert": int(counts.max()), "mean_tokens_per_expert": float(counts.mean())},
        "roofline": roofline,
        "stage_ms": stage,
        "weight_stream": {"gate_up_plus_down_GBps": (gu_bytes + dn_bytes) / (gu_s + dn_s) / 1e9,
                          "frac_of_hbm_peak": (gu_bytes + dn_bytes) / (gu_s + dn_s) / 1e9 / HBM_PEAK_GBPS,
                          "measured_stream_read_GBps": read_gbps},
        "mfma": {"gate_up_plus_down_TFLOPs": (gu_flops + dn_flops) / (gu_s + dn_s) / 1e12,
                 "frac_of_bf16_peak": (gu_flops + dn_flops) / (gu_s + dn_s) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                 "measured_mfma_loop_TFLOPs": mfma_tflops},
        "device": info, "setup_s": t_gen,
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
    print(json.dumps(out))


if __name__ == "__main__":
    main()
