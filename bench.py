#!/usr/bin/env python3
"""Benchmark of the one-GPU MoE-layer forward (libmoe) on MI355X.

A step is one pass of the whole hot path -- gate, dispatch plan, pack, expert FFN,
combine -- over one batch of seeded synthetic tokens, through moe_layer_chunked.
Inputs and packed weights are resident in HBM before the timed region.  Prints one
JSON line: layer tokens/s, the roofline position of the dominant kernel (first
expert GEMM, timed with HIP events on its own stream during the timed steps), and
the CPU oracle's rate on the same workload as a baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16/fp16 MFMA
PEAK_HBM_GBPS = 8000.0        # MI355X HBM3E


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="gpt2s_moe",
                    help="one of workloads.CONFIGS (default: the configuration the metric is quoted on)")
    ap.add_argument("--chunks", type=int, default=1, help="n_chunks of moe_layer_chunked")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stages", action="store_true",
                    help="after the timed region, run extra steps with every stage timed")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2210_17223_amd as moe
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = wl.CONFIGS[args.workload]
    if cfg["layers"] != 1:
        print("bench.py: stack workloads are benchmarked layer by layer; pick a one-layer workload",
              file=sys.stderr)
        return 2
    li = wl.make_layer(cfg, seed=0, threads=16)
    s = moe.Shape.make(li.T, li.d, li.E, li.h, li.k, li.C,
                       dtype="bf16" if li.dtype == "bf16" else "f32", act="gelu")

    def up(a):
        if li.dtype == "bf16":
            bits = wl.bf16_bits(a).view(np.int16).reshape(a.shape)
            return torch.from_numpy(bits).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    x, Wg = up(li.x), up(li.Wg)
    bias = None if li.gate_bias is None else torch.from_numpy(li.gate_bias).to(dev)
    b = moe.alloc_buffers(s, args.chunks, dev)
    moe.moe_pack_gate(s, Wg, b["Wgp"])
    W1, W2 = up(li.W1), up(li.W2)
    moe.moe_pack_weights(s, W1, W2, b["W1p"], b["W2p"])
    torch.cuda.synchronize()
    del W1, W2

    def step():
        moe.moe_layer_chunked(s, args.chunks, x, b["Wgp"], bias, li.bias_token_stride,
                              b["W1p"], None, b["W2p"], None, b["expert_idx"], b["gate"],
                              b["counts"], b["offsets"], b["slot_of"], b["src_of"], b["xe"],
                              b["ye"], b["y"], None, b["workspace"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    G1 = moe.STAGES.index("gemm1")
    moe.moe_profile_enable(1 << G1, args.steps * args.chunks)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    g1_ms = np.array(moe.moe_profile_read(G1, args.steps * args.chunks))
    moe.moe_profile_enable(0, 0)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = li.T / (ms_per_step * 1e-3)
    A = int(b["offsets"].cpu().numpy()[-1])
    counts = b["counts"].cpu().numpy()
    # first expert GEMM: 2*A*d*h flops per layer; one launch per chunk
    g1_avg_ms = float(g1_ms.mean())
    g1_flops_per_launch = 2.0 * A * li.d * li.h / args.chunks
    g1_tflops = g1_flops_per_launch / (g1_avg_ms * 1e-3) / 1e12
    out = {
        "metric": "moe_layer_tokens_per_s", "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if li.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: T={li.T} d_model={li.d} E={li.E} d_ff={li.h} "
                               f"k={li.k} capacity={li.C} {li.dtype}, seed 0",
                   "n_chunks": args.chunks, "kept_rows_A": A,
                   "dropped_assignments": int(li.T * li.k - A),
                   "count_min": int(counts.min()), "count_max": int(counts.max())},
        "roofline": {"bound": "mfma", "kernel": "grouped_gemm_mfma_kernel<bf16 in, fp16 out, GeLU> (first expert GEMM)",
                     "achieved": g1_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": g1_tflops / PEAK_BF16_TFLOPS, "traffic": None,
                     "avg_launch_us": g1_avg_ms * 1e3, "launches": int(g1_ms.size)},
    }

    if args.stages:
        n = min(args.steps, 50)
        moe.moe_profile_enable((1 << len(moe.STAGES)) - 1, n * args.chunks)
        for _ in range(n):
            step()
        torch.cuda.synchronize()
        st = {}
        for i, name in enumerate(moe.STAGES):
            v = np.array(moe.moe_profile_read(i, n * args.chunks))
            st[name] = float(v.sum() / n * 1e3) if v.size else None     # us per layer
        moe.moe_profile_enable(0, 0)
        esz = 2 if li.dtype == "bf16" else 4
        kept_tokens = int((b["slot_of"].view(li.T, li.k) >= 0).any(1).sum().item())
        disp_bytes = (kept_tokens + A) * li.d * esz            # read routed tokens, write slots
        comb_bytes = (A + li.T) * li.d * 4                     # fp32 expert rows in, fp32 y out
        st["dispatch_GBps"] = disp_bytes / (st["scatter"] * 1e-6) / 1e9
        st["combine_GBps"] = comb_bytes / (st["combine"] * 1e-6) / 1e9
        st["dispatch_combine_frac_of_hbm_peak"] = ((disp_bytes + comb_bytes) /
                                                   ((st["scatter"] + st["combine"]) * 1e-6) / 1e9 / PEAK_HBM_GBPS)
        st["ffn_mfma_util"] = (4.0 * A * li.d * li.h) / ((st["gemm1"] + st["gemm2"]) * 1e-6) / 1e12 / PEAK_BF16_TFLOPS
        out["stages_us"] = st

    if not args.no_cpu_baseline:
        import oracle
        # Bounded sample: whole passes of the oracle over the workload (gate and plan over
        # all tokens; expert FFN and combine for a leading slice of tokens when one full
        # pass would take minutes), repeated until about 20 core-seconds have been spent.
        sample = li.T
        est_flops = 4.0 * li.T * li.k * li.d * li.h
        if est_flops > 4e11:
            sample = max(64, int(li.T * 4e11 / est_flops))
        toks = np.arange(sample, dtype=np.int32)
        cores = oracle.threads()
        passes, c0 = 0, time.perf_counter()
        while True:
            oracle.moe_layer(li.x, li.Wg, li.W1, li.W2, k=li.k, capacity=li.C, bias=li.gate_bias,
                             bias_stride=li.bias_token_stride,
                             tokens=None if sample == li.T else toks)
            passes += 1
            elapsed = time.perf_counter() - c0
            if elapsed * cores >= 20.0 or passes >= 50:
                break
        out["cpu_baseline"] = {"value": sample * passes / elapsed, "unit": "tokens/s",
                               "cores": cores, "kind": "oracle",
                               "sample": f"{passes} pass(es): gate+plan over all {li.T} tokens, expert "
                                         f"FFN+combine for the first {sample} tokens, {elapsed:.2f} s wall"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
