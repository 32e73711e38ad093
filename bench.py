#!/usr/bin/env python3
"""Benchmark of the one-GPU MoE-layer forward (libmoe) on MI355X.

A step is one pass of the whole hot path -- gate, dispatch plan, pack, expert FFN,
combine -- over one batch of seeded synthetic tokens, through moe_layer_chunked (for
the 4-layer inference workload: the four layers back to back, each reading the
previous layer's output).  Inputs and packed weights are resident in HBM before the
timed region.  The default workload is the largest single-GPU configuration
(large_chunked: T=32768, d_model=2048, E=64, d_ff=8192, top-2), unchunked.  Prints one
JSON line: layer tokens/s, the roofline position of the dominant kernel (first expert
GEMM, timed with HIP events attached to its own dispatches during the timed steps), the
metric's two other quantities (dispatch+combine HBM rate, expert-FFN matrix-core
utilisation, from stage-timed steps after the timed region), and the CPU oracle's rate
on a bounded sample of the same workload as a baseline.
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
INFINITY_CACHE_BYTES = 256 << 20

# HBM bytes per launch of the first expert GEMM, from rocprofv3 --pmc FETCH_SIZE and
# --pmc WRITE_SIZE runs of this script (readings, scale factors and commands: profiles/).
# The counters cannot be read from inside the process, so the figure is a stored
# measurement, reported only for the workload and launch configuration it was taken on
# (null for any other): {(workload, n_chunks): (FETCH_SIZE KiB, WRITE_SIZE KiB)} per launch.
GEMM1_TRAFFIC_KIB = {("large_chunked", 1): (1559144.2, 1017952.0),     # profiles/layer_hbm_traffic_pmc.txt
                     ("gpt2s_moe", 1): (69506.5, 50068.6)}
FETCH_UNIT, WRITE_UNIT = 2.0, 1.0     # what the plain-copy calibration reads per counted KiB


def gemm1_traffic_bytes(workload, chunks):
    kib = GEMM1_TRAFFIC_KIB.get((workload, chunks))
    return None if kib is None else (kib[0] * FETCH_UNIT + kib[1] * WRITE_UNIT) * 1024.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="large_chunked",
                    help="one of workloads.CONFIGS (default: the largest single-GPU configuration), "
                         "or 'popularity': the inference scheduler's estimate + two-phase decision")
    ap.add_argument("--chunks", type=int, default=1, help="n_chunks of moe_layer_chunked")
    ap.add_argument("--group-rows", type=int, default=0,
                    help="with --chunks > 1: rows per expert an FFN launch must hold on average "
                         "(moe_tune_ffn_group_rows; 0 = the library's default, 1 = one FFN launch per chunk)")
    ap.add_argument("--four-calls", action="store_true",
                    help="a step is the four entry points one after the other on one stream "
                         "(moe_route, moe_dispatch, moe_expert_ffn, moe_combine) instead of moe_layer_chunked: "
                         "the expert FFN then reads the packed buffer and nothing overlaps")
    ap.add_argument("--comm", action="store_true",
                    help="the workload's layer in the padded equal-split layout with both all-to-alls "
                         "on the stand-in link (moe_layer_padded), alone and while a gradient "
                         "allreduce competes for the link under both scheduling policies")
    ap.add_argument("--link-blocks", type=int, default=32,
                    help="workgroups of the stand-in link's copy kernel (its rate)")
    ap.add_argument("--micro-mib", type=int, default=16,
                    help="with --comm: size of an allreduce micro-op in MiB")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a HIP graph (reported beside the eager figure)")
    ap.add_argument("--stages", action="store_true",
                    help="also print the per-stage times (mean, median, min) of the stage-timed steps "
                         "that follow the timed region (their summary figures are always printed)")
    ap.add_argument("--cold-sets", type=int, default=4,
                    help="after the timed region, time the same steps rotating through this many "
                         "copies of every buffer, so that no step finds its data in the 256 MB "
                         "Infinity Cache (skipped when one copy alone exceeds the cache; 0 = off)")
    ap.add_argument("--backward", action="store_true",
                    help="a step is forward + backward of the layer (moe_layer_backward); the roofline "
                         "object is then for the second layer's weight-gradient GEMM")
    ap.add_argument("--recompute", action="store_true",
                    help="with --backward: the forward is the plain layer call and the backward pass "
                         "computes the first GEMM again (default: moe_layer_forward_keep keeps it)")
    ap.add_argument("--offload", type=int, default=0, metavar="R",
                    help="expert weights stay in (pinned) host memory and stream through R device "
                         "slots (moe_expert_ffn_offloaded); the step is gate, dispatch, that FFN and "
                         "combine; a stack workload contributes its first layer")
    ap.add_argument("--calibrate", action="store_true",
                    help="measure the two roofs and exit: the library's plain copy kernel over 1 GiB "
                         "(HBM GB/s, read + write; under rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE its "
                         "reading fixes the counters' unit) and its register-resident MFMA loop with "
                         "constant and with random operands (TFLOP/s)")
    ap.add_argument("--gemm-ablation", action="store_true",
                    help="time the 256 x 256 expert-GEMM kernel alone on the large layer's two GEMM shapes "
                         "(64 experts of 1024 rows), whole and with parts left out (moe_calib_gemm), on random "
                         "and on all-ones operands, and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        return 2
    if args.calibrate:
        return calibrate()
    if args.gemm_ablation:
        return gemm_ablation()
    import numpy as np
    import torch

    import paper_2210_17223_amd as moe
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.workload == "popularity":
        return bench_popularity(args, moe, np, torch, dev)
    if args.comm:
        return bench_comm(args, moe, wl, np, torch, dev)
    if args.group_rows > 0:
        moe.moe_tune_ffn_group_rows(args.group_rows)
    cfg = wl.CONFIGS[args.workload]
    n_layers = cfg["layers"]
    host = wl.make_stack(cfg, seed=0, threads=16) if n_layers > 1 else [wl.make_layer(cfg, seed=0, threads=16)]
    if args.offload:
        host, n_layers = host[:1], 1
    l0 = host[0]
    bf16 = l0.dtype == "bf16"
    s = moe.Shape.make(l0.T, l0.d, l0.E, l0.h, l0.k, l0.C, dtype="bf16" if bf16 else "f32", act="gelu")
    esz = 2 if bf16 else 4

    def up(a):
        if bf16:
            bits = wl.bf16_bits(a).view(np.int16).reshape(a.shape)
            return torch.from_numpy(bits).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    class DevLayer:
        """One layer's device buffers; `x` is None for the later layers of a stack."""

        def __init__(self, li=None, like=None):
            self.b = moe.alloc_buffers(s, args.chunks, dev, y_act=n_layers > 1)
            if like is None:
                self.x = up(li.x) if li.x.shape[0] else None
                self.bias = None if li.gate_bias is None else torch.from_numpy(li.gate_bias).to(dev)
                self.stride = li.bias_token_stride
                moe.moe_pack_gate(s, up(li.Wg), self.b["Wgp"])
                W1, W2 = up(li.W1), up(li.W2)
                moe.moe_pack_weights(s, W1, W2, self.b["W1p"], self.b["W2p"])
                torch.cuda.synchronize()
                if args.offload:
                    self.W1h, self.W2h = self.b["W1p"].cpu().pin_memory(), self.b["W2p"].cpu().pin_memory()
                    self.staging = torch.empty(moe.moe_offload_staging_bytes(s, args.offload),
                                               dtype=torch.uint8, device=dev)
                    self.ows = torch.empty(moe.moe_offload_workspace_bytes(s), dtype=torch.uint8, device=dev)
                if args.backward:
                    self.W1, self.W2 = W1, W2
                    f32 = lambda n: torch.empty(n, dtype=torch.float32, device=dev)
                    self.dy = torch.randn(l0.T * l0.d, dtype=torch.float32, device=dev)
                    self.g = [f32(l0.T * l0.d), f32(l0.d * l0.E), f32(l0.E * l0.d * l0.h),
                              f32(l0.E * l0.d * l0.h), f32(l0.T * l0.k)]
                    self.bws = torch.empty(moe.moe_backward_workspace_bytes(s), dtype=torch.uint8, device=dev)
                    self.pre = None if args.recompute else torch.empty(
                        moe.moe_max_rows(s) * l0.h, dtype=torch.float16, device=dev)
                    self.hid = None if args.recompute else torch.empty_like(self.pre)
            else:       # a second copy of the same layer at other addresses
                self.x = None if like.x is None else like.x.clone()
                self.bias = None if like.bias is None else like.bias.clone()
                self.stride = like.stride
                for name in ("Wgp", "W1p", "W2p"):
                    self.b[name].copy_(like.b[name])

        def bytes(self):
            n = sum(t.numel() * t.element_size() for t in self.b.values() if t is not None)
            return n + (0 if self.x is None else self.x.numel() * esz)

        def run(self, x):
            b = self.b
            if args.offload:
                moe.moe_route(s, x, b["Wgp"], self.bias, self.stride, b["expert_idx"], b["gate"])
                moe.moe_dispatch(s, x, b["expert_idx"], b["counts"], b["offsets"], b["slot_of"],
                                 b["src_of"], b["xe"], b["workspace"])
                moe.moe_expert_ffn_offloaded(s, b["xe"], b["offsets"], self.W1h, self.W2h, None, None,
                                             b["ye"], self.staging, args.offload, self.ows)
                moe.moe_combine(s, b["ye"], b["slot_of"], b["gate"], b["y"], b["y_act"])
                return
            if args.four_calls:
                moe.moe_route(s, x, b["Wgp"], self.bias, self.stride, b["expert_idx"], b["gate"])
                moe.moe_dispatch(s, x, b["expert_idx"], b["counts"], b["offsets"], b["slot_of"],
                                 b["src_of"], b["xe"], b["workspace"])
                moe.moe_expert_ffn(s, b["xe"], b["offsets"], b["W1p"], None, b["W2p"], None, b["ye"],
                                   b["workspace"])
                moe.moe_combine(s, b["ye"], b["slot_of"], b["gate"], b["y"], b["y_act"])
                return
            if args.backward and self.pre is not None:
                moe.moe_layer_forward_keep(s, x, b["Wgp"], self.bias, self.stride, b["W1p"], None, b["W2p"],
                                           None, b["expert_idx"], b["gate"], b["counts"], b["offsets"],
                                           b["slot_of"], b["src_of"], b["xe"], b["ye"], self.pre, self.hid, b["y"],
                                           b["workspace"])
            else:
                moe.moe_layer_chunked(s, args.chunks, x, b["Wgp"], self.bias, self.stride, b["W1p"], None,
                                      b["W2p"], None, b["expert_idx"], b["gate"], b["counts"], b["offsets"],
                                      b["slot_of"], b["src_of"], b["xe"], b["ye"], b["y"], b["y_act"],
                                      b["workspace"])
            if args.backward:
                moe.moe_layer_backward(s, x, b["Wgp"], self.bias, self.stride, self.W1, self.W2, b["W1p"],
                                       b["expert_idx"], b["gate"], b["offsets"], b["slot_of"], b["src_of"],
                                       b["xe"], b["ye"], self.pre, self.hid, self.dy, *self.g, self.bws)

    sets = [[DevLayer(li) for li in host]]
    for li in host:       # the host copies of the weights are needed again only by the oracle
        if args.no_cpu_baseline:
            li.W1 = li.W2 = None

    def step(layers):
        x = layers[0].x
        for L in layers:
            L.run(x)
            x = L.b["y_act"]

    def timed(n, which):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            step(sets[which(i)])
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    launches = args.steps * args.chunks * n_layers
    for _ in range(args.warmup):
        step(sets[0])
    if args.offload and (args.backward or args.chunks != 1 or not bf16):
        print("bench.py: --offload takes a bf16 workload, --chunks 1, no --backward", file=sys.stderr)
        return 2
    if args.backward and (n_layers != 1 or args.chunks != 1 or not bf16):
        print("bench.py: --backward takes a one-layer bf16 workload and --chunks 1", file=sys.stderr)
        return 2
    G1 = moe.STAGES.index("bwd_wgrad2" if args.backward else "gemm1")
    torch.cuda.synchronize()
    moe.moe_profile_enable(1 << G1, launches)
    ms_per_step = timed(args.steps, lambda i: 0)
    g1_ms = np.array(moe.moe_profile_read(G1, launches))
    moe.moe_profile_enable(0, 0)

    tokens_per_s = l0.T / (ms_per_step * 1e-3)
    offs = [L.b["offsets"].cpu().numpy() for L in sets[0]]
    cnts = [L.b["counts"].cpu().numpy() for L in sets[0]]
    A = float(np.mean([o[-1] for o in offs]))                               # kept rows per layer
    live = float(np.mean([(np.diff(o) > 0).sum() for o in offs]))           # experts with rows
    # first expert GEMM, per launch (one launch per chunk and layer): 2*A*d*h flops; reads the
    # packed rows and the weights of the experts that have rows, writes the hidden rows
    g1_avg_ms = float(g1_ms.mean())
    g1_flops = 2.0 * A * l0.d * l0.h / args.chunks
    g1_bytes = (A * l0.d * 2 + A * l0.h * 2) / args.chunks + live * l0.d * l0.h * 2
    g1_tflops = g1_flops / (g1_avg_ms * 1e-3) / 1e12
    g1_gbps = g1_bytes / (g1_avg_ms * 1e-3) / 1e9
    # Which roof bounds the expert FFN at this shape: its 4*A*d*h flops on the matrix cores
    # against streaming the live experts' weights and the packed rows once from HBM.
    ffn_mfma_s = 4.0 * A * l0.d * l0.h / (PEAK_BF16_TFLOPS * 1e12)
    ffn_hbm_s = (2 * live * l0.d * l0.h * 2 + A * l0.d * (2 + 4)) / (PEAK_HBM_GBPS * 1e9)
    hbm_bound = ffn_hbm_s > ffn_mfma_s
    if args.backward:
        # dW2[e] = act(P)^T dye: reads both operands once, writes fp32 dW2
        g1_bytes = A * l0.h * 2 + A * l0.d * 2 + l0.E * l0.d * l0.h * 4
        g1_gbps = g1_bytes / (g1_avg_ms * 1e-3) / 1e9
    roof = {"kernel": ("weight-gradient GEMM dW2 = act(P)^T dye (wgrad_w4_kernel where 256 x 256 tiles fill the chip, else wgrad_gemm_kernel)" if args.backward else
                       moe.moe_expert_gemm_kernel(s, 0) + " <bf16 in, fp16 out, GeLU> (first expert GEMM)"
                       if bf16 else "grouped_gemm_f32_kernel (first expert GEMM)"),
            "avg_launch_us": g1_avg_ms * 1e3, "launches": int(g1_ms.size),
            "algorithmic_flops": g1_flops, "algorithmic_bytes": g1_bytes,
            "traffic": None if args.backward else gemm1_traffic_bytes(args.workload, args.chunks),
            "mfma_tflops": g1_tflops, "hbm_gbps": g1_gbps}
    if hbm_bound:
        roof.update({"bound": "hbm", "achieved": g1_gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                     "frac": g1_gbps / PEAK_HBM_GBPS})
    else:
        roof.update({"bound": "mfma", "achieved": g1_tflops, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": g1_tflops / PEAK_BF16_TFLOPS})
    if args.offload:
        # the step is bound by the host link: every expert's packed weights cross it once
        link_bytes = 2.0 * l0.E * l0.d * l0.h * 2
        roof = {"bound": "hbm", "kernel": "host-to-device copies of the expert weights (copy engine)",
                "note": "bound by the host link, not by HBM: 'peak' is PCIe 5.0 x16, 64 GB/s per direction",
                "achieved": link_bytes / (ms_per_step * 1e-3) / 1e9, "peak": 64.0, "unit": "GB/s",
                "frac": link_bytes / (ms_per_step * 1e-3) / 1e9 / 64.0, "traffic": None,
                "algorithmic_bytes": link_bytes, "resident_slots": args.offload,
                "first_gemm_avg_launch_us": g1_avg_ms * 1e3}
    if not bf16:
        roof = {"bound": "alu", "note": "fp32 correctness configuration: launch-bound, no roofline claimed",
                "achieved": None, "peak": None, "unit": None, "frac": None, "traffic": None,
                "avg_launch_us": g1_avg_ms * 1e3}
    out = {
        "metric": ("moe_layer_fwd_bwd_tokens_per_s" if args.backward else
                   "moe_layer_offloaded_tokens_per_s" if args.offload else "moe_layer_tokens_per_s"),
        "value": tokens_per_s * n_layers, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("bf16 (x, Wg, W1, xe bf16; hidden activations and W2 fp16; fp32 accumulate; "
                  "gate fp32; expert output ye fp16; y fp32)") if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: T={l0.T} d_model={l0.d} E={l0.E} d_ff={l0.h} "
                               f"k={l0.k} capacity={l0.C} {l0.dtype}, seed 0"
                               + (f", {n_layers} layers back to back (value counts layer-tokens)" if n_layers > 1 else ""),
                   "n_chunks": args.chunks, "ffn_group_rows": moe.moe_tune_ffn_group_rows(0), "kept_rows_A": A,
                   "dropped_assignments": float(l0.T * l0.k - A),
                   "count_min": int(min(c.min() for c in cnts)), "count_max": int(max(c.max() for c in cnts))},
        "roofline": roof,
    }

    # ---- the same steps replayed from a HIP graph (launch overhead off the host) -----------
    if args.graph and not args.offload:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(sets[0])
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        out["graph_replay"] = {"ms_per_step": g_ms, "value": l0.T * n_layers / (g_ms * 1e-3), "unit": "tokens/s",
                               "note": "one step captured into a HIP graph and replayed; outputs are "
                                       "bit-identical to the eager call (tests/test_gpu_graph.py)"}

    # ---- the same steps with cold caches -------------------------------------------------
    set_bytes = sum(L.bytes() for L in sets[0])
    if (args.cold_sets > 1 and n_layers == 1 and set_bytes <= 4 * INFINITY_CACHE_BYTES
            and not args.backward and not args.offload):
        while len(sets) < args.cold_sets:
            sets.append([DevLayer(like=L) for L in sets[0]])
        n = len(sets)
        for i in range(n):
            step(sets[i])
        cold_ms = timed(args.steps, lambda i: i % n)
        out["cold_cache"] = {"ms_per_step": cold_ms, "value": l0.T / (cold_ms * 1e-3), "unit": "tokens/s",
                             "sets": n, "bytes_per_set": set_bytes,
                             "note": "every step runs on the copy least recently used"}
    else:
        out["cold_cache"] = None    # one step's working set alone does not fit the cache

    def stage_times(n_chunks_unused=None):
        n = min(args.steps, 50)
        cap = n * args.chunks * n_layers
        moe.moe_profile_enable((1 << len(moe.STAGES)) - 1, cap)
        for _ in range(n):
            step(sets[0])
        torch.cuda.synchronize()
        mean, med, mn = {}, {}, {}
        for i, name in enumerate(moe.STAGES):
            v = np.array(moe.moe_profile_read(i, cap))
            if v.size == 0:
                mean[name] = med[name] = mn[name] = None
                continue
            per_step = v.reshape(n, -1).sum(1) * 1e3                      # us per step
            mean[name], med[name], mn[name] = float(per_step.mean()), float(np.median(per_step)), float(per_step.min())
        moe.moe_profile_enable(0, 0)
        return mean, med, mn

    def row_mover_times():
        """Pack and combine alone (moe_dispatch, moe_combine on the layer's own routing): their
        stage times with nothing else running beside them, us per layer."""
        n = min(args.steps, 50)
        i_plan, i_sc, i_cb = (moe.STAGES.index(k) for k in ("plan", "scatter", "combine"))
        moe.moe_profile_enable((1 << i_plan) | (1 << i_sc) | (1 << i_cb), n * n_layers)
        for _ in range(n):
            x = sets[0][0].x
            for L in sets[0]:
                b = L.b
                moe.moe_dispatch(s, x, b["expert_idx"], b["counts"], b["offsets"], b["slot_of"], b["src_of"],
                                 b["xe"], b["workspace"])
                moe.moe_combine(s, b["ye"], b["slot_of"], b["gate"], b["y"], b["y_act"])
                x = b["y_act"]
        torch.cuda.synchronize()
        t = {k: np.array(moe.moe_profile_read(i, n * n_layers)) for k, i in (("plan", i_plan), ("scatter", i_sc), ("combine", i_cb))}
        moe.moe_profile_enable(0, 0)
        per = lambda v: None if v.size == 0 else float(v.reshape(n, -1).sum(1).mean() * 1e3)
        return per(t["plan"]), per(t["scatter"]), per(t["combine"])

    if not args.offload:
        st, med, mn = stage_times()
        alone_plan_us, alone_pack_us, alone_combine_us = row_mover_times()
        kept_tokens = float(np.mean([(L.b["slot_of"].view(l0.T, l0.k) >= 0).any(1).sum().item() for L in sets[0]]))
        ye_sz = sets[0][0].b["ye"].element_size()
        # The method's bytes (what the two all-to-all payloads carry, in the storage type):
        # pack reads every routed token once and writes every kept slot; unpack reads every kept
        # row and writes every token.  The bytes this build really moves differ where it keeps
        # the expert output and y wider than the storage type.
        disp_alg = (kept_tokens + A) * l0.d * esz * n_layers
        comb_alg = (A + l0.T) * l0.d * esz * n_layers
        comb_moved = (A * ye_sz + l0.T * 4 + (l0.T * esz if n_layers > 1 else 0)) * l0.d * n_layers + 8.0 * l0.T * l0.k * n_layers
        # (an unchunked layer of up to 64 MiB of token rows packs them in its plan launch: then
        # there is no pack stage and the bytes are set against the plan stage's time)
        # (inside the layer call the pack of a large layer runs beside the first expert GEMM, so
        # its own rate is taken from the stand-alone calls)
        # The combine figure is the layer's own stage (it runs alone on the caller's stream
        # there); the stand-alone call's is printed beside it (its rows come from HBM, inside
        # the layer part of them is still in the Infinity Cache).
        pack_in_plan = alone_pack_us is None
        pack_us = alone_plan_us if pack_in_plan else alone_pack_us
        comb_us = st["combine"] if args.chunks == 1 else alone_combine_us
        dc_us = (pack_us + comb_us) * 1e-6
        out["dispatch_combine"] = {
            "pack_us": pack_us, "combine_us": comb_us, "pack_in_plan_launch": pack_in_plan,
            "timed": "pack: moe_dispatch alone on the layer's routing; combine: its stage inside the layer call",
            "combine_alone_us": alone_combine_us,
            "algorithmic_bytes": disp_alg + comb_alg,
            "GBps": (disp_alg + comb_alg) / dc_us / 1e9,
            "frac_of_hbm_peak": (disp_alg + comb_alg) / dc_us / 1e9 / PEAK_HBM_GBPS,
            "pack_GBps": disp_alg / (pack_us * 1e-6) / 1e9,
            "combine_GBps": comb_alg / (comb_us * 1e-6) / 1e9,
            "moved_bytes": disp_alg + comb_moved,
            "moved_GBps": (disp_alg + comb_moved) / dc_us / 1e9,
            "combine_moved_GBps": comb_moved / (comb_us * 1e-6) / 1e9,
            "note": "algorithmic = (T'+A)*d*s packed + (A+T)*d*s unpacked, s = storage element size (the "
                    "target figure); moved = what the kernels transfer: expert rows as stored "
                    f"({ye_sz} B/element), y in fp32"}
        ffn_us = (st["gemm1"] + st["gemm2"]) * 1e-6
        ffn_bytes = (2 * live * l0.d * l0.h * 2 + A * l0.d * 2 + 2 * A * l0.h * 2 + A * l0.d * ye_sz) * n_layers
        out["ffn"] = {"gemm1_us": st["gemm1"], "gemm2_us": st["gemm2"],
                      "mfma_tflops": (4.0 * A * l0.d * l0.h * n_layers) / ffn_us / 1e12,
                      "mfma_util": (4.0 * A * l0.d * l0.h * n_layers) / ffn_us / 1e12 / PEAK_BF16_TFLOPS,
                      "gemm2_mfma_util": (2.0 * A * l0.d * l0.h * n_layers) / (st["gemm2"] * 1e-6) / 1e12 / PEAK_BF16_TFLOPS,
                      "GBps": ffn_bytes / ffn_us / 1e9}
        # gate: T*d*E sequential-order fp32 FMAs against the unpacked vector rate
        # (256 CUs x 64 lanes x 2.4 GHz = 39.3 TFMA/s; packed-fp32 instructions are off)
        out["gate"] = {"us": st["route"],
                       "alu_frac": (l0.T * l0.d * l0.E * n_layers) / (st["route"] * 1e-6) / 39.3e12}
        if args.backward:
            bw = [n for n in ("bwd_recompute", "bwd_dP", "bwd_dxe", "bwd_wgrad2", "bwd_wgrad1")
                  if st[n] is not None]          # no recomputation when the forward kept P
            out["bwd_gemm_mfma_util"] = (len(bw) * 2.0 * A * l0.d * l0.h) / (sum(st[n] for n in bw) * 1e-6) / 1e12 / PEAK_BF16_TFLOPS
        if args.stages:
            out["stages_us"] = st
            out["stages_us_median"] = med
            out["stages_us_min"] = mn
        if args.chunks > 1 and st["scatter"] is not None:
            # How much of the pack and unpack time the chunk pipeline hides behind the expert
            # FFN (Sec. 4.2's pipelining efficiency, with the pack kernel in the all-to-all's
            # place): 1 - (t_pipelined - t_ffn) / (t_pack + t_unpack), stage times summed over
            # the chunks, t_pipelined = the layer minus gate and plan.
            t_pipe = ms_per_step * 1e3 - st["route"] - st["plan"] - (st["tiles"] or 0.0)
            t_ffn = st["gemm1"] + st["gemm2"]
            out["chunk_overlap"] = {"t_pipelined_us": t_pipe, "t_ffn_us": t_ffn,
                                    "t_pack_us": st["scatter"], "t_unpack_us": st["combine"],
                                    "hidden_fraction": 1.0 - (t_pipe - t_ffn) / (st["scatter"] + st["combine"])}

    if not args.no_cpu_baseline and args.backward:
        # The backward oracle (fp64 numpy matmuls, forward included) once over the whole layer.
        from oracle import bwd_oracle
        li = host[0]
        dy_host = np.random.Generator(np.random.PCG64(7)).standard_normal((l0.T, l0.d))
        c0 = time.perf_counter()
        bwd_oracle.moe_layer_backward(li.x, li.Wg, li.W1, li.W2, dy_host, k=li.k, capacity=li.C,
                                      bias=li.gate_bias, bias_stride=li.bias_token_stride)
        elapsed = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": l0.T / elapsed, "unit": "tokens/s", "cores": os.cpu_count(),
                               "kind": "oracle",
                               "sample": f"one forward + backward pass of the fp64 oracle over all {l0.T} "
                                         f"tokens (numpy's BLAS threads), {elapsed:.2f} s wall"}
    elif not args.no_cpu_baseline:
        import oracle
        # Bounded sample: whole passes of the oracle over the workload (gate and plan over
        # all tokens; expert FFN and combine for a leading slice of tokens when one full
        # pass would take minutes), repeated until about 20 core-seconds have been spent.
        sample = l0.T
        est_flops = 4.0 * l0.T * l0.k * l0.d * l0.h * n_layers
        if est_flops > 4e11 and n_layers == 1:   # a stack needs every token of a layer for the next
            sample = max(64, int(l0.T * 4e11 / est_flops))
        toks = np.arange(sample, dtype=np.int32)
        cores = oracle.threads()
        passes, c0 = 0, time.perf_counter()
        while True:
            x_l = host[0].x
            for li in host:
                o = oracle.moe_layer(x_l, li.Wg, li.W1, li.W2, k=li.k, capacity=li.C, bias=li.gate_bias,
                                     bias_stride=li.bias_token_stride,
                                     tokens=None if sample == l0.T else toks)
                if n_layers > 1:
                    x_l = wl.bf16_round(o.y)      # the next layer reads the rounded output
            passes += 1
            elapsed = time.perf_counter() - c0
            if elapsed * cores >= 20.0 or passes >= 50:
                break
        out["cpu_baseline"] = {"value": sample * n_layers * passes / elapsed, "unit": "tokens/s",
                               "cores": cores, "kind": "oracle",
                               "sample": f"{passes} pass(es) over {n_layers} layer(s): gate+plan over all "
                                         f"{l0.T} tokens, expert FFN+combine for the first {sample} "
                                         f"tokens, {elapsed:.2f} s wall"}
    print(json.dumps(out))
    return 0


def calibrate() -> int:
    """Measured roofs of this box, one JSON line (not a step of the layer)."""
    import torch

    import paper_2210_17223_amd as moe
    dev = "cuda:0"
    torch.cuda.set_device(0)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    out = {"calibration": True, "nominal": {"hbm_GBps": PEAK_HBM_GBPS, "bf16_mfma_tflops": PEAK_BF16_TFLOPS}}
    nbytes = 1 << 30
    src = torch.full((nbytes // 4,), 1.0, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    times = []
    for _ in range(12):
        a, b = ev(), ev()
        a.record()
        moe.moe_calib_copy(dst, src, nbytes)
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b))
    assert torch.equal(dst[:1 << 20], src[:1 << 20])
    best, med = min(times[2:]), sorted(times[2:])[len(times[2:]) // 2]
    out["copy"] = {"bytes_read": nbytes, "bytes_written": nbytes, "launches": len(times),
                   "us_median": med * 1e3, "us_min": best * 1e3,
                   "GBps_median": 2 * nbytes / (med * 1e-3) / 1e9, "GBps_best": 2 * nbytes / (best * 1e-3) / 1e9,
                   "frac_of_nominal": 2 * nbytes / (med * 1e-3) / 1e9 / PEAK_HBM_GBPS}
    del src, dst
    out["mfma"] = {}
    for wps in (1, 2):
        sink = torch.empty(256 * wps * 256, dtype=torch.float32, device=dev)
        for rnd in (False, True):
            iters = 20000
            ms = []
            for _ in range(4):
                a, b = ev(), ev()
                a.record()
                flops = moe.moe_calib_mfma(sink, wps, iters, rnd)
                b.record()
                torch.cuda.synchronize()
                ms.append(a.elapsed_time(b))
            t = sorted(ms[1:])[1]
            out["mfma"][f"{'random' if rnd else 'constant'}_operands_{wps}_wave_per_simd"] = {
                "ms": t, "tflops": flops / (t * 1e-3) / 1e12,
                "frac_of_nominal": flops / (t * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
    # a yardstick, not a roof: the vendor library's dense bf16 GEMM (through torch.matmul) on
    # random data of the two sizes that bracket the layer's GEMMs
    out["vendor_dense_gemm"] = {}
    for m, n, k in ((8192, 8192, 8192), (65536, 8192, 2048), (65536, 2048, 8192)):
        a = torch.randn(m, k, device=dev, dtype=torch.bfloat16)
        b = torch.randn(k, n, device=dev, dtype=torch.bfloat16)
        for _ in range(3):
            torch.matmul(a, b)
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(10):
            torch.matmul(a, b)
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1) / 10
        out["vendor_dense_gemm"][f"{m}x{n}x{k}"] = {"ms": t, "tflops": 2.0 * m * n * k / (t * 1e-3) / 1e12,
                                                      "frac_of_nominal": 2.0 * m * n * k / (t * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
        del a, b
    print(json.dumps(out))
    return 0


def gemm_ablation() -> int:
    """What each part of the 256 x 256 expert-GEMM kernel costs: the kernel the layer runs,
    alone, with parts left out (their outputs are wrong by construction; only variant 0's is
    checked, on sampled elements against an fp64 dot product)."""
    import numpy as np
    import torch

    import paper_2210_17223_amd as moe
    dev = "cuda:0"
    torch.cuda.set_device(0)
    E, rows_e, BM = 64, 1024, 256
    variants = [(0, "whole kernel"), (8, "no output stores"),
                (6, "MFMAs + barriers only (one stage of operands)"), (4, "MFMAs + LDS fragment reads"),
                (2, "MFMAs + global loads + LDS writes"), (1, "everything but the MFMAs"),
                (7, "barriers, prologue and epilogue only")]
    out = {"gemm_ablation": True, "shape": f"{E} experts x {rows_e} rows, 256 x 256 tiles", "problems": {}}
    for tag, N, K, gelu in (("first GEMM  (N=8192, K=2048, GeLU)", 8192, 2048, True),
                            ("second GEMM (N=2048, K=8192)", 2048, 8192, False)):
        rows = E * rows_e
        mt, nt = rows_e // BM, N // 256
        gn = max(1, 32 // mt)
        items = []
        for e in range(E):
            for pn in range(0, nt, gn):
                for m in range(mt):
                    for n in range(pn, min(nt, pn + gn)):
                        items.append((e, e * rows_e + m * BM, e * rows_e + (m + 1) * BM, n * 256))
        items_d = torch.tensor(items, dtype=torch.int32, device=dev).reshape(-1)
        n_items = torch.tensor([len(items)], dtype=torch.int32, device=dev)
        flops = 2.0 * rows * N * K
        res = {}
        for data in ("random", "ones"):
            if data == "random":
                g = torch.Generator(device=dev).manual_seed(1)
                A = torch.randn(rows, K, device=dev, dtype=torch.float32, generator=g).to(torch.bfloat16)
                W = (torch.randn(E * N, K, device=dev, dtype=torch.float32, generator=g) * 0.02).to(torch.bfloat16)
            else:
                A = torch.ones(rows, K, device=dev, dtype=torch.bfloat16)
                W = torch.full((E * N, K), 0.0078125, device=dev, dtype=torch.bfloat16)
            Cout = torch.zeros(rows, N, device=dev, dtype=torch.float16)
            for var, name in (variants if data == "random" else variants[:1]):
                for _ in range(2):
                    moe.moe_calib_gemm(A, W, Cout, items_d, n_items, N, K, var, gelu)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(5):
                    moe.moe_calib_gemm(A, W, Cout, items_d, n_items, N, K, var, gelu)
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) / 5 * 1e3
                res[f"{name} [{data} operands]"] = {"variant": var, "us": us, "tflops_if_whole": flops / (us * 1e-6) / 1e12}
                if var == 0 and data == "random":
                    prng = np.random.Generator(np.random.PCG64(3))
                    rr, cc = prng.integers(0, rows, 256), prng.integers(0, N, 256)
                    a = A[torch.from_numpy(rr).to(dev)].double().cpu().numpy()
                    w = W.view(E, N, K)[torch.from_numpy(rr // rows_e).to(dev), torch.from_numpy(cc).to(dev)].double().cpu().numpy()
                    want = (a * w).sum(1)
                    if gelu:
                        import math
                        want = np.array([0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in want])
                    got = Cout[torch.from_numpy(rr).to(dev), torch.from_numpy(cc).to(dev)].double().cpu().numpy()
                    err = float(np.abs(got - want).max() / (np.abs(want).max() + 1e-30))
                    assert err < 5e-3, err
                    res["check_max_err_rel_to_max"] = err
            del A, W, Cout
        out["problems"][tag] = res
    print(json.dumps(out))
    return 0


def bench_comm(args, moe, wl, np, torch, dev) -> int:
    """Sec. 4.2 / 6.1 on one GPU.  (a) The layer in the padded layout with both all-to-alls cut
    into n micro-ops on the library's own stand-in link, FFN pipelined behind each micro-op:
    time per layer for n = 1, 2, 4, 8.  (b) The same layer through the scheduler while the
    gradient of its expert weights (E*d*h fp32) is being "allreduced" over the same link:
    uncut and in arrival order, against cut into micro-ops with all-to-all priority.
    A step of the headline figure is (b)'s prioritised case: layer + allreduce together."""
    from paper_2210_17223_amd import comm
    cfg = wl.CONFIGS[args.workload]
    if cfg["layers"] != 1:
        print("bench.py: --comm takes a one-layer workload", file=sys.stderr)
        return 2
    li = wl.make_layer(cfg, seed=0, threads=16)
    bf16 = li.dtype == "bf16"
    s = moe.Shape.make(li.T, li.d, li.E, li.h, li.k, li.C, dtype="bf16" if bf16 else "f32", act="gelu")
    esz = 2 if bf16 else 4

    def up(a):
        if bf16:
            return torch.from_numpy(wl.bf16_bits(a).view(np.int16).reshape(a.shape)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    b = moe.alloc_buffers(s, 1, dev)
    x = up(li.x)
    bias = None if li.gate_bias is None else torch.from_numpy(li.gate_bias).to(dev)
    moe.moe_pack_gate(s, up(li.Wg), b["Wgp"])
    moe.moe_pack_weights(s, up(li.W1), up(li.W2), b["W1p"], b["W2p"])
    slots = li.E * li.C
    i32 = lambda n: torch.empty(n, dtype=torch.int32, device=dev)
    p = dict(expert_idx=i32(li.T * li.k), gate=torch.empty(li.T * li.k, device=dev), counts=i32(li.E),
             slot_of=i32(li.T * li.k), src_of=i32(slots),
             xs=torch.empty(slots * li.d, dtype=s.torch_dtype, device=dev),
             xr=torch.empty(slots * li.d, dtype=s.torch_dtype, device=dev),
             ys=torch.zeros(slots * li.d, dtype=s.ye_dtype, device=dev),
             yr=torch.zeros(slots * li.d, dtype=s.ye_dtype, device=dev),
             y=torch.empty(li.T * li.d, device=dev))
    ws = {n: torch.empty(moe.moe_padded_workspace_bytes(s, n), dtype=torch.uint8, device=dev) for n in (1, 2, 4, 8)}

    def padded(n, link=None):
        moe.moe_layer_padded(s, n, link, args.link_blocks, x, b["Wgp"], bias, li.bias_token_stride, b["W1p"],
                             None, b["W2p"], None, p["expert_idx"], p["gate"], p["counts"], p["slot_of"],
                             p["src_of"], p["xs"], p["xr"], p["ys"], p["yr"], p["y"], ws[n])

    def compact():
        moe.moe_layer_chunked(s, 1, x, b["Wgp"], bias, li.bias_token_stride, b["W1p"], None, b["W2p"], None,
                              b["expert_idx"], b["gate"], b["counts"], b["offsets"], b["slot_of"], b["src_of"],
                              b["xe"], b["ye"], b["y"], None, b["workspace"])

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ysz = p["ys"].element_size()
    a2a_bytes = slots * li.d * (esz + ysz)                    # both all-to-alls of one layer
    res = {"compact_layer_ms": timed(compact, args.steps, args.warmup)}
    for n in (1, 2, 4, 8):
        res[f"padded_own_link_n{n}_ms"] = timed(lambda: padded(n), args.steps, args.warmup)
    assert torch.equal(p["y"].view(torch.int32), b["y"].view(torch.int32)), "padded y differs from the compact layer's"

    # the link alone: one all-to-all's worth of bytes as a single micro-op, timed on the device
    c = comm.moe_comm_create(comm.PRIORITY, args.link_blocks, 2)
    link_ms = []
    for i in range(6):
        op = comm.moe_comm_submit(c, comm.ALL_TO_ALL, p["ys"], p["yr"], li.E, li.C, li.d * ysz, 1)
        comm.moe_comm_post(c, op, 0, 1)
        link_ms.append(comm.moe_comm_finish(c, op))
    comm.moe_comm_destroy(c)
    link_gbps = slots * li.d * ysz / (min(link_ms[1:]) * 1e-3) / 1e9
    res["link_GBps"] = link_gbps

    # (b) contention: the layer through a scheduler that also carries a gradient allreduce
    grad = torch.randn(li.E * li.d * li.h, device=dev)
    gout = torch.empty_like(grad)
    grad_bytes = grad.numel() * 4
    micro_bytes = args.micro_mib << 20
    steps_b = max(5, min(args.steps, 30))

    def contended(policy, n_ar, n_micro, with_ar=True):
        c = comm.moe_comm_create(policy, args.link_blocks, 2)
        try:
            padded(n_micro, c)                                # first use: code load
            torch.cuda.synchronize()
            layer_ms, ar_ms = [], []
            for _ in range(steps_b):
                torch.cuda.synchronize()
                ar = None
                if with_ar:
                    ar = comm.moe_comm_submit(c, comm.ALLREDUCE, grad, gout, 1, grad.numel() // 4, 16, n_ar)
                    comm.moe_comm_post(c, ar, 0, n_ar)
                t0 = time.perf_counter()
                padded(n_micro, c)
                torch.cuda.synchronize()
                layer_ms.append((time.perf_counter() - t0) * 1e3)
                if ar is not None:
                    ar_ms.append(comm.moe_comm_finish(c, ar))
            return float(np.median(layer_ms)), (float(np.median(ar_ms)) if ar_ms else None)
        finally:
            comm.moe_comm_destroy(c)

    n_ar = (grad_bytes + micro_bytes - 1) // micro_bytes
    alone, _ = contended(comm.PRIORITY, 1, 4, with_ar=False)
    fifo, ar_fifo = contended(comm.ARRIVAL_ORDER, 1, 4)
    prio, ar_prio = contended(comm.PRIORITY, n_ar, 4)
    assert torch.equal(gout, grad)
    assert torch.equal(p["y"].view(torch.int32), b["y"].view(torch.int32))
    res.update({"scheduled_layer_alone_ms": alone, "scheduled_layer_behind_uncut_allreduce_ms": fifo,
                "scheduled_layer_prioritised_ms": prio, "allreduce_uncut_ms": ar_fifo,
                "allreduce_micro_ops_ms": ar_prio, "allreduce_bytes": grad_bytes,
                "allreduce_micro_ops": int(n_ar), "all_to_all_bytes_per_layer": a2a_bytes,
                "layer_slowdown_arrival_order": fifo / alone, "layer_slowdown_priority": prio / alone})
    out = {"metric": "moe_padded_layer_with_allreduce_tokens_per_s", "value": li.T / (prio * 1e-3),
           "unit": "tokens/s", "n_gpus": 1, "steps": steps_b, "warmup": 1, "ms_per_step": prio,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
           "config": {"workload": f"{args.workload}: T={li.T} d_model={li.d} E={li.E} d_ff={li.h} k={li.k} "
                                  f"capacity={li.C} {li.dtype}, seed 0; padded layout, 4 micro-ops per all-to-all, "
                                  f"stand-in link of {args.link_blocks} workgroups, {grad_bytes >> 20} MiB allreduce "
                                  f"in {int(n_ar)} micro-ops competing"},
           "roofline": {"bound": "hbm", "kernel": "link_copy_kernel (the stand-in link, one all-to-all's bytes)",
                        "achieved": 2 * link_gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                        "frac": 2 * link_gbps / PEAK_HBM_GBPS, "traffic": None,
                        "avg_launch_us": min(link_ms[1:]) * 1e3, "algorithmic_bytes": 2 * slots * li.d * ysz,
                        "note": "read + write of every byte; the kernel is confined to link_blocks workgroups "
                                "on purpose (it stands for a network link), so the fraction is a setting, "
                                "not an achievement"},
           "comm": res}
    if not args.no_cpu_baseline:
        from oracle import comm_oracle as co
        from oracle import moe_oracle as fo
        c0 = time.perf_counter()
        n = 0
        while time.perf_counter() - c0 < 10.0:
            o = fo.moe_layer(li.x, li.Wg, li.W1, li.W2, k=li.k, capacity=li.C, bias=li.gate_bias,
                             bias_stride=li.bias_token_stride)
            _, _, src = co.padded_plan(o.expert_idx, li.E, li.C)
            co.pack_padded(li.x, src, li.k)
            n += 1
        el = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": li.T * n / el, "unit": "tokens/s", "cores": fo.threads(), "kind": "oracle",
                               "sample": f"{n} pass(es) of the oracle layer plus the padded plan and pack over all "
                                         f"{li.T} tokens, {el:.2f} s wall"}
    print(json.dumps(out))
    return 0


def bench_popularity(args, moe, np, torch, dev) -> int:
    """The inference scheduler of Sec. 5.2 on the paper's inference shape (Sec. 7.1: 12 MoE
    layers, 16 experts, k = 1, sample-path length 3, at most 4 experts packed per device,
    one device per expert).  A step = one batch through all nine layers that have a
    three-layer history: estimate on the GPU, the estimate's 16 sums to the host, both
    scheduling phases on the host.  Also reports the estimation accuracy the paper's way
    (share of layers whose top-2k lists are identical)."""
    from workloads import paths
    L, E, k, l, N, max_pack = 12, 16, 1, 3, 16, 4
    N_t, T_prof = 8192, 1 << 20
    s = moe.PathShape(L, E, k, l)
    P, tables = moe.moe_path_count(s), L - l
    out = {"metric": "popularity_schedule_tokens_per_s", "unit": "tokens/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": f"popularity: L={L} E={E} k={k} l={l} N={N} max_pack={max_pack}, "
                                  f"{T_prof} profiled tokens, batches of {N_t}, seeded traces"}}
    acc = {}
    for kind in ("latent", "markov"):
        trace = paths.trace_generator(kind)(0, L, T_prof + 64 * N_t, E, k)
        prof = torch.from_numpy(np.ascontiguousarray(trace[:, :T_prof])).to(dev)
        counts = torch.zeros(tables * P * E, dtype=torch.int32, device=dev)
        top_e = torch.empty(tables * P * k, dtype=torch.int32, device=dev)
        top_q = torch.empty(tables * P * k, dtype=torch.int64, device=dev)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        moe.moe_path_profile(s, prof, T_prof, counts)
        moe.moe_path_finalize(s, counts, top_e, top_q)
        torch.cuda.synchronize()
        build_ms = (time.perf_counter() - t0) * 1e3
        S_dev = torch.empty(E, dtype=torch.int64, device=dev)
        batches = [torch.from_numpy(np.ascontiguousarray(trace[:, T_prof + b * N_t:T_prof + (b + 1) * N_t])).to(dev)
                   for b in range(64)]
        hits = total = resched = 0

        def one_batch(bt, score):
            nonlocal hits, total, resched
            for a in range(tables):
                moe.moe_popularity_estimate(s, bt[a:a + l], N_t, top_e[a * P * k:(a + 1) * P * k],
                                            top_q[a * P * k:(a + 1) * P * k], S_dev)
                S = S_dev.cpu().numpy().view(np.uint64)
                cnt = torch.bincount(bt[a + l].reshape(-1), minlength=E).to(torch.int32).cpu().numpy()
                again = moe.moe_schedule_layer(N, E, k, N_t, S, cnt, max_pack)[4]
                if score:
                    hits += 0 if again else 1
                    resched += 1 if again else 0
                    total += 1

        for b in range(args.warmup):
            one_batch(batches[b % 64], False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for b in range(args.steps):
            one_batch(batches[b % 64], b < 64)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        acc[kind] = {"top2k_lists_identical": hits / total, "phase_two_reschedules": resched / total,
                     "table_build_ms": build_ms, "ms_per_batch": ms}
        if kind == "latent":
            # the estimate kernel alone, timed with events on its stream
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            ev[0].record()
            for _ in range(200):
                moe.moe_popularity_estimate(s, batches[0][0:l], N_t, top_e[:P * k], top_q[:P * k], S_dev)
            ev[1].record()
            torch.cuda.synchronize()
            est_us = ev[0].elapsed_time(ev[1]) * 1e3 / 200
            bytes_per_launch = N_t * (l * k * 4 + k * 12) + E * 8
            out.update({"value": N_t / (ms * 1e-3), "ms_per_step": ms})
            out["roofline"] = {"bound": "hbm", "kernel": "popularity_estimate_kernel (+ its 64-lane clear)",
                               "achieved": bytes_per_launch / (est_us * 1e-6) / 1e9, "peak": PEAK_HBM_GBPS,
                               "unit": "GB/s", "frac": bytes_per_launch / (est_us * 1e-6) / 1e9 / PEAK_HBM_GBPS,
                               "traffic": None, "avg_launch_us": est_us,
                               "algorithmic_bytes": bytes_per_launch,
                               "note": "two launches over 8192 tokens: bound by launch latency, not by bytes"}
            if not args.no_cpu_baseline:
                from oracle import sched_oracle as so
                sample = 4096
                C = so.profile_counts(trace[:, :sample], l, E)        # tables from a bounded sample
                hist = trace[:, T_prof:T_prof + sample]
                c0 = time.perf_counter()
                n = 0
                while time.perf_counter() - c0 < 10.0:
                    for a in range(tables):
                        so.two_phase(C[a], hist[a:a + l], hist[a + l], E, k, N, max_pack)
                    n += 1
                el = time.perf_counter() - c0
                out["cpu_baseline"] = {"value": sample * n / el, "unit": "tokens/s", "cores": 1,
                                       "kind": "oracle",
                                       "sample": f"{n} pass(es) of estimate + two-phase decision for {sample} "
                                                 f"tokens over {tables} layers (tables from {sample} profiled "
                                                 f"tokens), {el:.2f} s wall"}
    out["estimation"] = acc
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
