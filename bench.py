#!/usr/bin/env python3
"""Benchmark of the LLSA layer (forward + backward) on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input already resident in HBM:
llsa_forward (pooling, hierarchical Top-K selection, attention over the gathered lists) followed by
llsa_backward (D, index transpose, dQ, dK/dV of every level, pooling adjoint).

Workload: benchmark configs[3], the shape its metric is quoted on: batch 1, 16 heads, d = 64,
N = 65536 (256 x 256 pixel tokens, row-major), B = 16, K = 8, L = 3, all levels enriched, bf16 I/O with
fp32 accumulation, smooth-field Q/K/V (the pixel-grid stand-in for DiT activations).

Prints ONE JSON line.  `value` is effective TFLOP/s = algorithmic sparse FLOPs of forward + backward
(4 d M N b h for the forward, 2.5 x that for the backward; M = gathered tokens per query) / step time.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E
PEAK_F32_TFLOPS = 157.3     # MI355X fp32 vector


def algorithmic_flops(cfg, M):
    fwd = 4.0 * cfg["d"] * M * cfg["N"] * cfg["batch"] * cfg["heads"]
    return fwd, 2.5 * fwd


def cpu_baseline(cfg, x, threads):
    """The CPU oracle, as it stands, on the first `threads` heads of the same inputs (one head per thread)."""
    from oracle import llsa_oracle as orc
    orc.build()
    g = orc.Geometry(cfg["N"], cfg["d"], cfg["B"], cfg["K"], cfg["L"])
    heads = [(b, h) for b in range(cfg["batch"]) for h in range(cfg["heads"])][:threads]

    def one(bh):
        b, h = bh
        f = orc.forward(x["Q"][b, h], x["K"][b, h], x["V"][b, h], g, bf16=cfg["dtype"] == "bf16")
        orc.backward(x["Q"][b, h], f["Kp"], f["Vp"], f["idx_cat"], x["dO"][b, h], g)
        return 0

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=len(heads)) as ex:
        list(ex.map(one, heads))
    dt = time.perf_counter() - t0
    fwd, bwd = algorithmic_flops(cfg, g.list_len(g.L))
    flops = (fwd + bwd) * len(heads) / (cfg["batch"] * cfg["heads"])
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": len(heads), "kind": "oracle",
            "sample": f"{len(heads)} of {cfg['batch'] * cfg['heads']} heads of the same workload, forward+backward, "
                      f"one head per thread, {dt:.1f} s"}


def measured_traffic(stage, workload, kind):
    """HBM bytes per launch of a stage's kernel as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by
    the plain-copy calibration) and recorded in profiles/hbm_traffic.txt; None if that workload was not measured."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) >= 5 and not line.startswith("#") and f[0] == stage and f[1] == workload and f[2] == kind:
            return float(f[3]) + float(f[4])
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="index into BASELINE.json configs (default: headline)")
    ap.add_argument("--kind", default=None, help="override the input kind: smooth | gaussian")
    ap.add_argument("--Le", type=int, default=None, help="override the number of enrichment levels (default: L)")
    ap.add_argument("--stage", default="auto", help="stage whose kernel is bracketed by HIP events in the timed region")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--all-stages", action="store_true", help="after the timed region, one more pass timing every stage")
    ap.add_argument("--dense-compare", action="store_true", help="also time dense bf16 SDPA (forward) on this GPU")
    ap.add_argument("--force-generic", action="store_true", help="run the portable scalar kernels")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of HIP-graph replays of the step")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 512 MiB (to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_16615_amd import inputs, llsa

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.calibrate_copy:
        src = torch.zeros(512 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel(), "copy_bytes_written": dst.numel(), "copies": 3}))
        return
    llsa.load()                                               # fails loudly if the HIP library is not built

    cfg = dict(inputs.CONFIGS[args.config])
    if args.kind:
        cfg["kind"] = args.kind
    seed = inputs.config_seed(args.config)
    t0 = time.time()
    x = {}
    with ThreadPoolExecutor(max_workers=4) as ex:
        futs = {n: ex.submit(inputs.make_tensor, cfg["kind"], seed, n, cfg["batch"], cfg["heads"], cfg["N"], cfg["d"])
                for n in ("Q", "K", "V", "dO")}
        for n, f in futs.items():
            x[n] = f.result()
    bf16 = cfg["dtype"] == "bf16"
    dev = {n: (torch.from_numpy(v).cuda().to(torch.bfloat16) if bf16 else torch.from_numpy(v).cuda()) for n, v in x.items()}
    if bf16:                                                  # the oracle leg must see the rounded values
        x = {n: dev[n].float().cpu().numpy() for n in x}
    print(f"[bench] inputs ready in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)

    plan = llsa.Plan(cfg["batch"], cfg["heads"], cfg["N"], cfg["d"], cfg["B"], cfg["K"], cfg["L"],
                     Le=args.Le, dtype=llsa.BF16 if bf16 else llsa.F32, kernel_path=1 if args.force_generic else 0)
    ws = plan.alloc_workspace(True)
    idx = plan.alloc_indices()
    Q, K, V, dO = dev["Q"], dev["K"], dev["V"], dev["dO"]
    O = torch.empty_like(Q)
    LSE = torch.empty(cfg["batch"], cfg["heads"], cfg["N"], dtype=torch.float32, device="cuda")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(Q)

    def step():
        llsa.forward(plan, Q, K, V, O, LSE, idx, ws)
        llsa.backward(plan, Q, K, V, O, LSE, idx, dO, ws, dQ, dK, dV)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    M = sum(li.K_l * cfg["B"] for li in plan.levels) + cfg["N"] // cfg["B"] ** cfg["L"]
    fwd_flops, bwd_flops = algorithmic_flops(cfg, M)
    stage = "dkv_fine" if args.stage == "auto" else args.stage

    # Eager pass: K steps with two HIP events per step around ONE kernel (the roofline kernel).
    llsa.stage_timing_begin(stage, max_calls=args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    eager_ms = (time.perf_counter() - t0) / args.steps * 1e3
    st = llsa.stage_timing_end()
    kern_ms = st[stage][0] / max(st[stage][1], 1)
    ms_per_step, mode = eager_ms, "eager launches"

    # The library neither allocates nor synchronises, so a whole step can be replayed from a HIP graph, which
    # removes the host launch gaps between its ~25 kernels.  Same kernels, same buffers, K replays timed.
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(max(1, args.warmup)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        ms_per_step, mode = (time.perf_counter() - t0) / args.steps * 1e3, "HIP graph replay of one step"

    # algorithmic work of one launch of the bracketed kernel
    bhNd = cfg["batch"] * cfg["heads"] * cfg["N"] * cfg["d"]
    elt = 2 if bf16 else 4
    per_level_pairs = 2.0 * cfg["d"] * cfg["N"] * cfg["batch"] * cfg["heads"] * (plan.levels[0].K_l * cfg["B"])
    work = {  # stage -> (bound, algorithmic flops or bytes of one launch)
        "attn_fwd": ("mfma", fwd_flops),
        "dq": ("mfma", 1.5 * fwd_flops),                      # S, dP, dQ = dS K: three contractions over the list
        "dkv_fine": ("mfma", 4.0 * per_level_pairs),          # S, dP, dV, dK over the level-0 pairs
        "pool": ("hbm", 3.0 * bhNd * elt * (1.0 + 1.0 / (cfg["B"] - 1))),
    }
    bound, amount = work.get(stage, ("mfma", 0.0))
    if args.force_generic or not bf16:
        roof_bound, peak, unit = ("alu", PEAK_F32_TFLOPS, "TFLOP/s") if bound == "mfma" else ("hbm", PEAK_HBM_GBPS, "GB/s")
    else:
        roof_bound, peak, unit = ("mfma", PEAK_BF16_TFLOPS, "TFLOP/s") if bound == "mfma" else ("hbm", PEAK_HBM_GBPS, "GB/s")
    achieved = amount / (kern_ms * 1e-3) / (1e12 if unit == "TFLOP/s" else 1e9) if kern_ms > 0 else 0.0
    roofline = {"kernel": stage, "bound": roof_bound, "achieved": achieved, "peak": peak, "unit": unit,
                "frac": achieved / peak, "traffic": measured_traffic(stage, cfg["name"], cfg["kind"]), "kernel_ms": kern_ms}

    out = {
        "metric": "llsa_fwd_bwd_effective_tflops_n65536_h16_d64_bf16" if args.config == 3 else
                  f"llsa_fwd_bwd_effective_tflops_{cfg['name']}",
        "value": (fwd_flops + bwd_flops) / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"BASELINE configs[{args.config}] {cfg['name']}: batch {cfg['batch']}, heads {cfg['heads']}, "
                               f"d {cfg['d']}, N {cfg['N']}, B {cfg['B']}, K {cfg['K']}, L {cfg['L']}, Le {cfg['L']}, "
                               f"{cfg['kind']} inputs, forward+backward",
                   "gathered_tokens_per_query": M, "kernels": "generic" if args.force_generic else "default",
                   "launch": mode, "eager_ms_per_step": eager_ms},
        "roofline": roofline,
    }

    if args.all_stages:
        llsa.stage_timing_begin(-1, max_calls=args.steps)
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        out["stages_ms"] = {k: (v[0] / v[1] if v[1] else None) for k, v in llsa.stage_timing_end().items()}

    if args.dense_compare:
        import torch.nn.functional as F
        for _ in range(2):
            F.scaled_dot_product_attention(Q, K, V)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            F.scaled_dot_product_attention(Q, K, V)
        torch.cuda.synchronize()
        out["dense_sdpa_fwd_ms"] = (time.perf_counter() - t0) / 3 * 1e3

    if not args.no_cpu:
        threads = min(16, os.cpu_count() or 1, cfg["batch"] * cfg["heads"])
        out["cpu_baseline"] = cpu_baseline(cfg, x, threads)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
