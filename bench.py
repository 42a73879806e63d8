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

`--sweep n|L|Le|K|all` instead runs the same kernels over other shapes (sequence length at fixed head
geometry, number of levels, enrichment depth, Top-K) and prints one JSON line per case plus a table on stderr.
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
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": len(heads), "nproc": os.cpu_count(), "kind": "oracle",
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


def device_inputs(cfg, seed, threads=16, keep_host=False):
    """Seeded synthetic Q, K, V, dO on the GPU in the I/O type (and, if asked, the same rounded values on the host)."""
    import torch
    from paper_2512_16615_amd import inputs
    bf16 = cfg["dtype"] == "bf16"
    shape = (cfg["batch"], cfg["heads"], cfg["N"], cfg["d"])
    dev = {n: torch.empty(shape, dtype=torch.bfloat16 if bf16 else torch.float32, device="cuda")
           for n in ("Q", "K", "V", "dO")}
    jobs = [(n, b, h) for n in dev for b in range(cfg["batch"]) for h in range(cfg["heads"])]

    def one(job):
        n, b, h = job
        return job, inputs.make_head(cfg["kind"], seed, n, b, h, cfg["N"], cfg["d"])

    with ThreadPoolExecutor(max_workers=threads) as ex:
        for (n, b, h), v in ex.map(one, jobs):
            dev[n][b, h].copy_(torch.from_numpy(v))          # rounds to nearest even for bf16 I/O
    host = {n: dev[n].float().cpu().numpy() for n in dev} if keep_host else None
    return dev, host


def step_events(fn, steps):
    """K calls of fn, each bracketed by two HIP events on the current stream (which is the stream the library is
    given): (median, min) milliseconds per call.  L2 / Infinity Cache are not flushed between the calls."""
    import torch
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in ev)
    return ms[len(ms) // 2], ms[0]


def timed(fn, steps, warmup, graph):
    """Milliseconds per call of fn (which only enqueues work): eager launches, then optionally replays of a HIP
    graph holding one call.  Returns (eager_ms, graph_ms or None)."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    eager = (time.perf_counter() - t0) / steps * 1e3
    if not graph:
        return eager, None
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
        with torch.cuda.graph(g, stream=side):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(max(1, warmup)):
        g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        g.replay()
    torch.cuda.synchronize()
    return eager, (time.perf_counter() - t0) / steps * 1e3


class Case:
    """Plan and buffers of one workload; step() enqueues forward + backward."""

    def __init__(self, cfg, dev, Le=None, force_generic=False, single_stream=False):
        import torch
        from paper_2512_16615_amd import llsa
        self.llsa, self.cfg = llsa, cfg
        bf16 = cfg["dtype"] == "bf16"
        self.plan = llsa.Plan(cfg["batch"], cfg["heads"], cfg["N"], cfg["d"], cfg["B"], cfg["K"], cfg["L"], Le=Le,
                              dtype=llsa.BF16 if bf16 else llsa.F32, kernel_path=1 if force_generic else 0,
                              single_stream=1 if single_stream else 0)
        self.Le = cfg["L"] if Le is None else Le
        self.ws = self.plan.alloc_workspace(True)
        self.idx = self.plan.alloc_indices()
        self.Q, self.K, self.V, self.dO = dev["Q"], dev["K"], dev["V"], dev["dO"]
        self.O = torch.empty_like(self.Q)
        self.LSE = torch.empty(cfg["batch"], cfg["heads"], cfg["N"], dtype=torch.float32, device="cuda")
        self.dQ, self.dK, self.dV = torch.empty_like(self.Q), torch.empty_like(self.Q), torch.empty_like(self.Q)
        # gathered tokens per query: K_l * B of every enriched sparse level, all n_L tokens if the top is enriched
        self.M = sum(li.K_l * cfg["B"] for l, li in enumerate(self.plan.levels) if l <= self.Le)
        if self.Le == cfg["L"]:
            self.M += cfg["N"] // cfg["B"] ** cfg["L"]

    def forward(self):
        self.llsa.forward(self.plan, self.Q, self.K, self.V, self.O, self.LSE, self.idx, self.ws)

    def step(self):
        self.forward()
        self.llsa.backward(self.plan, self.Q, self.K, self.V, self.O, self.LSE, self.idx, self.dO, self.ws,
                           self.dQ, self.dK, self.dV)

    def stages(self, steps):
        import torch
        self.llsa.stage_timing_begin(-1, max_calls=steps)
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        return {k: (v[0] / v[1] if v[1] else None) for k, v in self.llsa.stage_timing_end().items()}


def sweep_cases(which):
    base = dict(batch=1, d=64, B=16, K=8, dtype="bf16", kind="smooth")
    heads_for = {4096: 16, 16384: 16, 65536: 16, 262144: 8, 1048576: 4}     # distinct heads; throughput is per token
    deepest = {4096: 2, 16384: 3, 65536: 3, 262144: 4, 1048576: 4}          # L = ceil(log_B N) - 1
    out = []

    def add(group, N, L, Le=None, K=8):
        out.append((group, dict(base, name=f"{group}_N{N}_L{L}_Le{L if Le is None else Le}_K{K}", N=N, L=L, K=K,
                                heads=heads_for[N]), Le))

    if which in ("n", "all", "mask"):
        for N in (4096, 16384, 65536, 262144, 1048576):
            add("n", N, deepest[N])
    if which in ("L", "all"):
        for N, Ls in ((65536, (1, 2, 3)), (262144, (1, 2, 3, 4))):
            for L in Ls:
                add("L", N, L)
    if which in ("Le", "all"):
        for Le in (0, 1, 2, 3):
            add("Le", 65536, 3, Le=Le)
    if which in ("K", "all"):
        for K in (4, 8, 16, 32):
            add("K", 65536, 3, K=K)
    if which in ("B", "all"):                                  # the paper's other block size (Fig. 3), same tokens per level
        out.append(("B", dict(base, name="B_N65536_B64_L2_K2", N=65536, B=64, L=2, K=2, heads=16), None))
        out.append(("B", dict(base, name="B_N65536_B64_L2_K8", N=65536, B=64, L=2, K=8, heads=16), None))
    return out


def run_sweep(args):
    import torch
    rows, cache = [], {}
    for group, cfg, Le in sweep_cases(args.sweep):
        key = (cfg["N"], cfg["heads"])
        if key not in cache:                                   # the inputs depend on the shape only
            cache.clear()
            torch.cuda.empty_cache()
            t0 = time.time()
            cache[key] = device_inputs(cfg, 0x115A1000 + cfg["N"] % 9973)[0]
            print(f"[sweep] inputs N={cfg['N']} heads={cfg['heads']} ready in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)
        case = Case(cfg, cache[key], Le=Le, single_stream=args.single_stream)
        steps = max(3, min(args.steps, int(2e8 // (cfg["N"] * cfg["heads"])) + 3))
        f_eager, f_graph = timed(case.forward, steps, args.warmup, not args.no_graph)
        s_eager, s_graph = timed(case.step, steps, args.warmup, not args.no_graph)
        fwd_ms, step_ms = (f_graph or f_eager), (s_graph or s_eager)
        fwd_flops, bwd_flops = algorithmic_flops(cfg, case.M)
        st = case.stages(steps)
        row = {"case": cfg["name"], "group": group, "N": cfg["N"], "heads": cfg["heads"], "d": cfg["d"], "B": cfg["B"],
               "K": cfg["K"], "L": cfg["L"], "Le": case.Le, "gathered_tokens_per_query": case.M, "steps": steps,
               "fwd_ms": fwd_ms, "fwd_bwd_ms": step_ms, "eager_fwd_bwd_ms": s_eager,
               "fwd_tflops": fwd_flops / fwd_ms / 1e9, "fwd_bwd_tflops": (fwd_flops + bwd_flops) / step_ms / 1e9,
               "fwd_bwd_mtokens_per_s": cfg["N"] * cfg["heads"] / step_ms / 1e3,
               "kv_backward_ms": (st.get("dkv_coarse") or 0.0) + (st.get("dkv_fine") or 0.0) + (st.get("index_transpose") or 0.0),
               "stages_ms": st}
        row["kv_backward_mtokens_per_s"] = cfg["N"] * cfg["heads"] / row["kv_backward_ms"] / 1e3
        # Sec. 5.4 / Fig. 4: key/value backward of level 0 alone, lists from Alg. 2 against lists from a dense
        # T x T block mask (built and scanned inside the timed call); the mask must fit (here: up to 40 GB)
        T = cfg["N"] // cfg["B"]
        row["kv0_csc_ms"] = row["kv0_mask_ms"] = None
        if group == "n" or args.sweep == "mask":
            llsa_mod = case.llsa
            a = (case.Q, case.K, case.V, case.dO, case.LSE, case.idx, case.ws)
            dK0, dV0 = torch.empty_like(case.Q), torch.empty_like(case.Q)
            case.step()                                        # D and the pooled levels in the workspace
            row["kv0_csc_ms"] = timed(lambda: llsa_mod.kv_backward_level0(case.plan, False, *a, dK0=dK0, dV0=dV0), steps, 1, False)[0]
            if cfg["heads"] * T * T <= 40e9:
                mask = torch.empty(case.plan.batch * case.plan.heads * T * T + 256, dtype=torch.uint8, device="cuda")
                row["kv0_mask_ms"] = timed(lambda: llsa_mod.kv_backward_level0(case.plan, True, *a, mask=mask, dK0=dK0, dV0=dV0),
                                           steps, 1, False)[0]
                del mask
            for k in ("kv0_csc_ms", "kv0_mask_ms"):
                if row[k]:
                    row[k.replace("_ms", "_mtokens_per_s")] = cfg["N"] * cfg["heads"] / row[k] / 1e3
        rows.append(row)
        print(json.dumps(row), flush=True)
        del case
    hdr = (f"{'case':34s} {'M':>5s} {'fwd ms':>9s} {'f+b ms':>9s} {'fwd TF/s':>9s} {'f+b TF/s':>9s} {'f+b Mtok/s':>11s} "
           f"{'KV-bwd Mtok/s':>14s} {'kv0 csc ms':>11s} {'kv0 mask ms':>12s}")
    print(hdr, file=sys.stderr)
    fmt = lambda v: f"{v:.3f}" if v else "-"
    for r in rows:
        print(f"{r['case']:34s} {r['gathered_tokens_per_query']:5d} {r['fwd_ms']:9.3f} {r['fwd_bwd_ms']:9.3f} {r['fwd_tflops']:9.1f} "
              f"{r['fwd_bwd_tflops']:9.1f} {r['fwd_bwd_mtokens_per_s']:11.1f} {r['kv_backward_mtokens_per_s']:14.1f} "
              f"{fmt(r['kv0_csc_ms']):>11s} {fmt(r['kv0_mask_ms']):>12s}", file=sys.stderr)


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
    ap.add_argument("--order", default="raster", choices=["raster", "nested"],
                    help="token order of the pixel grid: raster (BASELINE's) or the paper's nested-patch index reordering, "
                         "applied once with llsa_reorder before the timed region")
    ap.add_argument("--single-stream", action="store_true",
                    help="keep the backward on the caller's stream (no fork onto the plan's auxiliary stream)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 512 MiB (to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--glue", action="store_true",
                    help="only time llsa_qknorm_rope_pool (QK-Norm + RoPE fused with pooling) against llsa_pool")
    ap.add_argument("--pool-cache", action="store_true",
                    help="only time the pooling stage warm (back to back) and with the caches flushed by a 1 GiB copy between calls")
    ap.add_argument("--sweep", default=None, choices=["n", "L", "Le", "K", "B", "all", "mask"],
                    help="run the shape sweep instead of the headline workload")
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
    if args.sweep:
        run_sweep(args)
        return

    cfg = dict(inputs.CONFIGS[args.config])
    if args.kind:
        cfg["kind"] = args.kind
    bf16 = cfg["dtype"] == "bf16"
    t0 = time.time()
    dev, x = device_inputs(cfg, inputs.config_seed(args.config), keep_host=not args.no_cpu)
    print(f"[bench] inputs ready in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)

    if args.order == "nested":                               # once per model in the paper: outside the timed region
        from oracle import llsa_oracle as orc
        dev = {n: llsa.reorder(v) for n, v in dev.items()}
        if x is not None:
            x = {n: np.stack([np.stack([orc.reorder(v[b, h]) for h in range(v.shape[1])]) for b in range(v.shape[0])])
                 for n, v in x.items()}
    case = Case(cfg, dev, Le=args.Le, force_generic=args.force_generic, single_stream=args.single_stream)
    for _ in range(args.warmup):
        case.step()
    torch.cuda.synchronize()
    fwd_flops, bwd_flops = algorithmic_flops(cfg, case.M)
    if args.glue:
        # the fused glue + pooling pass against pooling alone (what a separate glue kernel would have to be added to)
        elt = 2 if bf16 else 4
        bhNd = cfg["batch"] * cfg["heads"] * cfg["N"] * cfg["d"]
        cos, sin = (torch.from_numpy(a).cuda() for a in inputs.rope_tables(cfg["N"], cfg["d"]))
        gq, gk = (torch.from_numpy(inputs.norm_gain(1, w, cfg["d"])).cuda() for w in ("Q", "K"))
        ws2 = case.plan.alloc_workspace(False)
        res = {}
        for name, fn in (("qknorm_rope_pool", lambda: llsa.qknorm_rope_pool(case.plan, case.Q, case.K, case.V, gq, gk, cos, sin, 1e-6, ws2)),
                         ("pool", lambda: llsa.pool(case.plan, case.Q, case.K, case.V, case.ws))):
            for _ in range(3):
                fn()
            med, mn = step_events(fn, args.steps)
            res[name] = {"median_ms": med, "min_ms": mn}
        pool_bytes = 3.0 * bhNd * elt * (1.0 + 1.0 / (cfg["B"] - 1))
        glue_bytes = pool_bytes + 2.0 * bhNd * elt            # plus Qout and Kout written
        res["qknorm_rope_pool"]["algorithmic_bytes"] = glue_bytes
        res["qknorm_rope_pool"]["gbps_at_median"] = glue_bytes / res["qknorm_rope_pool"]["median_ms"] / 1e6
        res["pool"]["algorithmic_bytes"] = pool_bytes
        res["pool"]["gbps_at_median"] = pool_bytes / res["pool"]["median_ms"] / 1e6
        res["unfused_estimate_bytes"] = pool_bytes + 4.0 * bhNd * elt   # a separate glue kernel reads and writes Q and K
        print(json.dumps({"glue": res, "workload": cfg["name"]}))
        return
    if args.pool_cache:
        # pooling alone: back to back (its 400 MB of input were just read by the previous call: what stays in the
        # 256 MB Infinity Cache is warm), and after a 1 GiB copy that evicts L2 and Infinity Cache
        pool_bytes = 3.0 * cfg["batch"] * cfg["heads"] * cfg["N"] * cfg["d"] * (2 if bf16 else 4) * (1.0 + 1.0 / (cfg["B"] - 1))
        junk_a = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        junk_b = torch.empty_like(junk_a)
        res = {}
        for mode in ("warm", "flushed"):
            ev = []
            for _ in range(args.steps):
                if mode == "flushed":
                    junk_b.copy_(junk_a)
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                llsa.pool(case.plan, case.Q, case.K, case.V, case.ws)
                b.record()
                ev.append((a, b))
            torch.cuda.synchronize()
            ms = sorted(a.elapsed_time(b) for a, b in ev)
            res[mode] = {"median_ms": ms[len(ms) // 2], "min_ms": ms[0], "gbps_at_median": pool_bytes / ms[len(ms) // 2] / 1e6}
        print(json.dumps({"pool_all_levels": res, "algorithmic_bytes": pool_bytes, "workload": cfg["name"]}))
        return
    stage = args.stage
    if stage == "auto":      # the longest single kernel of the step, from one untimed pass that brackets every stage
        st = case.stages(2)
        longest = max(st.get(k) or 0.0 for k in ("attn_fwd", "dq", "dkv_fine"))
        # kernels within 5 % of the longest count as tied (dQ and the level-0 dK/dV kernel are, at the headline); the tie
        # goes to the one with the most algorithmic work, in this order, so that the choice does not flip from run to run
        stage = next(k for k in ("dq", "attn_fwd", "dkv_fine") if (st.get(k) or 0.0) >= 0.95 * longest)

    # Eager pass: K steps with two HIP events per step around ONE kernel (the roofline kernel).
    llsa.stage_timing_begin(stage, max_calls=args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        case.step()
    torch.cuda.synchronize()
    eager_ms = (time.perf_counter() - t0) / args.steps * 1e3
    st = llsa.stage_timing_end()
    kern_ms = st[stage][0] / max(st[stage][1], 1)
    ms_per_step, mode = eager_ms, "eager launches"
    median_ms, min_ms = step_events(case.step, args.steps)     # per-step HIP-event brackets: spread of the same step

    # The library neither allocates nor synchronises, so a whole step can be replayed from a HIP graph, which
    # removes the host launch gaps between its ~25 kernels.  Same kernels, same buffers, K replays timed.
    graph_ms = None
    if not args.no_graph:
        _, graph_ms = timed(case.step, args.steps, 0, True)
        if graph_ms < eager_ms:                               # report the faster of the two ways to launch the same step
            ms_per_step, mode = graph_ms, "HIP graph replay of one step"

    # algorithmic work of one launch of the bracketed kernel
    bhNd = cfg["batch"] * cfg["heads"] * cfg["N"] * cfg["d"]
    elt = 2 if bf16 else 4
    per_level_pairs = 2.0 * cfg["d"] * cfg["N"] * cfg["batch"] * cfg["heads"] * (case.plan.levels[0].K_l * cfg["B"])
    n_pooled = sum(cfg["N"] // cfg["B"] ** l for l in range(1, cfg["L"] + 1))
    sel_bytes = 0.0                                           # pooled Q, K read once, gathered candidate rows, indices written
    for l in range(1, cfg["L"] + 1):
        n_l = cfg["N"] // cfg["B"] ** l
        cand = n_l if l == cfg["L"] else case.plan.levels[l].K_l * cfg["B"]
        k_out = case.plan.levels[l - 1].K_l
        sel_bytes += cfg["batch"] * cfg["heads"] * (2.0 * n_l * cfg["d"] * elt + (n_l / cfg["B"]) * cand * cfg["d"] * elt
                                                    + n_l * k_out * 4.0)
    # stage -> (bound, ALGORITHMIC flops or bytes of one launch, contractions the kernels execute / the method defines)
    work = {
        "attn_fwd": ("mfma", fwd_flops, "2 / 2"),
        "dq": ("mfma", 1.5 * fwd_flops, "3 / 3"),             # S, dP, dQ = dS K
        "dkv_fine": ("mfma", 2.0 * per_level_pairs, "4 / 2"), # dV, dK (S and dP are recomputed: executed, not counted)
        "dkv_coarse": ("mfma", fwd_flops - 2.0 * per_level_pairs if case.Le >= 1 else 0.0, "4 / 2"),
        "pool": ("hbm", 3.0 * bhNd * elt * (1.0 + 1.0 / (cfg["B"] - 1)), None),
        "select": ("hbm", sel_bytes, None),
    }
    bound, amount, _ = work.get(stage, ("mfma", 0.0, None))
    if args.force_generic or not bf16:
        roof_bound, peak, unit = ("alu", PEAK_F32_TFLOPS, "TFLOP/s") if bound == "mfma" else ("hbm", PEAK_HBM_GBPS, "GB/s")
    else:
        roof_bound, peak, unit = ("mfma", PEAK_BF16_TFLOPS, "TFLOP/s") if bound == "mfma" else ("hbm", PEAK_HBM_GBPS, "GB/s")
    achieved = amount / (kern_ms * 1e-3) / (1e12 if unit == "TFLOP/s" else 1e9) if kern_ms > 0 else 0.0
    roofline = {"kernel": stage, "bound": roof_bound, "achieved": achieved, "peak": peak, "unit": unit,
                "frac": achieved / peak, "traffic": measured_traffic(stage, cfg["name"], cfg["kind"]), "kernel_ms": kern_ms,
                "traffic_source": "profiles/hbm_traffic.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, "
                                  "recorded beforehand (counters cannot be read inside the run)"}
    # what this GPU delivers on nothing but MFMAs / on a plain copy, and the fraction against that as well
    peaks = llsa.measured_peaks()
    measured_peak = peaks["mfma_bf16_tflops"] if unit == "TFLOP/s" else peaks["copy_gbps"]
    roofline["measured_peak"] = measured_peak
    roofline["frac_of_measured_peak"] = achieved / measured_peak if measured_peak > 0 else None

    out = {
        "metric": "llsa_fwd_bwd_effective_tflops_n65536_h16_d64_bf16" if args.config == 3 else
                  f"llsa_fwd_bwd_effective_tflops_{cfg['name']}",
        "value": (fwd_flops + bwd_flops) / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": median_ms, "ms_per_step_min": min_ms, "caches": "warm (no flush between steps)",
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"BASELINE configs[{args.config}] {cfg['name']}: batch {cfg['batch']}, heads {cfg['heads']}, "
                               f"d {cfg['d']}, N {cfg['N']}, B {cfg['B']}, K {cfg['K']}, L {cfg['L']}, Le {case.Le}, "
                               f"{cfg['kind']} inputs in {args.order} token order, forward+backward",
                   "gathered_tokens_per_query": case.M, "kernels": "generic" if args.force_generic else "default",
                   "launch": mode, "eager_ms_per_step": eager_ms, "graph_ms_per_step": graph_ms,
                   "streams": "caller's stream only" if args.single_stream else "caller's stream + one auxiliary stream inside llsa_backward"},
        "roofline": roofline,
        "measured_peaks": peaks,
    }

    # every stage of the step against its own roofline (one more pass outside the timed region; bracketing every
    # stage keeps the backward on one stream, so index_transpose is not hidden here as it is in the timed step)
    st_all = case.stages(min(args.steps, 10))
    kernels = {}
    for name, (b, amt, contr) in work.items():
        ms = st_all.get(name)
        if not ms or amt <= 0:
            continue
        mf = b == "mfma" and bf16 and not args.force_generic
        pk, un = (PEAK_BF16_TFLOPS, "TFLOP/s") if mf else (PEAK_F32_TFLOPS, "TFLOP/s") if b == "mfma" else (PEAK_HBM_GBPS, "GB/s")
        ach = amt / (ms * 1e-3) / (1e12 if un == "TFLOP/s" else 1e9)
        kernels[name] = {"ms": ms, "bound": "mfma" if mf else "alu" if b == "mfma" else "hbm", "achieved": ach, "unit": un,
                         "frac": ach / pk}
        if contr:
            kernels[name]["contractions_executed_over_algorithmic"] = contr
    out["kernels"] = kernels
    if args.all_stages:
        out["stages_ms"] = st_all

    if args.dense_compare:
        import torch.nn.functional as F
        for _ in range(2):
            F.scaled_dot_product_attention(case.Q, case.K, case.V)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            F.scaled_dot_product_attention(case.Q, case.K, case.V)
        torch.cuda.synchronize()
        out["dense_sdpa_fwd_ms"] = (time.perf_counter() - t0) / 3 * 1e3

    if not args.no_cpu:
        threads = min(16, os.cpu_count() or 1, cfg["batch"] * cfg["heads"])
        out["cpu_baseline"] = cpu_baseline(cfg, x, threads)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
