"""Shared helpers of the GPU parity tests: seeded inputs -> GPU library and CPU oracle -> comparisons.

Tolerances (written here once, used by every parity test):
  * pooled levels: bit-exact (the pooling order and rounding are a contract, selection depends on them);
  * selection indices: bit-exact, level by level with teacher forcing (the oracle's level-l selection is fed the
    GPU's own parent lists); a row may differ only where the gap between the K-th and (K+1)-th fp64 score is
    below 1e-5 relative;
  * O, dQ, dK, dV: max-abs error <= 2e-2 (bf16 I/O) or 1e-4 (fp32 I/O), where for bf16 outputs of magnitude
    above 1 the bound scales with the magnitude (half an ulp of bf16 is 2^-9 relative, so a bf16 result cannot
    be closer than that to the fp64 value): |err| <= tol * max(1, |ref|);
  * LSE (always fp32): 1e-4 (fp32 I/O) or 1e-3 (bf16 I/O).
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

from oracle import llsa_oracle as orc
from paper_2512_16615_amd import inputs, llsa

TOL = {"f32": dict(out=1e-4, lse=1e-4), "bf16": dict(out=2e-2, lse=1e-3)}


def make_inputs(cfg: dict, seed: int):
    """fp32 numpy tensors [batch, heads, N, d] already rounded to the I/O type."""
    out = {}
    for name in ("Q", "K", "V", "dO"):
        x = inputs.make_tensor(cfg["kind"], seed, name, cfg["batch"], cfg["heads"], cfg["N"], cfg["d"])
        out[name] = orc.to_bf16(x) if cfg["dtype"] == "bf16" else x
    return out


def to_dev(x: np.ndarray, cfg: dict) -> torch.Tensor:
    t = torch.from_numpy(x).cuda()
    return t.to(torch.bfloat16) if cfg["dtype"] == "bf16" else t   # exact: values are bf16-representable


def make_plan(cfg: dict, **kw) -> llsa.Plan:
    args = dict(batch=cfg["batch"], heads=cfg["heads"], N=cfg["N"], d=cfg["d"], B=cfg["B"], K=cfg["K"], L=cfg["L"],
                Le=cfg.get("Le"), dtype=llsa.BF16 if cfg["dtype"] == "bf16" else llsa.F32,
                reweight=cfg.get("reweight", 1), sm_scale=cfg.get("sm_scale", 0.0))
    args.update(kw)
    return llsa.Plan(**args)


def gpu_forward_backward(cfg: dict, x: dict, plan: llsa.Plan | None = None, backward: bool = True):
    plan = plan or make_plan(cfg)
    Q, K, V, dO = (to_dev(x[n], cfg) for n in ("Q", "K", "V", "dO"))
    ws = plan.alloc_workspace(True)
    O, LSE, idx, _ = llsa.forward(plan, Q, K, V, workspace=ws)
    res = {"plan": plan, "O": O, "LSE": LSE, "indices": idx, "ws": ws, "Q": Q, "K": K, "V": V, "dO": dO}
    if backward:
        res["dQ"], res["dK"], res["dV"] = llsa.backward(plan, Q, K, V, O, LSE, idx, dO, ws)
    torch.cuda.synchronize()
    return res


def geometry(cfg: dict) -> orc.Geometry:
    return orc.Geometry(cfg["N"], cfg["d"], cfg["B"], cfg["K"], cfg["L"])


def oracle_head(cfg: dict, x: dict, b: int, h: int, backward: bool = True, rows=None):
    g = geometry(cfg)
    Le = cfg.get("Le")
    Le = g.L if Le is None else Le
    sc = cfg.get("sm_scale", 0.0)
    sc = None if sc <= 0 else sc
    f = orc.forward(x["Q"][b, h], x["K"][b, h], x["V"][b, h], g, Le=Le, bf16=cfg["dtype"] == "bf16",
                    reweight=cfg.get("reweight", 1), scale=sc, rows=rows, want_margin=True)
    if backward:
        f.update(orc.backward(x["Q"][b, h], f["Kp"], f["Vp"], f["idx_cat"], x["dO"][b, h], g, Le=Le,
                              reweight=cfg.get("reweight", 1), scale=sc))
    return f


def oracle_all_heads(cfg: dict, x: dict, heads=None, backward: bool = True, threads: int = 8):
    heads = heads or [(b, h) for b in range(cfg["batch"]) for h in range(cfg["heads"])]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        res = list(ex.map(lambda bh: oracle_head(cfg, x, bh[0], bh[1], backward), heads))
    return dict(zip(heads, res))


def f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def check_pyramid(cfg, gpu, ref, b, h):
    plan = gpu["plan"]
    for x, name in enumerate(("Qp", "Kp", "Vp")):
        for l in range(1, cfg["L"] + 1):
            got = f32(plan.pyramid_level(gpu["ws"], x, l)[b, h])
            assert np.array_equal(got, ref[name][l]), f"pooled {name} level {l} head {(b, h)} not bit-exact"


def check_indices(cfg, gpu, ref, b, h, x):
    """Teacher-forced, level-by-level comparison; returns (#rows differing from the free-running oracle,
    #rows excused as near-ties)."""
    plan, g = gpu["plan"], geometry(cfg)
    excused = free_diff = 0
    for l in range(g.L, 0, -1):
        got = plan.level_indices(gpu["indices"], l - 1)[b, h].cpu().numpy()
        assert got.shape == (g.n(l), g.K_l(l - 1))
        assert np.all(np.diff(got, axis=1) > 0), "rows must be ascending and distinct"
        parent = None if l == g.L else plan.level_indices(gpu["indices"], l)[b, h].cpu().numpy()
        want, margin = orc.select_level(ref["Qp"][l], ref["Kp"][l], g.B, parent, g.K_l(l - 1), want_margin=True)
        bad = np.nonzero((got != want).any(axis=1))[0]
        for i in bad:
            assert margin[i] < 1e-5, f"level {l} row {i} head {(b, h)}: indices differ, margin {margin[i]:.3e}"
        excused += len(bad)
        free_diff += int((got != ref["I"][l - 1]).any(axis=1).sum())
    return free_diff, excused


def max_err(got: np.ndarray, ref: np.ndarray):
    err = np.abs(got.astype(np.float64) - ref)
    scaled = err / np.maximum(1.0, np.abs(ref))
    return float(err.max()), float(scaled.max())


def check_close(name, got, ref, tol):
    err, scaled = max_err(got, ref)
    assert scaled <= tol, f"{name}: max-abs err {err:.3e} (scaled {scaled:.3e}) > {tol}"
    return err
