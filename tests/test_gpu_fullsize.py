"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot run these shapes whole in a test's time, so per configuration:
  * pooled levels and selection indices: bit-exact on a few heads (selection is cheap for the oracle);
  * O / LSE / dQ: element-wise on sampled query rows of those heads (each row is an independent oracle call);
  * dK / dV: element-wise on one whole head where the oracle's backward fits (N <= 65536), and on every head via
    properties that hold at any size: sum_t dV[t] = sum_q dO[q] and <dQ, Q> = <dK, K> (Euler identity of the
    bilinear logits; exact up to the bf16 rounding of the pooled levels and outputs).
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from tests import harness as H
from oracle import llsa_oracle as orc
from paper_2512_16615_amd import inputs, llsa

pytestmark = pytest.mark.gpu


def _make_inputs_parallel(cfg, seed, threads=8):
    out = {n: np.empty((cfg["batch"], cfg["heads"], cfg["N"], cfg["d"]), np.float32) for n in ("Q", "K", "V", "dO")}
    jobs = [(n, b, h) for n in out for b in range(cfg["batch"]) for h in range(cfg["heads"])]

    def one(job):
        n, b, h = job
        x = inputs.make_head(cfg["kind"], seed, n, b, h, cfg["N"], cfg["d"])
        out[n][b, h] = orc.to_bf16(x) if cfg["dtype"] == "bf16" else x

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(one, jobs))
    return out


def _properties_all_heads(cfg, gpu, x):
    """Checks that need no oracle: valid index lists, gradient sum identities."""
    plan, g = gpu["plan"], H.geometry(cfg)
    for l in range(g.L):
        I = plan.level_indices(gpu["indices"], l)
        assert bool((I[..., 1:] > I[..., :-1]).all()) if I.shape[-1] > 1 else True
        assert int(I.min()) >= 0 and int(I.max()) < g.n(l + 1)
        if l + 1 < g.L:        # every pick is a child of a pick of the parent row
            par = plan.level_indices(gpu["indices"], l + 1)                       # [b, h, rows/16, K]
            parent_of_pick = (I // cfg["B"]).unsqueeze(-1)                         # [b, h, rows, K, 1]
            rows = I.shape[2]
            par_rows = par[:, :, torch.arange(rows, device=I.device) // cfg["B"]]  # [b, h, rows, Kp]
            assert bool((parent_of_pick == par_rows.unsqueeze(-2)).any(-1).all())
    assert bool(torch.isfinite(gpu["LSE"]).all()) and bool(torch.isfinite(gpu["O"].float()).all())
    dO, dV = gpu["dO"].float(), gpu["dV"].float()
    s_ref, s_got = dO.sum(dim=2), dV.sum(dim=2)                                    # [b, h, d]
    scale = dO.abs().sum(dim=2)
    assert float(((s_ref - s_got).abs() / scale).max()) < 2e-3, "sum_t dV[t] != sum_q dO[q]"
    lhs = (gpu["dQ"].float() * gpu["Q"].float()).sum(dim=(2, 3))
    rhs = (gpu["dK"].float() * gpu["K"].float()).sum(dim=(2, 3))
    norm = (gpu["dQ"].float().abs() * gpu["Q"].float().abs()).sum(dim=(2, 3))
    assert float(((lhs - rhs).abs() / norm).max()) < 5e-3, "<dQ,Q> != <dK,K>"


def _sampled_parity(cfg, gpu, x, heads, n_row_chunks=6, chunk=32, full_backward_head=None):
    g = H.geometry(cfg)
    tol = H.TOL[cfg["dtype"]]
    rng = np.random.default_rng(1234)
    for (b, h) in heads:
        Qp, Kp, Vp = (orc.pyramid(x[n][b, h], g, cfg["dtype"] == "bf16") for n in ("Q", "K", "V"))
        ref = {"Qp": Qp, "Kp": Kp, "Vp": Vp, "I": orc.select_all(Qp, Kp, g)}
        H.check_pyramid(cfg, gpu, ref, b, h)
        free_diff, excused = H.check_indices(cfg, gpu, ref, b, h, x)
        assert excused == 0 and free_diff == 0
        idx = orc.cat_indices(ref["I"])
        Kc, Vc = orc.cat_pyramid(Kp), orc.cat_pyramid(Vp)
        starts = sorted(set([0, g.N - chunk] + [int(s) for s in rng.integers(0, g.N - chunk, n_row_chunks)]))
        for s0 in starts:
            o, lse = orc.attn_fwd(x["Q"][b, h], Kc, Vc, idx, g, g.L, rows=(s0, s0 + chunk))
            dq, _, _ = orc.attn_bwd(x["Q"][b, h], Kc, Vc, idx, x["dO"][b, h], g, g.L, rows=(s0, s0 + chunk))
            sl = slice(s0, s0 + chunk)
            H.check_close(f"O{(b, h, s0)}", H.f32(gpu["O"][b, h, sl]), o[sl], tol["out"])
            H.check_close(f"LSE{(b, h, s0)}", H.f32(gpu["LSE"][b, h, sl]), lse[sl], tol["lse"])
            H.check_close(f"dQ{(b, h, s0)}", H.f32(gpu["dQ"][b, h, sl]), dq[sl], tol["out"])
        if full_backward_head == (b, h):
            bw = orc.backward(x["Q"][b, h], Kp, Vp, idx, x["dO"][b, h], g)
            for name in ("dQ", "dK", "dV"):
                err = H.check_close(f"{name}{(b, h)}", H.f32(gpu[name][b, h]), bw[name], tol["out"])
                print(f"{cfg['name']} full-head {name} max-abs err {err:.3e}")


def test_headline_n65536_sampled():
    """BASELINE configs[3]: 16 heads, d=64, N=65536, B=16, K=8, L=3, smooth inputs; and the Gaussian control."""
    cfg = inputs.CONFIGS[3]
    x = _make_inputs_parallel(cfg, inputs.config_seed(3))
    gpu = H.gpu_forward_backward(cfg, x)
    _properties_all_heads(cfg, gpu, x)
    _sampled_parity(cfg, gpu, x, heads=[(0, 0), (0, 11)], full_backward_head=(0, 11))


def test_headline_gaussian_control():
    cfg = dict(inputs.CONFIGS[3], kind="gaussian", heads=4)
    x = _make_inputs_parallel(cfg, inputs.config_seed(3) + 100)
    gpu = H.gpu_forward_backward(cfg, x)
    _properties_all_heads(cfg, gpu, x)
    _sampled_parity(cfg, gpu, x, heads=[(0, 3)], n_row_chunks=3)


@pytest.mark.parametrize("K", [4, 8, 16])
def test_config2_n16384_k_sweep(K):
    """BASELINE configs[2]: batch 2, 16 heads, N=16384, L=3 (top level of 4 tokens), K in {4, 8, 16}."""
    cfg = dict(inputs.CONFIGS[2], K=K)
    x = _make_inputs_parallel(cfg, inputs.config_seed(2))
    gpu = H.gpu_forward_backward(cfg, x)
    _properties_all_heads(cfg, gpu, x)
    _sampled_parity(cfg, gpu, x, heads=[(1, 5)], n_row_chunks=3, full_backward_head=(1, 5))


def test_config4_extreme_n262144_d128():
    """BASELINE configs[4]: 8 heads, d=128, N=262144, B=16, K=16, L=4; also reports the HBM footprint of the
    indices, logsumexp and pooled levels."""
    cfg = inputs.CONFIGS[4]
    x = _make_inputs_parallel(cfg, inputs.config_seed(4))
    gpu = H.gpu_forward_backward(cfg, x)
    plan = gpu["plan"]
    print(f"config4 footprint: indices {plan.indices_bytes() / 2**20:.1f} MiB, LSE {gpu['LSE'].numel() * 4 / 2**20:.1f} MiB, "
          f"pooled levels (fwd workspace) {plan.workspace_bytes(False) / 2**20:.1f} MiB, backward workspace "
          f"{plan.workspace_bytes(True) / 2**20:.1f} MiB, one input tensor {gpu['Q'].numel() * 2 / 2**20:.1f} MiB")
    _properties_all_heads(cfg, gpu, x)
    _sampled_parity(cfg, gpu, x, heads=[(0, 2)], n_row_chunks=2)
