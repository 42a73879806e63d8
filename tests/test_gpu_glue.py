"""GPU parity of the layer glue fused with pooling (llsa_qknorm_rope_pool) and of llsa_forward_pooled.

  * Qout, Kout against the oracle's fp64 QK-Norm + RoPE: within one unit in the last place of the I/O type plus a
    small absolute term (the GPU works in fp32 and rounds once; a value that falls near a rounding boundary may
    round the other way) -- a decision taken in floating point, so the pooled levels, which depend on those rounded
    values, are compared teacher-forced: bit-exact against the oracle's pooling of the GPU's own Qout / Kout;
  * V's pooled levels: bit-exact;
  * llsa_forward_pooled on that workspace: bit-identical to llsa_forward on (Qout, Kout, V), and O within the usual
    bound of the oracle's layer on the same tensors.
"""
import numpy as np
import pytest
import torch

from oracle import llsa_oracle as orc
from paper_2512_16615_amd import inputs, llsa
from tests import harness as H

pytestmark = pytest.mark.gpu

CASES = [
    dict(name="glue_bf16", batch=1, heads=3, d=64, N=4096, B=16, K=8, L=2, dtype="bf16", kind="smooth"),
    dict(name="glue_bf16_d128", batch=2, heads=2, d=128, N=4096, B=16, K=4, L=2, dtype="bf16", kind="gaussian"),
    dict(name="glue_f32_b4", batch=1, heads=2, d=32, N=1024, B=4, K=2, L=3, dtype="f32", kind="gaussian"),
    dict(name="glue_bf16_b6_1d", batch=1, heads=2, d=16, N=432, B=6, K=2, L=2, dtype="bf16", kind="gaussian"),
]


@pytest.mark.parametrize("cfg", CASES, ids=[c["name"] for c in CASES])
def test_qknorm_rope_pool_matches_oracle(cfg):
    bf16 = cfg["dtype"] == "bf16"
    x = H.make_inputs(cfg, 0x115A3000)
    x = {n: v * (3.0 if n in ("Q", "K") else 1.0) for n, v in x.items()}        # pre-norm activations are not unit scale
    if bf16:
        x = {n: orc.to_bf16(v) for n, v in x.items()}
    cos, sin = inputs.rope_tables(cfg["N"], cfg["d"])
    gq, gk = inputs.norm_gain(1, "Q", cfg["d"]), inputs.norm_gain(1, "K", cfg["d"])
    plan = H.make_plan(cfg)
    Qpre, Kpre, V = (H.to_dev(x[n], cfg) for n in ("Q", "K", "V"))
    dev = lambda a: torch.from_numpy(a).cuda()
    eps = 1e-6
    Qout, Kout, ws = llsa.qknorm_rope_pool(plan, Qpre, Kpre, V, dev(gq), dev(gk), dev(cos), dev(sin), eps)
    torch.cuda.synchronize()
    g = H.geometry(cfg)
    ulp = 2.0 ** -8 if bf16 else 2.0 ** -23
    for b in range(cfg["batch"]):
        for h in range(cfg["heads"]):
            for name, pre, got, gam, tensor in (("Q", x["Q"], Qout, gq, 0), ("K", x["K"], Kout, gk, 1)):
                ref = orc.qknorm_rope(pre[b, h], gam, cos, sin, eps)
                out = H.f32(got[b, h])
                err = np.abs(out.astype(np.float64) - ref)
                assert (err <= ulp * np.abs(ref) + 1e-6).all(), f"{name}out {(b, h)}: max err {err.max():.3e}"
                lev = orc.pyramid(out, g, bf16)                       # teacher-forced: pool what the GPU wrote
                for l in range(1, g.L + 1):
                    assert np.array_equal(H.f32(plan.pyramid_level(ws, tensor, l)[b, h]), lev[l]), f"{name} level {l}"
            lev = orc.pyramid(x["V"][b, h], g, bf16)
            for l in range(1, g.L + 1):
                assert np.array_equal(H.f32(plan.pyramid_level(ws, 2, l)[b, h]), lev[l]), f"V level {l}"
    # the layer on the glued tensors: same results with and without its own compression loop
    O1, LSE1, idx1 = llsa.forward_pooled(plan, Qout, Kout, V, ws)
    O2, LSE2, idx2, _ = llsa.forward(plan, Qout, Kout, V)
    torch.cuda.synchronize()
    assert torch.equal(idx1, idx2) and torch.equal(LSE1, LSE2)
    assert torch.equal(O1.view(torch.int16 if bf16 else torch.int32), O2.view(torch.int16 if bf16 else torch.int32))
    tol = H.TOL[cfg["dtype"]]
    f = orc.forward(H.f32(Qout[0, 0]), H.f32(Kout[0, 0]), x["V"][0, 0], g, bf16=bf16)
    assert all(np.array_equal(plan.level_indices(idx1, l)[0, 0].cpu().numpy(), f["I"][l]) for l in range(g.L))
    H.check_close("O_glued(0, 0)", H.f32(O1[0, 0]), f["O"], tol["out"])
    H.check_close("LSE_glued(0, 0)", H.f32(LSE1[0, 0]), f["LSE"], tol["lse"])


# ---- key/value backward of level 0 with its lists from Alg. 2 or from a dense block mask (Sec. 5.4, Fig. 4)

@pytest.mark.parametrize("cfg", [
    dict(name="kv0_n4096", batch=1, heads=2, d=64, N=4096, B=16, K=8, L=2, dtype="bf16", kind="smooth"),
    dict(name="kv0_n16384_d128", batch=1, heads=1, d=128, N=16384, B=16, K=4, L=3, dtype="bf16", kind="gaussian"),
    dict(name="kv0_b32_odd_T", batch=1, heads=1, d=64, N=3072, B=32, K=4, L=1, dtype="bf16", kind="gaussian"),
], ids=lambda c: c["name"])
def test_kv_backward_level0_csc_and_mask_agree_with_the_oracle(cfg):
    x = H.make_inputs(cfg, 0x115A3100)
    gpu = H.gpu_forward_backward(cfg, x)
    plan, g = gpu["plan"], H.geometry(cfg)
    args = (gpu["Q"], gpu["K"], gpu["V"], gpu["dO"], gpu["LSE"], gpu["indices"], gpu["ws"])
    dK_c, dV_c, _ = llsa.kv_backward_level0(plan, False, *args)
    C_csc, Iq_csc = (t.clone() for t in plan.csc_level(gpu["ws"], 0))
    dK_m, dV_m, mask = llsa.kv_backward_level0(plan, True, *args)
    C_m, Iq_m = plan.csc_level(gpu["ws"], 0)
    torch.cuda.synchronize()
    # the mask holds exactly the listed pairs, and scanning it gives the very lists of Alg. 2 (ascending rows)
    T = g.n(1)
    I0 = plan.level_indices(gpu["indices"], 0)
    m = mask[: cfg["batch"] * cfg["heads"] * T * T].view(cfg["batch"], cfg["heads"], T, T)      # [key block, query block]
    assert int(m.sum()) == I0.numel()
    for h in range(cfg["heads"]):
        rows = torch.arange(T, device="cuda").repeat_interleave(I0.shape[-1])
        assert bool(m[0, h][I0[0, h].reshape(-1).long(), rows].all())
    assert torch.equal(C_m, C_csc) and torch.equal(Iq_m, Iq_csc)
    assert torch.equal(dK_m.view(torch.int16), dK_c.view(torch.int16)) and torch.equal(dV_m.view(torch.int16), dV_c.view(torch.int16))
    # and the gradient is level 0's share of the oracle's backward (rows 0..N-1 of the pyramid gradient, not un-pooled)
    ref = H.oracle_head(cfg, x, 0, 0)
    H.check_close("dK0(0, 0)", H.f32(dK_c[0, 0]), ref["dKpyr"][: g.N], 2e-2)
    H.check_close("dV0(0, 0)", H.f32(dV_c[0, 0]), ref["dVpyr"][: g.N], 2e-2)
