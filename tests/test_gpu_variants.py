"""GPU parity on the shapes of the paper's scaling and ablation studies (Fig. 4, Table 5), beyond the benchmark's five
configurations: longer sequences at the d = 64 head geometry, the paper's own choice of the number of levels
(L = 2 at 256 x 256), a single coarse level (L = 1, the prior single-level Top-K design), partial enrichment
(L_e < L), larger K, and the paper's other block size, 64.  Same bars as the other parity tests.
"""
import pytest

from tests import harness as H
from paper_2512_16615_amd import inputs

pytestmark = pytest.mark.gpu

BASE = dict(batch=1, d=64, B=16, K=8, dtype="bf16", kind="smooth")


def _run(cfg, seed, heads, **kw):
    x = H.make_inputs_parallel(cfg, seed)
    gpu = H.gpu_forward_backward(cfg, x)
    H.properties_all_heads(cfg, gpu, x)
    H.sampled_parity(cfg, gpu, x, heads=heads, **kw)


@pytest.mark.parametrize("L", [1, 2])
def test_n65536_fewer_levels(L):
    """N = 65536 with L = 2 (the paper's setting at 256 x 256: 8 + 8 + 16 key blocks per query) and L = 1 (one coarse
    level of 4096 tokens, scored densely)."""
    cfg = dict(BASE, name=f"n65536_L{L}", N=65536, heads=2, L=L)
    _run(cfg, 0x115A2000 + L, heads=[(0, 1)], n_row_chunks=3, full_backward_head=(0, 1))


@pytest.mark.parametrize("Le", [0, 1, 2])
def test_n16384_partial_enrichment(Le):
    """Levels 0..L_e only in the list (L_e = 0: no coarse token at all)."""
    cfg = dict(BASE, name=f"n16384_Le{Le}", N=16384, heads=4, L=3, Le=Le)
    _run(cfg, 0x115A2010, heads=[(0, 2)], n_row_chunks=3, full_backward_head=(0, 2))


def test_n65536_K32():
    cfg = dict(BASE, name="n65536_K32", N=65536, heads=2, L=3, K=32)
    _run(cfg, 0x115A2020, heads=[(0, 0)], n_row_chunks=3, full_backward_head=(0, 0))


@pytest.mark.timeout(400)
def test_n262144_d64_L4():
    cfg = dict(BASE, name="n262144_d64", N=262144, heads=2, L=4)
    _run(cfg, 0x115A2030, heads=[(0, 1)], n_row_chunks=3, full_backward_head=(0, 1))


@pytest.mark.timeout(600)
def test_n262144_single_level():
    """The single-level method at 512 x 512 tokens: 16384 coarse tokens, every one a selection candidate and a key of
    the dense level (the quadratic regime the paper's hierarchy removes)."""
    cfg = dict(BASE, name="n262144_L1", N=262144, heads=1, L=1)
    _run(cfg, 0x115A2035, heads=[(0, 0)], n_row_chunks=1)


@pytest.mark.timeout(600)
def test_n1048576_d64_L4():
    """1024 x 1024 pixel tokens, one head: 16^5 tokens, L = 4, coarsest level of 16 tokens."""
    cfg = dict(BASE, name="n1048576_d64", N=1048576, heads=1, L=4)
    _run(cfg, 0x115A2040, heads=[(0, 0)], n_row_chunks=2)


@pytest.mark.timeout(600)
def test_n1048576_K16_two_upper_launches():
    """K = 16 at L = 4: 32 listed blocks at levels 2 and 3, which the upper-level dK/dV kernel takes in two launches."""
    cfg = dict(BASE, name="n1048576_K16", N=1048576, heads=1, L=4, K=16)
    _run(cfg, 0x115A2070, heads=[(0, 0)], n_row_chunks=2)


def test_block_size_64():
    """B = 64 (the larger block of the paper's efficiency comparison): N = 16384 -> 256 -> 4 tokens, L = 2."""
    cfg = dict(BASE, name="n16384_B64", N=16384, heads=2, B=64, K=4, L=2)
    _run(cfg, 0x115A2050, heads=[(0, 1)], n_row_chunks=3, full_backward_head=(0, 1))


# ---- index reordering (Sec. 5.1): the tokens of a pixel grid in nested-patch order

@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_index_reordering_matches_oracle(dtype):
    import numpy as np
    import torch
    from oracle import llsa_oracle as orc
    from paper_2512_16615_amd import llsa
    rng = np.random.default_rng(7)
    bh, N, d = 3, 4096, 64
    x = rng.standard_normal((bh, N, d)).astype(np.float32)
    if dtype == "bf16":
        x = orc.to_bf16(x)
    dev = torch.from_numpy(x).cuda()
    dev = dev.to(torch.bfloat16) if dtype == "bf16" else dev
    fwd = llsa.reorder(dev)
    back = llsa.reorder(fwd, inverse=True)
    torch.cuda.synchronize()
    for h in range(bh):
        assert np.array_equal(fwd[h].float().cpu().numpy(), orc.reorder(x[h])), "forward order differs from the oracle"
    assert torch.equal(back, dev)
    with pytest.raises(llsa.LlsaError):                      # 2048 tokens are not a square power-of-two grid
        llsa.reorder(dev[:, :2048].contiguous())
    with pytest.raises(llsa.LlsaError):                      # in place is refused
        llsa.reorder(dev, out=dev)


def test_layer_on_reordered_tokens():
    """The layer on nested-patch token order (what the paper's DiT feeds it): inputs reordered on the GPU equal the
    oracle's reordering, and forward + backward on them meet the usual bars (16 consecutive tokens = a 4 x 4 patch)."""
    import numpy as np
    import torch
    from oracle import llsa_oracle as orc
    from paper_2512_16615_amd import llsa
    cfg = dict(BASE, name="n16384_nested", N=16384, heads=2, L=3)
    raster = H.make_inputs_parallel(cfg, 0x115A2060)
    nested = {n: np.stack([np.stack([orc.reorder(v[b, h]) for h in range(cfg["heads"])]) for b in range(cfg["batch"])])
              for n, v in raster.items()}
    for n in raster:
        got = llsa.reorder(H.to_dev(raster[n], cfg))
        assert torch.equal(got, H.to_dev(nested[n], cfg)), n
    gpu = H.gpu_forward_backward(cfg, nested)
    H.properties_all_heads(cfg, gpu, nested)
    H.sampled_parity(cfg, gpu, nested, heads=[(0, 1)], n_row_chunks=3, full_backward_head=(0, 1))


def test_level1_partials_carried_across_query_blocks():
    """Level-1 dK/dV where one workgroup walks 8 consecutive level-1 query blocks and carries a key block's sums in
    registers while the following query blocks keep listing it (64 heads x 64 level-1 query blocks: enough work for
    that kernel to be chosen).  Lists are forced (Alg. 1 allows any valid rows) so that the cases are certain to
    occur: alternating disjoint rows (a block dropped and taken up again inside one walk), a window sliding by one
    block per row, identical rows, rows whose new blocks sort before the ones kept, random rows."""
    import numpy as np
    import torch
    from oracle import llsa_oracle as orc
    from paper_2512_16615_amd import llsa
    cfg = dict(BASE, name="n16384_forced_lists", N=16384, batch=4, heads=16, L=3)
    g = H.geometry(cfg)
    two = H.make_inputs_parallel(dict(cfg, batch=1, heads=2), 0xC4A1)             # two distinct heads, repeated
    x = {n: np.ascontiguousarray(np.tile(v, (4, 8, 1, 1))) for n, v in two.items()}
    plan = H.make_plan(cfg)
    Q, K, V, dO = (H.to_dev(x[n], cfg) for n in ("Q", "K", "V", "dO"))
    ws, idx = plan.alloc_workspace(True), plan.alloc_indices()
    llsa.pool(plan, Q, K, V, ws)

    rng = np.random.default_rng(77)
    def rows(n_rows, n_keys, k):
        return np.stack([np.sort(rng.choice(n_keys, k, replace=False)) for _ in range(n_rows)]).astype(np.int32)
    A, Bs = np.arange(8), np.arange(8, 16)
    I1 = []
    for h in range(2):
        r = rows(g.n(2), g.n(2), 8)
        if h == 0:
            r[0:8] = np.stack([A, Bs, A, Bs, A, A, Bs, Bs])
            r[8:16] = np.stack([np.arange(i, i + 8) for i in range(8)])
            r[16:24] = np.array([3, 9, 17, 20, 33, 41, 50, 63])
            r[24:32] = np.stack([np.arange(40 - i, 48 - i) for i in range(8)])
        I1.append(r)
    I = [[rows(g.n(1), g.n(1), 8), I1[h], np.tile(np.arange(4, dtype=np.int32), (g.n(3), 1))] for h in range(2)]
    for l in range(3):
        lev = torch.from_numpy(np.stack([I[h][l] for h in range(2)])).cuda().repeat(4, 8, 1, 1)
        plan.level_indices(idx, l).copy_(lev)
    O, LSE = llsa.attention(plan, Q, K, V, idx, ws)
    dQ, dK, dV = llsa.backward(plan, Q, K, V, O, LSE, idx, dO, ws)
    torch.cuda.synchronize()
    tol = H.TOL["bf16"]
    for (b, h) in ((0, 0), (3, 15)):
        Kp, Vp = orc.pyramid(x["K"][b, h], g, True), orc.pyramid(x["V"][b, h], g, True)
        idx_cat = orc.cat_indices(I[h % 2])
        o, lse = orc.attn_fwd(x["Q"][b, h], orc.cat_pyramid(Kp), orc.cat_pyramid(Vp), idx_cat, g, 3)
        H.check_close(f"O{(b, h)}", H.f32(O[b, h]), o, tol["out"], tol["ulp"])
        H.check_close(f"LSE{(b, h)}", H.f32(LSE[b, h]), lse, tol["lse"])
        bw = H.oracle_backward_threads(x["Q"][b, h], Kp, Vp, idx_cat, x["dO"][b, h], g, 3)
        for name, got in (("dQ", dQ), ("dK", dK), ("dV", dV)):
            H.check_close(f"{name}{(b, h)}", H.f32(got[b, h]), bw[name], tol["out"], tol["ulp"])
    # all copies of a head get bit-identical gradients (different workgroups, same arithmetic)
    for t_ in (dK, dV):
        assert torch.equal(t_[0, 0], t_[3, 14]) and torch.equal(t_[0, 1], t_[2, 7])
