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
