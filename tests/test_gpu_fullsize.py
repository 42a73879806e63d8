"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot run these shapes whole in a test's time, so per configuration:
  * pooled levels and selection indices: bit-exact on a few heads (selection is cheap for the oracle);
  * O / LSE / dQ: element-wise on sampled query rows of those heads (each row is an independent oracle call);
  * dK / dV: element-wise on one whole head (the oracle's backward of that head runs as disjoint ranges of query
    rows on the host threads, the fp64 shares summed), and on every head via
    properties that hold at any size: sum_t dV[t] = sum_q dO[q] and <dQ, Q> = <dK, K> (Euler identity of the
    bilinear logits; exact up to the bf16 rounding of the pooled levels and outputs).
"""
import pytest

from tests import harness as H
from paper_2512_16615_amd import inputs

pytestmark = pytest.mark.gpu


def test_headline_n65536_sampled():
    """BASELINE configs[3]: 16 heads, d=64, N=65536, B=16, K=8, L=3, smooth inputs; and the Gaussian control."""
    cfg = inputs.CONFIGS[3]
    x = H.make_inputs_parallel(cfg, inputs.config_seed(3))
    gpu = H.gpu_forward_backward(cfg, x)
    H.properties_all_heads(cfg, gpu, x)
    H.sampled_parity(cfg, gpu, x, heads=[(0, 0), (0, 11)], full_backward_head=(0, 11))


def test_headline_gaussian_control():
    cfg = dict(inputs.CONFIGS[3], kind="gaussian", heads=4)
    x = H.make_inputs_parallel(cfg, inputs.config_seed(3) + 100)
    gpu = H.gpu_forward_backward(cfg, x)
    H.properties_all_heads(cfg, gpu, x)
    H.sampled_parity(cfg, gpu, x, heads=[(0, 3)], n_row_chunks=3)


@pytest.mark.parametrize("K", [4, 8, 16])
def test_config2_n16384_k_sweep(K):
    """BASELINE configs[2]: batch 2, 16 heads, N=16384, L=3 (top level of 4 tokens), K in {4, 8, 16}."""
    cfg = dict(inputs.CONFIGS[2], K=K)
    x = H.make_inputs_parallel(cfg, inputs.config_seed(2))
    gpu = H.gpu_forward_backward(cfg, x)
    H.properties_all_heads(cfg, gpu, x)
    H.sampled_parity(cfg, gpu, x, heads=[(1, 5)], n_row_chunks=3, full_backward_head=(1, 5))


def test_config4_extreme_n262144_d128():
    """BASELINE configs[4]: 8 heads, d=128, N=262144, B=16, K=16, L=4; also reports the HBM footprint of the
    indices, logsumexp and pooled levels."""
    cfg = inputs.CONFIGS[4]
    x = H.make_inputs_parallel(cfg, inputs.config_seed(4))
    gpu = H.gpu_forward_backward(cfg, x)
    plan = gpu["plan"]
    print(f"config4 footprint: indices {plan.indices_bytes() / 2**20:.1f} MiB, LSE {gpu['LSE'].numel() * 4 / 2**20:.1f} MiB, "
          f"pooled levels (fwd workspace) {plan.workspace_bytes(False) / 2**20:.1f} MiB, backward workspace "
          f"{plan.workspace_bytes(True) / 2**20:.1f} MiB, one input tensor {gpu['Q'].numel() * 2 / 2**20:.1f} MiB")
    H.properties_all_heads(cfg, gpu, x)
    H.sampled_parity(cfg, gpu, x, heads=[(0, 2)], n_row_chunks=2, full_backward_head=(0, 2))
