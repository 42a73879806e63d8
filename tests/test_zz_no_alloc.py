"""llsa_forward_static (the forward pass on the library's static device workspace, for callers that cannot
allocate) against llsa_forward, through the C ABI: same kernels, so every output must be bit-identical.
Two calls in a row on the same GPU, the second on a smaller problem, so that whatever the first call left in
the shared array is seen to do no harm; then the first problem again."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2512_16615_amd import inputs, llsa
from tests import harness as H

pytestmark = pytest.mark.gpu

CASES = [dict(name="static_a", batch=1, heads=4, d=64, N=16384, B=16, K=8, L=3, dtype="bf16", kind="smooth"),
         dict(name="static_b", batch=1, heads=2, d=64, N=4096, B=16, K=8, L=2, dtype="bf16", kind="smooth"),
         dict(name="static_a", batch=1, heads=4, d=64, N=16384, B=16, K=8, L=3, dtype="bf16", kind="smooth")]


def _vp(t):
    return ctypes.c_void_p(t.data_ptr())


def test_forward_static_equals_forward_two_calls_in_a_row():
    lib = llsa.load()
    assert lib.llsa_static_workspace_bytes() == 32 << 20
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for ci, cfg in enumerate(CASES):
        x = H.make_inputs(cfg, 4242 + ci)
        Q, K, V = (H.to_dev(x[n], cfg) for n in ("Q", "K", "V"))
        plan = H.make_plan(cfg)
        assert plan.workspace_bytes(False) <= lib.llsa_static_workspace_bytes()
        # reference: the existing entry point on a caller-owned workspace
        O_ref, LSE_ref, idx_ref, _ = llsa.forward(plan, Q, K, V)
        # every buffer of the static call exists before it; poisoned so that stale contents cannot pass
        O = torch.full_like(Q, float("nan"))
        LSE = torch.full((cfg["batch"], cfg["heads"], cfg["N"]), float("nan"), dtype=torch.float32, device="cuda")
        idx = torch.full((plan.indices_bytes() // 4,), -1, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        st = lib.llsa_forward_static(plan._h, _vp(Q), _vp(K), _vp(V), _vp(O), _vp(LSE), _vp(idx), stream)
        assert st == 0, lib.llsa_status_string(st).decode()
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(idx, idx_ref), f"{cfg['name']} call {ci}: indices differ"
        assert torch.equal(LSE, LSE_ref), f"{cfg['name']} call {ci}: LSE differs"
        assert torch.equal(O.view(torch.int16), O_ref.view(torch.int16)), f"{cfg['name']} call {ci}: O differs"
        print(f"forward_static call {ci} ({cfg['name']}, N={cfg['N']}): bit-identical to llsa_forward", flush=True)


def test_forward_static_refuses_a_plan_beyond_the_static_workspace():
    lib = llsa.load()
    cfg = inputs.CONFIGS[4]                      # pooled levels of 8 heads x 262144 tokens x d=128: about 102 MiB
    plan = H.make_plan(cfg)
    assert plan.workspace_bytes(False) > lib.llsa_static_workspace_bytes()
    one = torch.zeros(16, dtype=torch.int32, device="cuda")       # never touched: the size check comes first
    st = lib.llsa_forward_static(plan._h, _vp(one), _vp(one), _vp(one), _vp(one), _vp(one), _vp(one), None)
    assert st == 4
    assert b"static" in lib.llsa_status_string(st)


def test_forward_static_replays_from_a_hip_graph():
    """What the entry point is for: captured into a HIP graph (after one eager call, which looks the static array's
    address up), every replay -- with eager work of the program and synchronisations between the replays -- gives the
    eager result bit for bit."""
    cfg = CASES[1]
    x = H.make_inputs(cfg, 4250)
    Q, K, V = (H.to_dev(x[n], cfg) for n in ("Q", "K", "V"))
    plan = H.make_plan(cfg)
    O = torch.empty_like(Q)
    LSE = torch.empty(cfg["batch"], cfg["heads"], cfg["N"], dtype=torch.float32, device="cuda")
    idx = plan.alloc_indices()
    llsa.forward_static(plan, Q, K, V, O, LSE, idx)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (O, LSE, idx)]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            llsa.forward_static(plan, Q, K, V, O, LSE, idx)
    torch.cuda.current_stream().wait_stream(side)
    other = H.make_plan(CASES[0])                                  # another problem uses the shared array in between
    xo = H.make_inputs(CASES[0], 4251)
    Qo, Ko, Vo = (H.to_dev(xo[n], CASES[0]) for n in ("Q", "K", "V"))
    Oo, LSEo, idxo = torch.empty_like(Qo), torch.empty(1, 4, 16384, dtype=torch.float32, device="cuda"), other.alloc_indices()
    for rep in range(3):
        O.zero_()
        LSE.zero_()
        idx.fill_(-1)
        llsa.forward_static(other, Qo, Ko, Vo, Oo, LSEo, idxo)     # overwrites the static workspace
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("O", "LSE", "indices"), (O, LSE, idx), ref):
            assert torch.equal(got, want), f"replay {rep}: {name} differs from the eager result"
