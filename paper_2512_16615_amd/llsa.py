"""Thin ctypes binding of ``libllsa.so`` (see ``include/llsa.h``).

Argument marshalling only: PyTorch owns the device memory and the stream, every
step of the path runs in the library's HIP kernels.  There is no fallback: if
the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libllsa.so")
_lib = None

F32, BF16 = 0, 1


class LlsaError(RuntimeError):
    pass


class _Desc(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("N", ctypes.c_int64), ("d", ctypes.c_int32),
                ("B", ctypes.c_int32), ("K", ctypes.c_int32), ("L", ctypes.c_int32), ("Le", ctypes.c_int32),
                ("sm_scale", ctypes.c_float), ("dtype", ctypes.c_int32), ("reweight", ctypes.c_int32),
                ("bwd_repool", ctypes.c_int32), ("kernel_path", ctypes.c_int32), ("single_stream", ctypes.c_int32)]


EXPORTS = ["llsa_plan", "llsa_plan_destroy", "llsa_plan_workspace_bytes", "llsa_plan_indices_bytes",
           "llsa_plan_level_info", "llsa_plan_pyramid_info", "llsa_plan_csc_info", "llsa_forward", "llsa_backward",
           "llsa_pool", "llsa_select_level", "llsa_attention", "llsa_index_transpose", "llsa_reorder", "llsa_status_string",
           "llsa_stage_count", "llsa_stage_name", "llsa_stage_timing_begin", "llsa_stage_timing_end",
           "llsa_static_workspace_bytes", "llsa_forward_static", "llsa_qknorm_rope_pool", "llsa_forward_pooled",
           "llsa_kv_backward_mask_bytes", "llsa_kv_backward_level0", "llsa_calibrate_mfma", "llsa_calibrate_copy"]


def load():
    """Load the library built by ``paper_2512_16615_amd.build``; raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise LlsaError(f"{LIB_PATH} not found: run `python -m paper_2512_16615_amd.build` (needs hipcc)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    lib.llsa_plan.argtypes = [ctypes.POINTER(_Desc), ctypes.POINTER(vp)]
    lib.llsa_plan.restype = ctypes.c_int
    lib.llsa_plan_destroy.argtypes = [vp]
    lib.llsa_plan_destroy.restype = None
    lib.llsa_plan_workspace_bytes.argtypes = [vp, ctypes.c_int]
    lib.llsa_plan_workspace_bytes.restype = sz
    lib.llsa_plan_indices_bytes.argtypes = [vp]
    lib.llsa_plan_indices_bytes.restype = sz
    lib.llsa_plan_level_info.argtypes = [vp, i32, ctypes.POINTER(i64), ctypes.POINTER(i32), ctypes.POINTER(sz)]
    lib.llsa_plan_level_info.restype = i32
    lib.llsa_plan_pyramid_info.argtypes = [vp, i32, i32, ctypes.POINTER(i64), ctypes.POINTER(sz)]
    lib.llsa_plan_pyramid_info.restype = i32
    lib.llsa_plan_csc_info.argtypes = [vp, i32, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.llsa_plan_csc_info.restype = i32
    lib.llsa_forward.argtypes = [vp] * 9
    lib.llsa_forward.restype = ctypes.c_int
    lib.llsa_forward_static.argtypes = [vp] * 8
    lib.llsa_forward_static.restype = ctypes.c_int
    lib.llsa_static_workspace_bytes.argtypes = []
    lib.llsa_static_workspace_bytes.restype = sz
    lib.llsa_forward_pooled.argtypes = [vp] * 9
    lib.llsa_forward_pooled.restype = ctypes.c_int
    lib.llsa_qknorm_rope_pool.argtypes = [vp] * 8 + [ctypes.c_float] + [vp] * 4
    lib.llsa_qknorm_rope_pool.restype = ctypes.c_int
    lib.llsa_kv_backward_mask_bytes.argtypes = [vp]
    lib.llsa_kv_backward_mask_bytes.restype = sz
    lib.llsa_kv_backward_level0.argtypes = [vp, i32] + [vp] * 11
    lib.llsa_kv_backward_level0.restype = ctypes.c_int
    lib.llsa_calibrate_mfma.argtypes = [vp, i32, i32, vp]
    lib.llsa_calibrate_mfma.restype = ctypes.c_int
    lib.llsa_calibrate_copy.argtypes = [vp, vp, i64, vp]
    lib.llsa_calibrate_copy.restype = ctypes.c_int
    lib.llsa_backward.argtypes = [vp] * 13
    lib.llsa_backward.restype = ctypes.c_int
    lib.llsa_pool.argtypes = [vp] * 6
    lib.llsa_pool.restype = ctypes.c_int
    lib.llsa_select_level.argtypes = [vp, i32, vp, vp, vp, vp]
    lib.llsa_select_level.restype = ctypes.c_int
    lib.llsa_attention.argtypes = [vp] * 9
    lib.llsa_attention.restype = ctypes.c_int
    lib.llsa_index_transpose.argtypes = [vp] * 4
    lib.llsa_index_transpose.restype = ctypes.c_int
    lib.llsa_reorder.argtypes = [i64, i64, i32, i32, i32, vp, vp, vp]
    lib.llsa_reorder.restype = ctypes.c_int
    lib.llsa_stage_count.argtypes = []
    lib.llsa_stage_count.restype = i32
    lib.llsa_stage_name.argtypes = [i32]
    lib.llsa_stage_name.restype = ctypes.c_char_p
    lib.llsa_stage_timing_begin.argtypes = [i32, i32]
    lib.llsa_stage_timing_begin.restype = ctypes.c_int
    lib.llsa_stage_timing_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
    lib.llsa_stage_timing_end.restype = ctypes.c_int
    lib.llsa_status_string.argtypes = [ctypes.c_int]
    lib.llsa_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(st: int, what: str):
    if st != 0:
        raise LlsaError(f"{what}: {load().llsa_status_string(st).decode()} (status {st})")


def _ptr(t: torch.Tensor | None):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


@dataclass
class LevelInfo:
    rows: int
    K_l: int
    byte_offset: int


class Plan:
    """``llsa_plan``: validated problem description, level table and buffer sizes (host only)."""

    def __init__(self, batch, heads, N, d, B, K, L, Le=None, sm_scale=0.0, dtype=BF16, reweight=1, bwd_repool=0,
                 kernel_path=0, single_stream=0):
        lib = load()
        self.desc = _Desc(batch, heads, N, d, B, K, L, L if Le is None else Le, sm_scale, dtype, reweight,
                          bwd_repool, kernel_path, single_stream)
        h = ctypes.c_void_p()
        st = lib.llsa_plan(ctypes.byref(self.desc), ctypes.byref(h))
        self._h = h if st == 0 else None
        _check(st, "llsa_plan")
        self.batch, self.heads, self.N, self.d, self.B, self.K, self.L = batch, heads, N, d, B, K, L
        self.Le = self.desc.Le
        self.torch_dtype = torch.float32 if dtype == F32 else torch.bfloat16
        self.levels = [self.level_info(l) for l in range(L)]

    def __del__(self):
        if getattr(self, "_h", None) is not None and _lib is not None:
            _lib.llsa_plan_destroy(self._h)
            self._h = None

    def workspace_bytes(self, for_backward: bool) -> int:
        return load().llsa_plan_workspace_bytes(self._h, int(for_backward))

    def indices_bytes(self) -> int:
        return load().llsa_plan_indices_bytes(self._h)

    def level_info(self, l: int) -> LevelInfo:
        rows, kl, off = ctypes.c_int64(), ctypes.c_int32(), ctypes.c_size_t()
        if load().llsa_plan_level_info(self._h, l, ctypes.byref(rows), ctypes.byref(kl), ctypes.byref(off)) < 0:
            raise LlsaError("llsa_plan_level_info: bad level")
        return LevelInfo(rows.value, kl.value, off.value)

    def pyramid_info(self, tensor: int, l: int):
        tok, off = ctypes.c_int64(), ctypes.c_size_t()
        if load().llsa_plan_pyramid_info(self._h, tensor, l, ctypes.byref(tok), ctypes.byref(off)) < 0:
            raise LlsaError("llsa_plan_pyramid_info: bad arguments")
        return tok.value, off.value

    def csc_info(self, l: int):
        c, iq = ctypes.c_size_t(), ctypes.c_size_t()
        if load().llsa_plan_csc_info(self._h, l, ctypes.byref(c), ctypes.byref(iq)) < 0:
            raise LlsaError("llsa_plan_csc_info: bad level")
        return c.value, iq.value

    # ---- buffers (torch allocates, the library only reads the pointers) ----
    def alloc_workspace(self, for_backward: bool, device="cuda") -> torch.Tensor:
        return torch.empty(max(self.workspace_bytes(for_backward), 256), dtype=torch.uint8, device=device)

    def alloc_indices(self, device="cuda") -> torch.Tensor:
        return torch.empty(self.indices_bytes() // 4, dtype=torch.int32, device=device)

    def level_indices(self, indices: torch.Tensor, l: int) -> torch.Tensor:
        """View of I^(l) inside ``indices``: ``[batch, heads, rows, K_l]``."""
        li = self.levels[l]
        n = self.batch * self.heads * li.rows * li.K_l
        return indices[li.byte_offset // 4: li.byte_offset // 4 + n].view(self.batch, self.heads, li.rows, li.K_l)

    def pyramid_level(self, workspace: torch.Tensor, tensor: int, l: int) -> torch.Tensor:
        """View of pooled level l (>= 1) of Q/K/V (tensor 0/1/2) inside ``workspace``."""
        tok, off = self.pyramid_info(tensor, l)
        nbytes = self.batch * self.heads * tok * self.d * self.torch_dtype.itemsize
        return workspace[off: off + nbytes].view(self.torch_dtype).view(self.batch, self.heads, tok, self.d)

    def csc_level(self, workspace: torch.Tensor, l: int):
        """(C [bh, rows+1], Iq [bh, rows*K_l]) views inside a backward workspace."""
        c_off, iq_off = self.csc_info(l)
        li, bh = self.levels[l], self.batch * self.heads
        C = workspace[c_off: c_off + bh * (li.rows + 1) * 4].view(torch.int32).view(bh, li.rows + 1)
        Iq = workspace[iq_off: iq_off + bh * li.rows * li.K_l * 4].view(torch.int32).view(bh, li.rows * li.K_l)
        return C, Iq


def _chk_tensor(p: Plan, t: torch.Tensor, name: str):
    if not t.is_cuda or not t.is_contiguous() or t.dtype != p.torch_dtype or \
            tuple(t.shape) != (p.batch, p.heads, p.N, p.d):
        raise LlsaError(f"{name}: expected a contiguous cuda {p.torch_dtype} tensor of shape "
                        f"{(p.batch, p.heads, p.N, p.d)}, got {t.dtype} {tuple(t.shape)} on {t.device}")


def forward(p: Plan, Q, K, V, O=None, LSE=None, indices=None, workspace=None):
    """``llsa_forward``: returns ``(O, LSE, indices, workspace)``."""
    for t, n in ((Q, "Q"), (K, "K"), (V, "V")):
        _chk_tensor(p, t, n)
    O = torch.empty_like(Q) if O is None else O
    LSE = torch.empty(p.batch, p.heads, p.N, dtype=torch.float32, device=Q.device) if LSE is None else LSE
    indices = p.alloc_indices(Q.device) if indices is None else indices
    workspace = p.alloc_workspace(False, Q.device) if workspace is None else workspace
    if workspace.numel() < p.workspace_bytes(False) or indices.numel() * 4 < p.indices_bytes():
        raise LlsaError("workspace or indices buffer too small")
    _check(load().llsa_forward(p._h, _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(indices), _ptr(workspace),
                               _stream()), "llsa_forward")
    return O, LSE, indices, workspace


def qknorm_rope_pool(p: Plan, Qpre, Kpre, V, gamma_q, gamma_k, cos_table, sin_table, eps=1e-6, workspace=None):
    """``llsa_qknorm_rope_pool``: returns ``(Qout, Kout, workspace)`` (workspace holds every pooled level)."""
    for t, n in ((Qpre, "Qpre"), (Kpre, "Kpre"), (V, "V")):
        _chk_tensor(p, t, n)
    for t, shape, n in ((gamma_q, (p.d,), "gamma_q"), (gamma_k, (p.d,), "gamma_k"),
                        (cos_table, (p.N, p.d // 2), "cos_table"), (sin_table, (p.N, p.d // 2), "sin_table")):
        if not t.is_cuda or not t.is_contiguous() or t.dtype != torch.float32 or tuple(t.shape) != shape:
            raise LlsaError(f"{n}: expected a contiguous cuda float32 tensor of shape {shape}")
    Qout, Kout = torch.empty_like(Qpre), torch.empty_like(Kpre)
    workspace = p.alloc_workspace(False, Qpre.device) if workspace is None else workspace
    if workspace.numel() < p.workspace_bytes(False):
        raise LlsaError("workspace too small")
    _check(load().llsa_qknorm_rope_pool(p._h, _ptr(Qpre), _ptr(Kpre), _ptr(V), _ptr(gamma_q), _ptr(gamma_k),
                                        _ptr(cos_table), _ptr(sin_table), ctypes.c_float(eps), _ptr(Qout), _ptr(Kout),
                                        _ptr(workspace), _stream()), "llsa_qknorm_rope_pool")
    return Qout, Kout, workspace


def forward_pooled(p: Plan, Q, K, V, workspace, O=None, LSE=None, indices=None):
    """``llsa_forward_pooled``: forward pass on pooled levels already in ``workspace``."""
    for t, n in ((Q, "Q"), (K, "K"), (V, "V")):
        _chk_tensor(p, t, n)
    O = torch.empty_like(Q) if O is None else O
    LSE = torch.empty(p.batch, p.heads, p.N, dtype=torch.float32, device=Q.device) if LSE is None else LSE
    indices = p.alloc_indices(Q.device) if indices is None else indices
    if workspace.numel() < p.workspace_bytes(False) or indices.numel() * 4 < p.indices_bytes():
        raise LlsaError("workspace or indices buffer too small")
    _check(load().llsa_forward_pooled(p._h, _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(indices),
                                      _ptr(workspace), _stream()), "llsa_forward_pooled")
    return O, LSE, indices


def forward_static(p: Plan, Q, K, V, O, LSE, indices):
    """``llsa_forward_static``: forward pass on the library's static workspace; the caller passes every
    output buffer, and neither the binding nor the library allocates."""
    for t, n in ((Q, "Q"), (K, "K"), (V, "V"), (O, "O")):
        _chk_tensor(p, t, n)
    if indices.numel() * 4 < p.indices_bytes() or LSE.numel() < p.batch * p.heads * p.N:
        raise LlsaError("indices or LSE buffer too small")
    _check(load().llsa_forward_static(p._h, _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(indices), _stream()),
           "llsa_forward_static")


def static_workspace_bytes() -> int:
    return load().llsa_static_workspace_bytes()


def backward(p: Plan, Q, K, V, O, LSE, indices, dO, workspace, dQ=None, dK=None, dV=None):
    """``llsa_backward``: returns ``(dQ, dK, dV)``.  ``workspace`` must hold the backward size."""
    for t, n in ((Q, "Q"), (K, "K"), (V, "V"), (O, "O"), (dO, "dO")):
        _chk_tensor(p, t, n)
    if workspace.numel() < p.workspace_bytes(True):
        raise LlsaError("backward workspace too small")
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(Q) if dK is None else dK
    dV = torch.empty_like(Q) if dV is None else dV
    _check(load().llsa_backward(p._h, _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(indices), _ptr(dO),
                                _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(workspace), _stream()), "llsa_backward")
    return dQ, dK, dV


def kv_backward_level0(p: Plan, via_mask: bool, Q, K, V, dO, LSE, indices, workspace, mask=None, dK0=None, dV0=None):
    """``llsa_kv_backward_level0``: level 0's dK, dV with the key-major lists from Alg. 2 or from a dense block mask.
    ``workspace`` must be the one a preceding ``backward`` call used (it holds D).  Returns ``(dK0, dV0, mask)``."""
    for t, n in ((Q, "Q"), (K, "K"), (V, "V"), (dO, "dO")):
        _chk_tensor(p, t, n)
    if via_mask and mask is None:
        mask = torch.empty(load().llsa_kv_backward_mask_bytes(p._h), dtype=torch.uint8, device=Q.device)
    dK0 = torch.empty_like(Q) if dK0 is None else dK0
    dV0 = torch.empty_like(Q) if dV0 is None else dV0
    _check(load().llsa_kv_backward_level0(p._h, int(via_mask), _ptr(Q), _ptr(K), _ptr(V), _ptr(dO), _ptr(LSE),
                                          _ptr(indices), _ptr(mask), _ptr(workspace), _ptr(dK0), _ptr(dV0), _stream()),
           "llsa_kv_backward_level0")
    return dK0, dV0, mask


def pool(p: Plan, Q, K, V, workspace):
    """``llsa_pool``: fills the pooled levels in ``workspace``."""
    for t, n in ((Q, "Q"), (K, "K"), (V, "V")):
        _chk_tensor(p, t, n)
    _check(load().llsa_pool(p._h, _ptr(Q), _ptr(K), _ptr(V), _ptr(workspace), _stream()), "llsa_pool")


def select_level(p: Plan, l: int, workspace, parent, out):
    """``llsa_select_level``: one selection level from given parent lists."""
    _check(load().llsa_select_level(p._h, l, _ptr(workspace), _ptr(parent), _ptr(out), _stream()),
           "llsa_select_level")


def attention(p: Plan, Q, K, V, indices, workspace, O=None, LSE=None):
    """``llsa_attention``: attention over given lists and pooled levels."""
    O = torch.empty_like(Q) if O is None else O
    LSE = torch.empty(p.batch, p.heads, p.N, dtype=torch.float32, device=Q.device) if LSE is None else LSE
    _check(load().llsa_attention(p._h, _ptr(Q), _ptr(K), _ptr(V), _ptr(indices), _ptr(workspace), _ptr(O), _ptr(LSE),
                                 _stream()), "llsa_attention")
    return O, LSE


def index_transpose(p: Plan, indices, workspace):
    """``llsa_index_transpose``: key-major lists of every level into a backward workspace."""
    _check(load().llsa_index_transpose(p._h, _ptr(indices), _ptr(workspace), _stream()), "llsa_index_transpose")


def reorder(x: torch.Tensor, inverse: bool = False, out: torch.Tensor | None = None) -> torch.Tensor:
    """``llsa_reorder``: tokens of ``x [..., N, d]`` (N = W*W, raster order) into nested-patch order, or back."""
    if not x.is_contiguous():
        raise LlsaError("llsa_reorder needs a contiguous tensor")
    dtype = {torch.float32: F32, torch.bfloat16: BF16}.get(x.dtype)
    if dtype is None:
        raise LlsaError("llsa_reorder: fp32 or bf16 only")
    N, d = x.shape[-2], x.shape[-1]
    out = torch.empty_like(x) if out is None else out
    _check(load().llsa_reorder(x.numel() // (N * d), N, d, dtype, int(inverse), _ptr(x), _ptr(out), _stream()), "llsa_reorder")
    return out


def measured_peaks(mfma_iters: int = 20000, copy_bytes: int = 1 << 30, reps: int = 5) -> dict:
    """Times ``llsa_calibrate_mfma`` (2048 workgroups: 8 per CU) and ``llsa_calibrate_copy`` with HIP events: the
    bf16 MFMA rate and the copy bandwidth this GPU delivers, best of ``reps``."""
    lib = load()
    out = torch.zeros(4, dtype=torch.float32, device="cuda")
    src = torch.zeros(copy_bytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    wgs = 2048
    best = {"mfma": float("inf"), "copy": float("inf")}
    for rep in range(reps + 1):
        for name, call in (("mfma", lambda: lib.llsa_calibrate_mfma(_ptr(out), mfma_iters, wgs, _stream())),
                           ("copy", lambda: lib.llsa_calibrate_copy(_ptr(src), _ptr(dst), copy_bytes, _stream()))):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            _check(call(), f"llsa_calibrate_{name}")
            e1.record()
            e1.synchronize()
            if rep > 0:                                      # the first round warms up
                best[name] = min(best[name], e0.elapsed_time(e1))
    flop = wgs * 4 * 8 * mfma_iters * 16384.0
    return {"mfma_bf16_tflops": flop / (best["mfma"] * 1e-3) / 1e12, "copy_gbps": 2.0 * copy_bytes / (best["copy"] * 1e-3) / 1e9,
            "mfma_ms": best["mfma"], "copy_ms": best["copy"]}


def stage_names() -> list[str]:
    lib = load()
    return [lib.llsa_stage_name(i).decode() for i in range(lib.llsa_stage_count())]


def stage_timing_begin(stage: int | str = -1, max_calls: int = 64):
    """``llsa_stage_timing_begin``: bracket one stage (index or name; -1 = all) with HIP events."""
    if isinstance(stage, str):
        stage = stage_names().index(stage)
    _check(load().llsa_stage_timing_begin(stage, max_calls), "llsa_stage_timing_begin")


def stage_timing_end() -> dict[str, tuple[float, int]]:
    """``llsa_stage_timing_end``: ``{stage name: (summed ms, number of brackets)}``."""
    lib = load()
    n = lib.llsa_stage_count()
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int32 * n)()
    _check(lib.llsa_stage_timing_end(ms, cnt), "llsa_stage_timing_end")
    return {name: (ms[i], cnt[i]) for i, name in enumerate(stage_names())}
