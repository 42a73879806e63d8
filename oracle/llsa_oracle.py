"""ctypes front end of the CPU oracle (``llsa_oracle.c``).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
cpu_baseline leg may import this; the GPU product path never does, and this
module imports nothing from the GPU package.

All functions work on ONE (batch, head) slice: arrays are ``[N, d]``.
Level geometry (paper notation, Sec. 4.1): ``n_l = N / B**l`` tokens at level
``l = 0..L``; ``I^(l)`` has ``n_{l+1}`` rows of ``K_l = min(K, n_{l+1})`` key
block ids at level ``l``.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "llsa_oracle.c")
_LIB = os.path.join(_HERE, "libllsa_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
               "-mfma", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.llsa_oracle_list_len.restype = ctypes.c_int64
        _lib.llsa_oracle_kv_list.restype = ctypes.c_int64
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


@dataclass(frozen=True)
class Geometry:
    """Level table of one problem (Sec. 4.1)."""
    N: int
    d: int
    B: int
    K: int
    L: int

    def __post_init__(self):
        if self.L < 1 or self.N % (self.B ** self.L) != 0:
            raise ValueError("N must be divisible by B**L and L >= 1")

    def n(self, l: int) -> int:
        return self.N // self.B ** l

    def K_l(self, l: int) -> int:
        return min(self.K, self.n(l + 1))

    def pyr_offset(self, l: int) -> int:
        return sum(self.n(j) for j in range(l))

    def pyr_tokens(self) -> int:
        return self.pyr_offset(self.L + 1)

    def idx_offset(self, l: int) -> int:
        return sum(self.n(j + 1) * self.K_l(j) for j in range(l))

    def idx_entries(self) -> int:
        return self.idx_offset(self.L)

    def list_len(self, Le: int) -> int:
        return sum(self.K_l(l) * self.B if l < self.L else self.n(self.L) for l in range(Le + 1))


def to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest (even) bf16 value, returned as fp32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def pool(x: np.ndarray, B: int, bf16: bool) -> np.ndarray:
    """One pooling step, ``[n, d] -> [n // B, d]`` (Alg. 1, compression loop)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    n_out, d = x.shape[0] // B, x.shape[1]
    y = np.empty((n_out, d), np.float32)
    _load().llsa_oracle_pool(_p(x, ctypes.c_float), ctypes.c_int64(n_out), d, B, int(bf16), _p(y, ctypes.c_float))
    return y


def pyramid(x: np.ndarray, g: Geometry, bf16: bool) -> list[np.ndarray]:
    """Levels ``0..L`` of one tensor; each level pooled from the stored previous level."""
    levels = [np.ascontiguousarray(x, dtype=np.float32)]
    for _ in range(g.L):
        levels.append(pool(levels[-1], g.B, bf16))
    return levels


def select_level(Ql: np.ndarray, Kl: np.ndarray, B: int, parent, Kout: int, want_margin: bool = False):
    """Selection at one level: returns ``I^(l-1)`` ``[n_l, Kout]`` (and the fp64 margin per row)."""
    Ql = np.ascontiguousarray(Ql, dtype=np.float32)
    Kl = np.ascontiguousarray(Kl, dtype=np.float32)
    n_l, d = Ql.shape
    out = np.empty((n_l, Kout), np.int32)
    margin = np.empty(n_l, np.float64) if want_margin else None
    if parent is None:
        pp, Kp = None, 0
    else:
        parent = np.ascontiguousarray(parent, dtype=np.int32)
        assert parent.shape[0] * B == n_l
        pp, Kp = _p(parent, ctypes.c_int32), parent.shape[1]
    rc = _load().llsa_oracle_select(_p(Ql, ctypes.c_float), _p(Kl, ctypes.c_float), ctypes.c_int64(n_l), d, B,
                                    pp, Kp, Kout, _p(out, ctypes.c_int32),
                                    _p(margin, ctypes.c_double) if want_margin else None)
    if rc != 0:
        raise RuntimeError(f"llsa_oracle_select failed ({rc})")
    return (out, margin) if want_margin else out


def select_all(Qp: list[np.ndarray], Kp: list[np.ndarray], g: Geometry, want_margin: bool = False):
    """Hierarchical Top-K (Alg. 1, selection loop): returns ``[I^(0), ..., I^(L-1)]``."""
    I = [None] * g.L
    margins = [None] * g.L
    parent = None
    for l in range(g.L, 0, -1):
        res = select_level(Qp[l], Kp[l], g.B, parent, g.K_l(l - 1), want_margin)
        I[l - 1], margins[l - 1] = res if want_margin else (res, None)
        parent = I[l - 1]
    return (I, margins) if want_margin else I


def cat_indices(I: list[np.ndarray]) -> np.ndarray:
    return np.ascontiguousarray(np.concatenate([a.reshape(-1) for a in I]).astype(np.int32))


def cat_pyramid(levels: list[np.ndarray]) -> np.ndarray:
    return np.ascontiguousarray(np.concatenate(levels, axis=0), dtype=np.float64)


def kv_list(idx_cat: np.ndarray, g: Geometry, Le: int, block: int):
    """(levels, tokens) of the list fine query block ``block`` attends to."""
    cap = g.list_len(Le)
    lev = np.empty(cap, np.int32)
    tok = np.empty(cap, np.int64)
    m = _load().llsa_oracle_kv_list(_p(idx_cat, ctypes.c_int32), ctypes.c_int64(g.N), g.B, g.K, g.L, Le,
                                    ctypes.c_int64(block), _p(lev, ctypes.c_int32), _p(tok, ctypes.c_int64))
    assert m == cap
    return lev, tok


def attn_fwd(Q, Kpyr, Vpyr, idx_cat, g: Geometry, Le: int, reweight: int = 1, scale: float | None = None,
             rows: tuple[int, int] | None = None):
    """Attention over the gathered list, fp64.  Returns ``(O [N,d], LSE [N])``;
    with ``rows=(a, b)`` only rows ``a..b-1`` are computed (others are NaN)."""
    Q = np.ascontiguousarray(Q, dtype=np.float64)
    Kpyr = np.ascontiguousarray(Kpyr, dtype=np.float64)
    Vpyr = np.ascontiguousarray(Vpyr, dtype=np.float64)
    assert Kpyr.shape == (g.pyr_tokens(), g.d) and Vpyr.shape == Kpyr.shape and Q.shape == (g.N, g.d)
    scale = 1.0 / math.sqrt(g.d) if scale is None else scale
    a, b = rows if rows is not None else (0, g.N)
    O = np.full((g.N, g.d), np.nan)
    LSE = np.full(g.N, np.nan)
    rc = _load().llsa_oracle_attn_fwd(_p(Q, ctypes.c_double), _p(Kpyr, ctypes.c_double), _p(Vpyr, ctypes.c_double),
                                      _p(idx_cat, ctypes.c_int32), ctypes.c_int64(g.N), g.d, g.B, g.K, g.L, Le,
                                      reweight, ctypes.c_double(scale), ctypes.c_int64(a), ctypes.c_int64(b),
                                      _p(O, ctypes.c_double), _p(LSE, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"llsa_oracle_attn_fwd failed ({rc})")
    return O, LSE


def attn_bwd(Q, Kpyr, Vpyr, idx_cat, dO, g: Geometry, Le: int, reweight: int = 1, scale: float | None = None,
             rows: tuple[int, int] | None = None):
    """Gradients w.r.t. Q and every pyramid level (indices frozen), fp64.  ``rows=(a, b)`` restricts the sum to
    the contributions of query rows ``a..b-1``."""
    Q = np.ascontiguousarray(Q, dtype=np.float64)
    Kpyr = np.ascontiguousarray(Kpyr, dtype=np.float64)
    Vpyr = np.ascontiguousarray(Vpyr, dtype=np.float64)
    dO = np.ascontiguousarray(dO, dtype=np.float64)
    scale = 1.0 / math.sqrt(g.d) if scale is None else scale
    a, b = rows if rows is not None else (0, g.N)
    dQ = np.empty_like(Q)
    dKpyr = np.empty_like(Kpyr)
    dVpyr = np.empty_like(Vpyr)
    rc = _load().llsa_oracle_attn_bwd(_p(Q, ctypes.c_double), _p(Kpyr, ctypes.c_double), _p(Vpyr, ctypes.c_double),
                                      _p(idx_cat, ctypes.c_int32), _p(dO, ctypes.c_double), ctypes.c_int64(g.N),
                                      g.d, g.B, g.K, g.L, Le, reweight, ctypes.c_double(scale),
                                      ctypes.c_int64(a), ctypes.c_int64(b), _p(dQ, ctypes.c_double), _p(dKpyr, ctypes.c_double), _p(dVpyr, ctypes.c_double))
    if rc != 0:
        raise RuntimeError(f"llsa_oracle_attn_bwd failed ({rc})")
    return dQ, dKpyr, dVpyr


def unpool(gpyr: np.ndarray, g: Geometry) -> np.ndarray:
    """Adjoint of the pyramid: gradient of all levels folded into level 0, ``[N, d]``."""
    work = np.array(gpyr, dtype=np.float64, order="C", copy=True)
    gx = np.empty((g.N, g.d), np.float64)
    _load().llsa_oracle_unpool(_p(work, ctypes.c_double), ctypes.c_int64(g.N), g.d, g.B, g.L, _p(gx, ctypes.c_double))
    return gx


def transpose(I: np.ndarray, T_keys: int):
    """Alg. 2: ``I [T_rows, K]`` -> ``(Iq [T_rows*K], C [T_keys+1])``."""
    I = np.ascontiguousarray(I, dtype=np.int32)
    T_rows, K = I.shape
    Iq = np.empty(T_rows * K, np.int32)
    C = np.empty(T_keys + 1, np.int32)
    _load().llsa_oracle_transpose(_p(I, ctypes.c_int32), ctypes.c_int64(T_rows), K, ctypes.c_int64(T_keys),
                                  _p(Iq, ctypes.c_int32), _p(C, ctypes.c_int32))
    return Iq, C


# ------------------------------------------------------------------ index reordering (Sec. 5.1)

def nested_order(W: int) -> np.ndarray:
    """Index reordering for a ``W x W`` pixel grid (W a power of two): ``order[t]`` is the raster index ``y*W + x``
    of the pixel that becomes token ``t``, such that for every ``i`` the pixels of each aligned patch of size
    ``2**i x 2**i`` are consecutive tokens.  Written as that definition, recursively: the tokens of a patch are
    the tokens of its four half-size patches one after the other (upper left, upper right, lower left, lower
    right; the paper's figure fixes no order among the four, row-major is this build's reading)."""
    if W < 1 or W & (W - 1):
        raise ValueError("the pixel grid side must be a power of two")

    def patch(y0: int, x0: int, size: int) -> list[int]:
        if size == 1:
            return [y0 * W + x0]
        h = size // 2
        return patch(y0, x0, h) + patch(y0, x0 + h, h) + patch(y0 + h, x0, h) + patch(y0 + h, x0 + h, h)

    return np.array(patch(0, 0, W), dtype=np.int64)


def reorder(x: np.ndarray, inverse: bool = False) -> np.ndarray:
    """Applies the index reordering to the token axis of ``x [N, d]`` (N = W*W): raster order -> nested-patch
    order (``out[t] = x[order[t]]``), or back (``out[order[t]] = x[t]``)."""
    N = x.shape[0]
    W = math.isqrt(N)
    if W * W != N:
        raise ValueError("index reordering needs a square pixel grid")
    order = nested_order(W)
    out = np.empty_like(x)
    if inverse:
        out[order] = x
    else:
        out[:] = x[order]
    return out


# ------------------------------------------------------------------ layer glue (Sec. 5.2, "Training Settings")

def qknorm_rope(x: np.ndarray, gamma: np.ndarray, cos: np.ndarray, sin: np.ndarray, eps: float = 1e-6) -> np.ndarray:
    """QK-Norm followed by RoPE on one head ``x [N, d]``, fp64.  The paper names the two operators and cites them
    without giving their form; the forms taken here are the ones of the cited works: the norm divides every token by
    the root mean square of its d channels (plus ``eps`` under the root) and multiplies by a learned gain ``gamma
    [d]``; the rotary embedding turns every adjacent channel pair ``(2i, 2i+1)`` of token t by the angle whose
    cosine and sine are ``cos[t, i]``, ``sin[t, i]``."""
    x = np.asarray(x, dtype=np.float64)
    rms = np.sqrt((x * x).mean(axis=1, keepdims=True) + eps)
    y = x / rms * np.asarray(gamma, dtype=np.float64)[None, :]
    a, b = y[:, 0::2], y[:, 1::2]
    c, s_ = np.asarray(cos, dtype=np.float64), np.asarray(sin, dtype=np.float64)
    out = np.empty_like(y)
    out[:, 0::2] = a * c - b * s_
    out[:, 1::2] = a * s_ + b * c
    return out


# ------------------------------------------------------------------ whole layer

def forward(Q, K, V, g: Geometry, Le: int | None = None, bf16: bool = False, reweight: int = 1,
            scale: float | None = None, rows: tuple[int, int] | None = None, want_margin: bool = False):
    """Alg. 1 for one head.  Inputs must already be representable in the I/O type."""
    Le = g.L if Le is None else Le
    Qp, Kp, Vp = (pyramid(x, g, bf16) for x in (Q, K, V))
    sel = select_all(Qp, Kp, g, want_margin)
    I, margins = sel if want_margin else (sel, None)
    idx_cat = cat_indices(I)
    O, LSE = attn_fwd(Qp[0], cat_pyramid(Kp), cat_pyramid(Vp), idx_cat, g, Le, reweight, scale, rows)
    return {"Qp": Qp, "Kp": Kp, "Vp": Vp, "I": I, "idx_cat": idx_cat, "margins": margins, "O": O, "LSE": LSE}


def backward(Q, Kp: list[np.ndarray], Vp: list[np.ndarray], idx_cat, dO, g: Geometry, Le: int | None = None,
             reweight: int = 1, scale: float | None = None):
    """Gradients of one head w.r.t. Q, K, V with the selection frozen (through the pooled levels)."""
    Le = g.L if Le is None else Le
    dQ, dKpyr, dVpyr = attn_bwd(Q, cat_pyramid(Kp), cat_pyramid(Vp), idx_cat, dO, g, Le, reweight, scale)
    return {"dQ": dQ, "dK": unpool(dKpyr, g), "dV": unpool(dVpyr, g), "dKpyr": dKpyr, "dVpyr": dVpyr}
