"""Seeded synthetic inputs for the LLSA layer (shared by the tests, the benchmark
and the CPU oracle's callers).  Holds no arithmetic of the method itself.

Recipe.  A counter-based generator: ``splitmix64`` applied to ``key + i * GOLDEN``
gives the i-th 64-bit word of a stream; ``key`` is derived from the seed and a
stream id (tensor, batch, head, purpose).  Uniforms are the top 53 bits (offset
by one half so 0 is excluded); normals come from Box-Muller on word pairs.

Workloads (stand-ins for the pixel-token activations of a pixel-space DiT, which
need a dataset and trained weights that are not available here):

* ``gaussian``: every element i.i.d. N(0, 1).
* ``smooth``: token t is pixel (y, x) = (t // W, t % W) of a W x W grid, row-major.
  Per channel: sum of 8 sinusoids ``a_m sin(2 pi (fy_m y + fx_m x) / W + phi_m)``
  with integer frequencies in {0..3} (not both zero), ``phi_m ~ U[0, 2 pi)``,
  ``a_m ~ N(0, 1/4)`` (unit variance for the smooth part), plus ``0.1 N(0, 1)``.

Values are produced in fp64, cast to fp32 and, for bf16 I/O, rounded to nearest
even bf16 by the caller; that rounded tensor is what every consumer sees.
"""
from __future__ import annotations

import math

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

TENSOR_IDS = {"Q": 0, "K": 1, "V": 2, "dO": 3}


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z + _GOLDEN).astype(np.uint64)
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _key(seed: int, stream: tuple[int, ...]) -> np.uint64:
    k = np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64)
    with np.errstate(over="ignore"):
        for s in stream:
            k = _mix(k ^ _mix(np.array([s & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64)))
    return k[0]


def words(seed: int, stream: tuple[int, ...], count: int) -> np.ndarray:
    """The first ``count`` 64-bit words of a stream."""
    with np.errstate(over="ignore"):
        i = np.arange(count, dtype=np.uint64)
        return _mix(_key(seed, stream) + i * _GOLDEN)


def uniform(seed: int, stream: tuple[int, ...], count: int) -> np.ndarray:
    """U(0, 1), fp64, never exactly 0 or 1."""
    return ((words(seed, stream, count) >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, stream: tuple[int, ...], count: int) -> np.ndarray:
    """N(0, 1), fp64, Box-Muller on consecutive uniform pairs."""
    u = uniform(seed, stream, 2 * count)
    return np.sqrt(-2.0 * np.log(u[0::2])) * np.cos(2.0 * math.pi * u[1::2])


def gaussian_head(seed: int, tensor: str, b: int, h: int, N: int, d: int) -> np.ndarray:
    """``[N, d]`` fp32, i.i.d. N(0, 1)."""
    return normal(seed, (TENSOR_IDS[tensor], b, h, 0), N * d).reshape(N, d).astype(np.float32)


def smooth_head(seed: int, tensor: str, b: int, h: int, N: int, d: int) -> np.ndarray:
    """``[N, d]`` fp32 smooth pixel-grid field (see module docstring); N must be a square."""
    W = math.isqrt(N)
    if W * W != N:
        raise ValueError("smooth fields need a square token grid")
    tid = TENSOR_IDS[tensor]
    M = 8
    fw = words(seed, (tid, b, h, 1), 2 * M * d).reshape(M, d, 2)
    fy = (fw[..., 0] % np.uint64(4)).astype(np.int64)
    fx = (fw[..., 1] % np.uint64(4)).astype(np.int64)
    both0 = (fy == 0) & (fx == 0)
    fx = np.where(both0, 1 + (fw[..., 1] >> np.uint64(8)) % np.uint64(3), fx).astype(np.int64)
    phi = 2.0 * math.pi * uniform(seed, (tid, b, h, 2), M * d).reshape(M, d)
    amp = 0.5 * normal(seed, (tid, b, h, 3), M * d).reshape(M, d)
    pos = np.arange(W, dtype=np.float64) * (2.0 * math.pi / W)
    field = np.zeros((W, W, d), np.float64)
    for m in range(M):
        ay = pos[:, None] * fy[m][None, :] + phi[m][None, :]      # [W(y), d]
        bx = pos[:, None] * fx[m][None, :]                        # [W(x), d]
        field += amp[m] * (np.sin(ay)[:, None, :] * np.cos(bx)[None, :, :]
                           + np.cos(ay)[:, None, :] * np.sin(bx)[None, :, :])
    field = field.reshape(N, d) + 0.1 * normal(seed, (tid, b, h, 0), N * d).reshape(N, d)
    return field.astype(np.float32)


def make_head(kind: str, seed: int, tensor: str, b: int, h: int, N: int, d: int) -> np.ndarray:
    if tensor == "dO" or kind == "gaussian":
        return gaussian_head(seed, tensor, b, h, N, d)
    if kind == "smooth":
        return smooth_head(seed, tensor, b, h, N, d)
    raise ValueError(f"unknown input kind {kind!r}")


def make_tensor(kind: str, seed: int, tensor: str, batch: int, heads: int, N: int, d: int) -> np.ndarray:
    """``[batch, heads, N, d]`` fp32.  The upstream gradient ``dO`` is always Gaussian."""
    out = np.empty((batch, heads, N, d), np.float32)
    for b in range(batch):
        for h in range(heads):
            out[b, h] = make_head(kind, seed, tensor, b, h, N, d)
    return out


def rope_tables(N: int, d: int, base: float = 10000.0) -> tuple[np.ndarray, np.ndarray]:
    """Rotary-position tables ``(cos, sin)``, each ``[N, d // 2]`` fp32, for tokens in raster order: an input of the
    layer glue, built by whoever owns the token order.  If N is a square W x W pixel grid the two axes share the
    channel pairs (pairs ``0 .. d/4 - 1`` turn with the row y, pairs ``d/4 .. d/2 - 1`` with the column x, the usual
    axial form for images), otherwise all pairs turn with the 1-D position; pair i of an axis with P pairs has the
    frequency ``base ** (-i / P)``.  Angles are formed in fp64 and the tables rounded once to fp32."""
    half = d // 2
    W = math.isqrt(N)
    t = np.arange(N, dtype=np.float64)
    if W * W == N and half % 2 == 0:
        P = half // 2
        freq = base ** (-np.arange(P, dtype=np.float64) / P)
        ang = np.concatenate([(t // W)[:, None] * freq[None, :], (t % W)[:, None] * freq[None, :]], axis=1)
    else:
        freq = base ** (-np.arange(half, dtype=np.float64) / half)
        ang = t[:, None] * freq[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def norm_gain(seed: int, which: str, d: int) -> np.ndarray:
    """``[d]`` fp32 gain of the QK-Norm of ``which`` ("Q" or "K"): 1 + 0.1 N(0, 1), as after some training."""
    return (1.0 + 0.1 * normal(seed, (TENSOR_IDS[which], 0, 0, 7), d)).astype(np.float32)


# BASELINE.json's five configurations (index = position in its "configs" list).
CONFIGS = [
    dict(name="tiny_fp32", batch=1, heads=1, d=32, N=256, B=4, K=2, L=3, dtype="f32", kind="gaussian"),
    dict(name="n4096", batch=1, heads=16, d=64, N=4096, B=16, K=8, L=2, dtype="bf16", kind="smooth"),
    dict(name="n16384", batch=2, heads=16, d=64, N=16384, B=16, K=8, L=3, dtype="bf16", kind="smooth"),
    dict(name="headline_n65536", batch=1, heads=16, d=64, N=65536, B=16, K=8, L=3, dtype="bf16", kind="smooth"),
    dict(name="extreme_n262144", batch=1, heads=8, d=128, N=262144, B=16, K=16, L=4, dtype="bf16", kind="smooth"),
]


def config_seed(index: int) -> int:
    return 0x115A0000 + index
