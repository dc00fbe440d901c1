"""Seeded synthetic inputs shaped like the paper's video-DiT attention workloads.

This module only *makes inputs* (and converts between storage formats).  It holds
none of the method's arithmetic: no pooling, no draft map, no selection, no
permutation, no attention.  Both the CPU oracle's tests and the HIP path's tests
feed from it, so the two sides see the same bits.

The paper evaluates on HunyuanVideo / Wan2.1 activations (Section 4.1); those models
and prompts are not available here, so the tensors below are stand-ins with the same
shapes (heads, head dim, latent frame grids, frame counts) and the structure the
method relies on: queries and keys that vary smoothly over (t, y, x) (the premise of
the remark after Theorem 1) plus independent noise, and unstructured values.

Recipe, per (batch b, head h), from ``numpy.random.default_rng([seed, b, h])`` and in
exactly this draw order:

  f     = U(-1/16, 1/16)          shape (d, 8, 3)   cycles/token along (t, y, x)
  phi   = U(0, 2*pi)              shape (d, 8)
  drift = cumsum_t N(0, 0.15^2)   shape (T, d, 8)   only when ``drift`` is set
  nq    = N(0, 0.3^2)             shape (N, d)
  nk    = N(0, 0.3^2)             shape (N, d)
  V     = N(0, 1)                 shape (N, d)
  smooth[t,y,x,c] = sum_m cos(2*pi*(f[c,m,0]*t + f[c,m,1]*y + f[c,m,2]*x) + phi[c,m] + drift[t,c,m])
  Q = smooth + nq,  K = smooth + nk

All of it is computed in float64, rounded to float32 and, for bf16 storage, rounded
again to bf16 (round-to-nearest-even both times).  Token index is n = t*fh*fw + y*fw + x.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

F32 = 0
BF16 = 1


@dataclass(frozen=True)
class Workload:
    """One attention problem: Q, K, V of shape [B, H, N, d] with N = T*fh*fw."""
    name: str
    B: int
    H: int
    d: int
    T: int
    fh: int
    fw: int
    ph: int = 8
    pw: int = 8
    sparsity: float = 0.0
    dtype: int = BF16
    drift: bool = False
    seed: int = 0

    @property
    def N(self) -> int:
        return self.T * self.fh * self.fw

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five configurations named by the build's baseline file.
CONFIGS = {
    "tiny_fp32": Workload("tiny_fp32", B=1, H=2, d=64, T=2, fh=16, fw=16, sparsity=0.5, dtype=F32),
    "480p": Workload("480p", B=1, H=24, d=128, T=21, fh=30, fw=52, sparsity=0.75),
    "720p_hunyuan": Workload("720p_hunyuan", B=1, H=24, d=128, T=33, fh=45, fw=80, sparsity=0.90),
    "720p_wan": Workload("720p_wan", B=1, H=40, d=128, T=21, fh=45, fw=80, sparsity=0.75),
    "long": Workload("long", B=1, H=24, d=128, T=65, fh=45, fw=80, sparsity=0.90, drift=True),
}

# Beyond the baseline file: the window and frame shape of the paper's own experiments (Section 4.1):
# 8x16 patches, i.e. 128-token blocks, on a 48x80 latent grid that they divide.
EXTRA_CONFIGS = {
    "768p_8x16": Workload("768p_8x16", B=1, H=24, d=128, T=33, fh=48, fw=80, ph=8, pw=16, sparsity=0.90),
}


# ----------------------------------------------------------------------------
# storage-format helpers (format conversion only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x64: np.ndarray, dtype: int) -> np.ndarray:
    """float64 -> stored array: float32 values, or uint16 bf16 bit patterns."""
    if dtype == F32:
        return x64.astype(np.float32)
    return f32_to_bf16_bits(x64.astype(np.float32))


def storage_to_f64(x: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == F32:
        return np.asarray(x, dtype=np.float32).astype(np.float64)
    return bf16_bits_to_f32(x).astype(np.float64)


# ----------------------------------------------------------------------------
# the generator
# ----------------------------------------------------------------------------
def _smooth_field(rng: np.random.Generator, w: Workload) -> np.ndarray:
    """Sum of 8 random Fourier modes per channel over (t, y, x); returns [N, d] float64."""
    d, T, fh, fw = w.d, w.T, w.fh, w.fw
    f = rng.uniform(-1.0 / 16.0, 1.0 / 16.0, (d, 8, 3))
    phi = rng.uniform(0.0, 2.0 * np.pi, (d, 8))
    ang_t = 2.0 * np.pi * f[None, :, :, 0] * np.arange(T)[:, None, None] + phi[None]
    if w.drift:
        ang_t = ang_t + np.cumsum(rng.normal(0.0, 0.15, (T, d, 8)), axis=0)
    ang_y = 2.0 * np.pi * f[None, :, :, 1] * np.arange(fh)[:, None, None]
    ang_x = 2.0 * np.pi * f[None, :, :, 2] * np.arange(fw)[:, None, None]
    # cos(a+b+c) evaluated separably through complex exponentials per axis
    ety = np.exp(1j * ang_t)[:, None] * np.exp(1j * ang_y)[None]          # [T, fh, d, 8]
    ex = np.exp(1j * ang_x)                                               # [fw, d, 8]
    ety = ety.reshape(T * fh, d, 8)
    out = np.empty((T * fh, fw, d), dtype=np.float64)
    er, ei = np.ascontiguousarray(ety.real), np.ascontiguousarray(ety.imag)
    xr, xi = np.ascontiguousarray(ex.real), np.ascontiguousarray(ex.imag)
    for c0 in range(0, d, 16):                                            # bounded temporaries
        sl = slice(c0, c0 + 16)
        out[:, :, sl] = (np.einsum("acm,xcm->axc", er[:, sl], xr[:, sl])
                         - np.einsum("acm,xcm->axc", ei[:, sl], xi[:, sl]))
    return out.reshape(T * fh * fw, d)


def make_head(w: Workload, b: int, h: int):
    """Q, K, V for one (batch, head) in storage format, each [N, d]."""
    rng = np.random.default_rng([w.seed, b, h])
    smooth = _smooth_field(rng, w)
    N, d = w.N, w.d
    q = smooth + rng.normal(0.0, 0.3, (N, d))
    k = smooth + rng.normal(0.0, 0.3, (N, d))
    v = rng.normal(0.0, 1.0, (N, d))
    return to_storage(q, w.dtype), to_storage(k, w.dtype), to_storage(v, w.dtype)


def make_qkv(w: Workload, heads=None, threads: int = 8):
    """Q, K, V for the whole problem, [B, H', N, d] in storage format.

    ``heads`` (an iterable of head numbers) restricts generation to those heads, in
    that order; each head's content depends only on (seed, b, h).  Heads are made on a
    small thread pool (NumPy releases the GIL in the heavy parts); no processes are
    started, so this is safe to call from a process that already uses the GPU.
    """
    from concurrent.futures import ThreadPoolExecutor
    heads = list(range(w.H)) if heads is None else list(heads)
    np_dtype = np.float32 if w.dtype == F32 else np.uint16
    shape = (w.B, len(heads), w.N, w.d)
    Q, K, V = (np.empty(shape, np_dtype) for _ in range(3))

    def one(job):
        b, i, h = job
        Q[b, i], K[b, i], V[b, i] = make_head(w, b, h)

    jobs = [(b, i, h) for b in range(w.B) for i, h in enumerate(heads)]
    if threads <= 1 or len(jobs) == 1:
        for job in jobs:
            one(job)
    else:
        with ThreadPoolExecutor(min(threads, len(jobs))) as ex:
            list(ex.map(one, jobs))
    return Q, K, V
