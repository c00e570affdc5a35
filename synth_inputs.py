"""Seeded synthetic Q/K/V generators shared by the tests, the benchmark and the CPU oracle's callers.

This module holds no arithmetic of the method itself: it only draws inputs.  The tensors stand in
for video-transformer activations (not available offline): a sum of a few low-frequency 3-D Fourier
features over the (t, y, x) token grid, which makes neighbouring key tokens similar (the property
the paper's Fig. 2 reports for real models), plus white Gaussian noise.

Recipe, for every (batch, head):
    p_n      = (t/T, y/Hg, x/W) of token n in raster order of the grid
    f_m      integer frequency vectors, m = 1..8, shared by Q and K of the head
    A_m, phi_m  per tensor (Q, K, V): A_m ~ N(0,1)/sqrt(8) in R^d, phi_m ~ U[0, 2 pi) in R^d
    X[n]     = g * ( sum_m A_m * cos(2 pi f_m . p_n + phi_m) + 0.5 * eps_n ),  eps_n ~ N(0, I)
    g        per-head gain ~ N(1, 0.1) (1 for the tiny config)
Draw order is fixed (bank, gain, then Q, K, V) with numpy's PCG64 so every consumer sees the same
bytes.  bfloat16 tensors are returned as uint16 bit patterns (numpy has no bfloat16).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 20251204


# --------------------------------------------------------------------------- dtype helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit pattern (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit pattern (uint16) -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Stored tensor (float32 array, or uint16 bf16 bits) -> float64 values."""
    if dtype == "bf16":
        return bf16_bits_to_f32(x).astype(np.float64)
    return np.asarray(x, dtype=np.float32).astype(np.float64)


# --------------------------------------------------------------------------- workload descriptions
@dataclass(frozen=True)
class Workload:
    """One attention problem: shapes, block sizes, pyramid depth and the allocation rule."""
    name: str
    index: int                    # config index -> seed = BASE_SEED + index
    B: int
    Hq: int
    Hkv: int
    N: int
    d: int
    grid: Tuple[int, int, int]    # (T, Hg, W) raster the field is drawn on
    bq: int
    bk: int
    levels: int
    dtype: str                    # "bf16" | "f32"
    causal: bool = False
    text_tokens: int = 0          # leading pure-noise tokens (video-LLM prompt text)
    budget: float = 0.2
    per_head_gain: bool = True
    per_head_band: bool = False   # frequency band {lo..lo+3}, lo drawn per head
    budgets: Tuple[float, ...] = field(default_factory=tuple)

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


CONFIGS = {
    # tiny fp32 case the oracle finishes in seconds
    "tiny": Workload("tiny", 0, B=1, Hq=2, Hkv=2, N=1024, d=64, grid=(4, 16, 16), bq=64, bk=64,
                     levels=4, dtype="f32", budget=0.25, per_head_gain=False, budgets=(0.25,)),
    # video-DiT-1.3B-shaped self-attention (the configuration the headline metric is quoted on)
    "dit1p3b": Workload("dit1p3b", 1, B=1, Hq=12, Hkv=12, N=32760, d=128, grid=(21, 30, 52), bq=128,
                        bk=64, levels=4, dtype="bf16", budget=0.2, budgets=(0.1, 0.2, 0.3)),
    # video-DiT-14B-shaped self-attention
    "dit14b": Workload("dit14b", 2, B=1, Hq=40, Hkv=40, N=75600, d=128, grid=(21, 45, 80), bq=128,
                       bk=64, levels=4, dtype="bf16", budget=0.2, per_head_band=True, budgets=(0.2,)),
    # video-LLM prefill: causal, grouped-query, 64 text tokens then visual tokens
    "vlm_prefill": Workload("vlm_prefill", 3, B=1, Hq=28, Hkv=4, N=32768, d=128, grid=(16, 46, 46),
                            bq=128, bk=64, levels=4, dtype="bf16", causal=True, text_tokens=64,
                            budget=0.25, budgets=(0.25,)),
    # stress / ablation: long sequence, d=64, 5 levels
    "stress": Workload("stress", 4, B=2, Hq=16, Hkv=16, N=131072, d=64, grid=(32, 64, 64), bq=128,
                       bk=128, levels=5, dtype="bf16", budget=0.2, per_head_band=True,
                       budgets=(0.05, 0.1, 0.2, 0.3, 0.4, 0.5)),
}


def small_variant(w: Workload, N: int, Hq: Optional[int] = None, Hkv: Optional[int] = None,
                  B: Optional[int] = None) -> Workload:
    """Same recipe on a shorter sequence / fewer heads (parity-test sizes).  The field keeps the
    original grid raster; only its first N tokens are used."""
    Hq = w.Hq if Hq is None else Hq
    Hkv = w.Hkv if Hkv is None else Hkv
    return replace(w, N=N, Hq=Hq, Hkv=Hkv, B=w.B if B is None else B, name=f"{w.name}_N{N}")


# --------------------------------------------------------------------------- generator
def _positions(w: Workload, n_field: int) -> np.ndarray:
    T, Hg, W = w.grid
    n = np.arange(n_field, dtype=np.int64)
    t = n // (Hg * W)
    y = (n // W) % Hg
    x = n % W
    return np.stack([t / T, y / Hg, x / W], axis=1)  # [n, 3]; t may exceed T-1 only if N > grid size


def _draw(rng: np.random.Generator, n_field: int, d: int, n_text: int):
    """Every random number one [N, d] tensor needs, in the fixed draw order (amplitudes, phases, noise,
    text rows).  Only this part touches the generator, so it stays on the calling thread."""
    A = rng.standard_normal((8, d)) / np.sqrt(8.0)
    phi = rng.uniform(0.0, 2.0 * np.pi, size=(8, d))
    noise = rng.standard_normal((n_field, d))
    text = rng.standard_normal((n_text, d)) if n_text else None
    return A, phi, noise, text


def _finish(draw, cos_n: np.ndarray, sin_n: np.ndarray, gain: float, dtype: str, out: np.ndarray) -> None:
    """The arithmetic of one tensor from its draws (no randomness: may run on a worker thread)."""
    A, phi, noise, text = draw
    # cos(theta_n + phi_d) = cos(theta_n) cos(phi_d) - sin(theta_n) sin(phi_d): two rank-8 products
    smooth = cos_n @ (A * np.cos(phi)) - sin_n @ (A * np.sin(phi))
    x = gain * (smooth + 0.5 * noise)
    if text is not None:
        x = np.concatenate([text, x], axis=0)
    out[...] = _store(x.astype(np.float32), dtype)


def _store(x32: np.ndarray, dtype: str) -> np.ndarray:
    return f32_to_bf16_bits(x32) if dtype == "bf16" else x32


def generate_qkv(w: Workload):
    """Return (Q, K, V): Q [B,Hq,N,d], K,V [B,Hkv,N,d]; float32 arrays for dtype 'f32', uint16
    bfloat16 bit patterns for 'bf16'.  Query head hq shares the frequency bank of its key/value
    head hq // (Hq // Hkv); everything else about it is drawn independently.  The random numbers are
    drawn on the calling thread in a fixed order; the arithmetic on them runs on a few worker threads
    (same operations on the same numbers: the bytes do not depend on the thread count)."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    rng = np.random.default_rng(w.seed)
    n_field = w.N - w.text_tokens
    pos = _positions(w, n_field)
    store_dt = np.uint16 if w.dtype == "bf16" else np.float32
    Q = np.empty((w.B, w.Hq, w.N, w.d), dtype=store_dt)
    K = np.empty((w.B, w.Hkv, w.N, w.d), dtype=store_dt)
    V = np.empty((w.B, w.Hkv, w.N, w.d), dtype=store_dt)
    group = w.Hq // w.Hkv
    workers = max(1, min(8, (os.cpu_count() or 2) - 1))
    pending = []
    with ThreadPoolExecutor(max_workers=workers) as pool:
        def submit(out, cos_n, sin_n):
            gain = float(rng.normal(1.0, 0.1)) if w.per_head_gain else 1.0
            draw = _draw(rng, n_field, w.d, w.text_tokens)
            pending.append(pool.submit(_finish, draw, cos_n, sin_n, gain, w.dtype, out))
            while len(pending) > 2 * workers:          # bounds the draws held in memory
                pending.pop(0).result()
        for b in range(w.B):
            for hk in range(w.Hkv):
                lo = int(rng.integers(0, 5)) if w.per_head_band else 0
                bank = rng.integers(lo, lo + 4, size=(8, 3)).astype(np.float64)
                phase_n = 2.0 * np.pi * (pos @ bank.T)          # [n_field, 8]
                cos_n, sin_n = np.cos(phase_n), np.sin(phase_n)
                for g in range(group):
                    submit(Q[b, hk * group + g], cos_n, sin_n)
                gain = float(rng.normal(1.0, 0.1)) if w.per_head_gain else 1.0
                for out in (K[b, hk], V[b, hk]):           # K and V share the head's gain
                    draw = _draw(rng, n_field, w.d, w.text_tokens)
                    pending.append(pool.submit(_finish, draw, cos_n, sin_n, gain, w.dtype, out))
        for f in pending:
            f.result()
    return Q, K, V


def random_qkv(seed: int, B: int, Hq: int, Hkv: int, N: int, d: int, dtype: str, std: float = 1.0):
    """Plain i.i.d. Gaussian tensors for small unit cases."""
    rng = np.random.default_rng(seed)
    Q = (std * rng.standard_normal((B, Hq, N, d))).astype(np.float32)
    K = (std * rng.standard_normal((B, Hkv, N, d))).astype(np.float32)
    V = (std * rng.standard_normal((B, Hkv, N, d))).astype(np.float32)
    return _store(Q, dtype), _store(K, dtype), _store(V, dtype)
