"""Seeded synthetic Q/K/V generators for the S2O prefill-attention path.

This module serves both the CPU oracle and the HIP path and therefore holds
none of the method's arithmetic: it only draws random tensors with planted
structure (attention sinks, heavy "vertical stripe" key tokens, a slow
positional component shared by Q and K that yields a local diagonal) and
rounds them once to bf16.  The inputs stand in for Llama-3.1-8B activations
on long-context prompts (paper Sec. 4.1), which are not available offline.

Tensors are returned as numpy uint16 arrays holding bf16 bit patterns:
    Q [Z, H, L, D],  K [Z, Hkv, L, D],  V [Z, Hkv, L, D]
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Tuple

import numpy as np

_TENSOR_ID = {"q": 1, "k": 2, "v": 3, "walk": 4, "u": 5, "heavy": 6, "strength": 7,
              "redraw": 8}


@dataclass(frozen=True)
class Workload:
    """Shape + generator recipe + the method parameters a config is run with."""
    name: str
    Z: int = 1
    H: int = 1
    Hkv: int = 1
    L: int = 2048
    D: int = 128
    S: int = 256            # segment length
    BM: int = 64
    BN: int = 64
    seed: int = 0
    # planted structure
    n_sinks: int = 4
    heavy_rate: float = 0.01        # fraction of key positions boosted (uniform draw)
    n_bursts: int = 0               # >0: heavy set = bursts of `burst_len` tokens instead
    burst_len: int = 32
    k_boost: float = 3.0            # K[heavy] += k_boost * u
    q_boost: float = 1.0            # Q[:]     += q_boost * u
    u_norm: float = 1.0             # |u|
    walk: str = "literal"           # "literal": w_t = w_{t-1} + N(0, sigma^2)
                                    # "ar1":     w_t = rho w_{t-1} + N(0, sigma^2)
    walk_sigma: float = 0.05
    walk_rho: float = 1.0 - 1.0 / 4096.0
    walk_strength: Tuple[float, float] = (0.5, 0.5)   # U[lo, hi] per KV head
    unstructured_groups: int = 0    # first this many KV groups are pure N(0,1)
    taus: Tuple[float, ...] = (0.0,)

    @property
    def G(self) -> int:
        return self.H // self.Hkv

    @property
    def N(self) -> int:
        return self.L // self.S


def _rng(seed: int, tensor: str, *key: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([seed, _TENSOR_ID[tensor], *key]))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _walk(w: Workload, z: int, g: int) -> np.ndarray:
    """Slow positional component w_t in R^D for KV head g (fp32 [L, D])."""
    noise = _rng(w.seed, "walk", z, g).standard_normal((w.L, w.D), dtype=np.float32)
    noise *= np.float32(w.walk_sigma)
    if w.walk == "literal":
        return np.cumsum(noise, axis=0, dtype=np.float64).astype(np.float32)
    from scipy.signal import lfilter
    return lfilter([1.0], [1.0, -w.walk_rho], noise.astype(np.float64), axis=0).astype(np.float32)


def heavy_positions(w: Workload, z: int, g: int) -> np.ndarray:
    """Sorted positions of the boosted key tokens of KV head g."""
    r = _rng(w.seed, "heavy", z, g)
    pos = set(range(min(w.n_sinks, w.L)))
    if w.n_bursts > 0:
        starts = r.integers(0, w.L - w.burst_len, size=w.n_bursts)
        for s in starts:
            pos.update(range(int(s), int(s) + w.burst_len))
    else:
        k = int(round(w.heavy_rate * w.L))
        pos.update(int(p) for p in r.choice(w.L, size=k, replace=False))
    return np.array(sorted(pos), dtype=np.int64)


def make_qkv(w: Workload) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    Q = np.empty((w.Z, w.H, w.L, w.D), dtype=np.uint16)
    K = np.empty((w.Z, w.Hkv, w.L, w.D), dtype=np.uint16)
    V = np.empty((w.Z, w.Hkv, w.L, w.D), dtype=np.uint16)
    for z in range(w.Z):
        for g in range(w.Hkv):
            structured = g >= w.unstructured_groups
            k = _rng(w.seed, "k", z, g).standard_normal((w.L, w.D), dtype=np.float32)
            v = _rng(w.seed, "v", z, g).standard_normal((w.L, w.D), dtype=np.float32)
            if structured:
                u = _rng(w.seed, "u", z, g).standard_normal(w.D).astype(np.float32)
                u *= np.float32(w.u_norm / np.linalg.norm(u.astype(np.float64)))
                lo, hi = w.walk_strength
                a = np.float32(lo + (hi - lo) * _rng(w.seed, "strength", z, g).random())
                wk = _walk(w, z, g) * a
                k += wk
                k[heavy_positions(w, z, g)] += np.float32(w.k_boost) * u
            K[z, g] = f32_to_bf16_bits(k)
            V[z, g] = f32_to_bf16_bits(v)
            del k, v
            for j in range(w.G):
                h = g * w.G + j
                q = _rng(w.seed, "q", z, h).standard_normal((w.L, w.D), dtype=np.float32)
                if structured:
                    q += wk
                    q += np.float32(w.q_boost) * u
                Q[z, h] = f32_to_bf16_bits(q)
                del q
    return Q, K, V


def redraw_rows(w: Workload, X: np.ndarray, tensor: str, z: int, head: int, rows, attempt: int,
                pooled: int = 0) -> None:
    """Replace the N(0,1) part of the listed rows of Q ("q") or K ("k") head `head` by a
    fresh draw, in place.  Used by test fixtures that want inputs with no two ranking scores
    closer than a guard gap; what counts as "too close" is decided by the caller.

    pooled > 0: rows are grouped in consecutive ranges of `pooled` rows whose column sums
    should stay put (up to bf16 rounding); the change of each range's sum is absorbed by the
    highest row of the range that is not being re-drawn.  For K only the first range is
    treated this way."""
    rows = np.asarray(sorted({int(r) for r in rows}), dtype=np.int64)
    if rows.size == 0:
        return
    old = bf16_bits_to_f32(X[z, head, rows])
    fresh = _rng(w.seed, "redraw", _TENSOR_ID[tensor], z, head, attempt).standard_normal(
        (rows.size, w.D), dtype=np.float32)
    # new row = old row with its noise part replaced: the structure (old minus a unit
    # normal) is not known exactly after earlier re-draws, so mix instead of subtracting
    new = old + np.float32(0.5) * fresh
    newbits = f32_to_bf16_bits(new)
    X[z, head, rows] = newbits
    if pooled > 0:
        delta = bf16_bits_to_f32(newbits) - old
        for rng_id in np.unique(rows // pooled):
            if tensor == "k" and rng_id != 0:
                continue
            sel = rows // pooled == rng_id
            sink = (rng_id + 1) * pooled - 1
            taken = set(rows[sel].tolist())
            while sink in taken:
                sink -= 1
            if sink < rng_id * pooled:
                continue
            srow = bf16_bits_to_f32(X[z, head, sink]) - delta[sel].sum(axis=0)
            X[z, head, sink] = f32_to_bf16_bits(srow)


# ---------------------------------------------------------------------------
# The five workloads (shapes, structure and parameters of the benchmark configs)
# ---------------------------------------------------------------------------
_LLAMA = dict(Z=1, H=32, Hkv=8, D=128, BM=64, BN=64, n_sinks=4, walk="ar1",
              walk_strength=(0.2, 0.8))

WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload(name="tiny", L=2048, S=256, heavy_rate=0.01, taus=(0.0, 0.05)),
    "llama8k": Workload(name="llama8k", L=8192, S=1024, heavy_rate=0.005,
                        taus=(0.0, 1e-4, 1e-3, 1e-2), **_LLAMA),
    "llama32k": Workload(name="llama32k", L=32768, S=2048, n_bursts=16, burst_len=32,
                         taus=(1e-3,), **_LLAMA),
    "llama128k": Workload(name="llama128k", L=131072, S=2048, heavy_rate=0.005,
                          taus=(1e-5, 1e-4, 3e-4, 1e-3, 2e-3, 5e-3, 1e-2, 2e-2), **_LLAMA),
    "mixed128k": Workload(name="mixed128k", L=131072, S=2048, heavy_rate=0.005,
                          k_boost=5.0, unstructured_groups=4, taus=(5e-3,), **_LLAMA),
}


def workload(name: str, **overrides) -> Workload:
    return replace(WORKLOADS[name], **overrides)
