"""Seeded synthetic inputs shaped like the paper's video-DiT attention workloads.

This module only draws numbers and names shapes.  It holds none of the method's
arithmetic (no mask rule, no attention, no scaling) so that both the CPU oracle's
tests and the HIP path's callers can take their inputs from it without sharing code.

The real workloads (Wan2.1 1.3B / 14B activations on VBench prompts, Sec. 5.1) are not
available; these tensors take their shapes, dtypes and value ranges and stand in for them.

Random stream: a counter-based generator written out here (splitmix64 finaliser over
`key + counter`, Box-Muller for normals) so that values do not depend on any library's
RNG version.  Every tensor has its own key derived from (seed, tag); drawing one tensor
never shifts another.
"""
from __future__ import annotations

import concurrent.futures
import dataclasses
import os
from typing import Dict, List, Optional, Tuple

import numpy as np

_U64 = np.uint64
_MASK53 = _U64((1 << 53) - 1)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 output function applied elementwise to uint64 counters."""
    with np.errstate(over="ignore"):
        z = x + _U64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)
        z = z ^ (z >> _U64(31))
    return z


def _key(seed: int, tag: str) -> np.uint64:
    k = np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=_U64)
    for ch in tag.encode():
        with np.errstate(over="ignore"):
            k = _splitmix64(k ^ _U64(ch))
    return k[0]


def _uniform01(key: np.uint64, start: int, count: int) -> np.ndarray:
    """`count` doubles in (0, 1), counters start..start+count-1 of stream `key`."""
    ctr = np.arange(start, start + count, dtype=_U64)
    with np.errstate(over="ignore"):
        bits = _splitmix64(ctr * _U64(0xD1342543DE82EF95) + key)
    return ((bits >> _U64(11)) & _MASK53).astype(np.float64) * (1.0 / (1 << 53)) + (0.5 / (1 << 53))


def uniform(seed: int, tag: str, shape, lo: float = 0.0, hi: float = 1.0) -> np.ndarray:
    n = int(np.prod(shape))
    u = _uniform01(_key(seed, tag), 0, n)
    return (lo + (hi - lo) * u).reshape(shape)


def _normal_chunk(key: np.uint64, std: float, out: np.ndarray, s: int, c: int) -> None:
    u = _uniform01(key, 2 * s, 2 * c)
    r = np.sqrt(-2.0 * np.log(u[0::2]))
    out[s:s + c] = (std * r * np.cos(2.0 * np.pi * u[1::2])).astype(np.float32)


def normal(seed: int, tag: str, shape, std: float = 1.0, chunk: int = 1 << 20) -> np.ndarray:
    """N(0, std^2) float32 array; element i uses counters 2i and 2i+1 (Box-Muller, cosine branch).
    Chunks are filled by a small thread pool; the values do not depend on the chunking."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    key = _key(seed, tag)
    starts = list(range(0, n, chunk))
    if len(starts) <= 1:
        for s in starts:
            _normal_chunk(key, std, out, s, min(chunk, n - s))
    else:
        workers = max(1, min(16, os.cpu_count() or 1))
        with concurrent.futures.ThreadPoolExecutor(workers) as ex:
            list(ex.map(lambda s: _normal_chunk(key, std, out, s, min(chunk, n - s)), starts))
    return out.reshape(shape)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    with np.errstate(over="ignore"):
        r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(x.shape)


@dataclasses.dataclass(frozen=True)
class Workload:
    """One benchmark configuration: shapes, dtype and the seeded recipe."""
    name: str
    B: int
    H: int
    d: int
    T: int
    Hh: int
    W: int
    dtype: str            # "f32" or "bf16"
    sparsity: float       # fraction of KV blocks dropped per query block
    seed: int
    block: int = 64
    input_head_scale: bool = False   # Mid config: per-head U(0.5,2) magnitude on Q, K, V
    lam: float = 1.0
    eps: float = 1e-6

    @property
    def N(self) -> int:
        return self.T * self.Hh * self.W

    @property
    def D(self) -> int:
        return self.H * self.d

    @property
    def nb(self) -> int:
        return (self.N + self.block - 1) // self.block

    def with_sparsity(self, sparsity: float, name: Optional[str] = None) -> "Workload":
        return dataclasses.replace(self, sparsity=sparsity,
                                   name=name or f"{self.name}@{sparsity:g}")


# Shapes follow the paper's Wan2.1 settings (Sec. 5.1): 480p ~30k tokens, 720p ~100k tokens,
# 12 heads x 128 for the 1.3B model and 40 x 128 for the 14B model.
TINY = Workload("tiny", 1, 2, 64, 4, 16, 16, "f32", 0.75, seed=0)
MID = Workload("mid", 1, 12, 128, 8, 30, 52, "bf16", 0.75, seed=1, input_head_scale=True)
WAN13_480P = Workload("wan1.3b-480p", 1, 12, 128, 21, 30, 52, "bf16", 0.90, seed=2)
WAN14_720P = Workload("wan14b-720p", 1, 40, 128, 21, 45, 80, "bf16", 0.90, seed=3)
SWEEP = [WAN13_480P.with_sparsity(s) for s in (0.0, 0.5, 0.75, 0.90, 0.95)]

WORKLOADS: Dict[str, Workload] = {w.name: w for w in (TINY, MID, WAN13_480P, WAN14_720P)}


def small(name: str, B: int, H: int, d: int, T: int, Hh: int, W: int, dtype: str,
          sparsity: float, seed: int, **kw) -> Workload:
    """Ad-hoc workload for tests (ragged tails, several tiles, odd grids)."""
    return Workload(name, B, H, d, T, Hh, W, dtype, sparsity, seed, **kw)


def head_kinds(w: Workload) -> np.ndarray:
    """Synthetic head assignment: odd heads use the temporal token order, even heads the default."""
    return (np.arange(w.H) % 2).astype(np.uint8)


def make_inputs(w: Workload, want_x: bool = True) -> Dict[str, np.ndarray]:
    """Draw Q, K, V [B,H,N,d], X_t [B,N,D], gate weights [D], static per-head scale [H].

    All returned arrays are float32.  For a bf16 workload the values of Q, K, V and X_t are
    already rounded to bfloat16, so a bf16 device copy is exact and a CPU checker that reads
    the float32 arrays sees the same numbers as the GPU.
    """
    B, H, N, d, D = w.B, w.H, w.N, w.d, w.D
    out: Dict[str, np.ndarray] = {}
    mult = {}
    if w.input_head_scale:
        for t in "qkv":
            mult[t] = uniform(w.seed, f"in_scale_{t}", (H,), 0.5, 2.0).astype(np.float32)
    for t in "qkv":
        x = normal(w.seed, t, (B, H, N, d))
        if w.input_head_scale:
            x *= mult[t][None, :, None, None]
        out[t] = round_to_bf16(x) if w.dtype == "bf16" else x
    if want_x:
        x = normal(w.seed, "x_t", (B, N, D))
        out["x_t"] = round_to_bf16(x) if w.dtype == "bf16" else x
    out["w_gate"] = normal(w.seed, "w_gate", (D,), std=0.02)
    out["head_scale"] = uniform(w.seed, "head_scale", (H,), 0.0, 1.0).astype(np.float32)
    return out


def sample_blocks(nb: int, count: int, seed: int) -> np.ndarray:
    """Query blocks used for sampled parity at full size: first, last (the ragged tail), the
    block before it, and seeded picks in between; ascending and unique."""
    fixed = {0, nb - 1, max(0, nb - 2), nb // 2}
    if count >= nb:
        return np.arange(nb, dtype=np.int32)
    u = uniform(seed, "sample_blocks", (4 * count,))
    for x in u:
        if len(fixed) >= count:
            break
        fixed.add(int(x * nb) % nb)
    return np.array(sorted(fixed), dtype=np.int32)


def rope_tables(T: int, Hh: int, W: int, d: int, base: float = 10000.0):
    """Cosine and sine tables [N, d/2] (float32) of a 3D rotary embedding for the token grid, token n = (t, y, x) in
    stored order: the d/2 channel pairs are split over the t, y, x axes (the remainder goes to t) and pair i of an
    axis with m pairs turns by position * base^(-i/m).  An input generator like the others: the layer only ever
    sees the two tables."""
    half = d // 2
    my = mx = half // 3
    mt = half - my - mx
    n = np.arange(T * Hh * W)
    pos = {"t": n // (Hh * W), "y": (n // W) % Hh, "x": n % W}
    cols = []
    for axis, m in (("t", mt), ("y", my), ("x", mx)):
        freq = base ** (-np.arange(m, dtype=np.float64) / max(m, 1))
        cols.append(pos[axis][:, None].astype(np.float64) * freq[None, :])
    theta = np.concatenate(cols, axis=1)
    return np.cos(theta).astype(np.float32), np.sin(theta).astype(np.float32)
