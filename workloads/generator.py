"""Counter-based, order-independent generation of one unit's Q, K, V.

A *unit* is one (layer, sequence, KV head).  Every tensor gets its own Philox
stream keyed by (workload seed; cfg_id, layer, seq, head, tensor, attempt), so
the values never depend on the order or the number of threads in which units
are drawn.  `attempt` only enters the Query stream: a caller that has to
reject a unit (for instance because an acceptance test of its own fails)
redraws the Queries and keeps K and V.

Values are drawn in float32/float64, rounded ONCE (round-to-nearest-even) to the
workload's I/O dtype and handed out widened to float32: those rounded values
are the inputs of every consumer.
"""

from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np
from scipy.signal import lfilter

from .configs import Workload

_T_LEN, _T_RHO, _T_OUTLIER, _T_K, _T_V, _T_Q, _T_COUNT = range(7)


def _rng(w: Workload, layer: int, seq: int, head: int, tensor: int, attempt: int = 0):
    ss = np.random.SeedSequence(entropy=w.seed,
                                spawn_key=(w.cfg_id, layer, seq, head, tensor, attempt))
    return np.random.Generator(np.random.Philox(ss))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _round_io(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x))
    raise ValueError(f"unknown dtype {dtype!r}")


def unit_lengths(w: Workload) -> List[int]:
    """Token count of every sequence (fixed by the workload seed)."""
    kind = w.length[0]
    if kind == "fixed":
        return [int(w.length[1])] * w.n_seq
    if kind == "uniform":
        lo, hi = int(w.length[1]), int(w.length[2])
        return [int(_rng(w, 0, s, 0, _T_LEN).integers(lo, hi, endpoint=True)) for s in range(w.n_seq)]
    raise ValueError(kind)


def unit_budget(w: Workload, n: int) -> int:
    kind = w.budget[0]
    if kind == "fixed":
        return int(w.budget[1])
    if kind == "fraction":
        return (n * int(w.budget[1])) // int(w.budget[2])
    raise ValueError(kind)


@dataclass
class UnitInputs:
    layer: int
    seq: int
    head: int
    attempt: int
    n: int
    budget: int
    rho: float
    Q: np.ndarray   # [G, W, D] float32, values representable in the I/O dtype
    K: np.ndarray   # [n, D]
    V: np.ndarray   # [n, D]
    counts: Optional[np.ndarray] = None   # [n] int32 tokens every row stands for (streaming workloads only)


def _draw_k(w: Workload, layer: int, seq: int, head: int, n: int):
    kind = w.k_rho[0]
    if kind == "fixed":
        rho = float(w.k_rho[1])
    else:
        rho = float(_rng(w, layer, seq, head, _T_RHO).uniform(w.k_rho[1], w.k_rho[2]))
    d = w.head_dim
    eps = _rng(w, layer, seq, head, _T_K).standard_normal((n, d), dtype=np.float32).astype(np.float64)
    # AR(1) along tokens, k_t = rho k_{t-1} + eps_t, started in its stationary law.
    eps[0] /= np.sqrt(1.0 - rho * rho)
    k = lfilter([1.0], [1.0, -rho], eps, axis=0)
    if w.k_outlier_channels:
        ch = _rng(w, layer, seq, head, _T_OUTLIER).choice(d, size=w.k_outlier_channels, replace=False)
        k[:, ch] *= w.k_outlier_scale
    return rho, k


def _draw_v(w: Workload, layer: int, seq: int, head: int, n: int):
    g = _rng(w, layer, seq, head, _T_V)
    if w.v_dist == "normal":
        return g.standard_normal((n, w.head_dim), dtype=np.float32)
    if w.v_dist == "student_t4":
        # Var[t_4] = 4 / (4 - 2) = 2
        return g.standard_t(4.0, size=(n, w.head_dim)) / np.sqrt(2.0)
    raise ValueError(w.v_dist)


def _draw_counts(w: Workload, layer: int, seq: int, head: int, n: int) -> np.ndarray:
    """Cardinality of every row: 1 for the sink rows and the fresh tail, geometric with mean mean_count
    for the slots in between."""
    c = np.ones(n, dtype=np.int32)
    lo, hi = min(w.n_sink, n), max(min(w.n_sink, n), n - w.fresh_tail)
    if hi > lo:
        c[lo:hi] = _rng(w, layer, seq, head, _T_COUNT).geometric(1.0 / w.mean_count, size=hi - lo)
    return c


def _draw_q(w: Workload, layer: int, seq: int, head: int, attempt: int):
    return _rng(w, layer, seq, head, _T_Q, attempt).standard_normal(
        (w.group, w.window, w.head_dim), dtype=np.float32)


def generate_unit(w: Workload, layer: int, seq: int, head: int, attempt: int = 0,
                  n: Optional[int] = None, kv_from: Optional[UnitInputs] = None) -> UnitInputs:
    """Draw one unit.  `kv_from` reuses K and V of an earlier attempt (only Q is redrawn)."""
    if n is None:
        n = unit_lengths(w)[seq]
    counts = None
    if kv_from is not None:
        rho, K, V, counts = kv_from.rho, kv_from.K, kv_from.V, kv_from.counts
    else:
        rho, k = _draw_k(w, layer, seq, head, n)
        K = _round_io(k, w.dtype)
        v = _draw_v(w, layer, seq, head, n)
        if w.mean_count > 0:
            # a slot's Value row is a sum over its tokens: the sum of c unit-variance draws is one draw
            # scaled by sqrt(c)
            counts = _draw_counts(w, layer, seq, head, n)
            v = v * np.sqrt(counts.astype(np.float64))[:, None]
        V = _round_io(v, w.dtype)
    Q = _round_io(_draw_q(w, layer, seq, head, attempt), w.dtype)
    return UnitInputs(layer=layer, seq=seq, head=head, attempt=attempt, n=n,
                      budget=unit_budget(w, n), rho=rho, Q=Q, K=K, V=V, counts=counts)


def gaussian_unit(seed: int, n: int, head_dim: int, group: int, window: int, dtype: str, k_scale: float = 2.0):
    """A unit of independent Gaussian rows (no correlation along tokens, no outlier channels), for tests whose
    length makes the recipe above too slow to draw: (Q [G, W, D], K [n, D], V [n, D]) as float32 arrays that are
    exactly representable in `dtype`."""
    rng = np.random.default_rng([0x6B7673, seed])
    K = _round_io(k_scale * rng.standard_normal((n, head_dim), dtype=np.float32), dtype)
    V = _round_io(rng.standard_normal((n, head_dim), dtype=np.float32), dtype)
    Q = _round_io(rng.standard_normal((group, window, head_dim), dtype=np.float32), dtype)
    return Q, K, V
