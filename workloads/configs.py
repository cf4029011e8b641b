"""The synthetic workloads: shapes and distributions only, no arithmetic.

Each entry stands in for a long-context inference workload on a
Llama-3.1-8B-shaped attention layer (the paper evaluates on LongBench and
LongBenchV2 prompts, Sec. 5; those prompts, the model weights and their
activations are not available, so tensors of the same shape with controlled
statistics are drawn instead).  The paper's defaults that matter here: the
first 32 tokens are always preserved (Sec. 5, implementation details).
"""

from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int                 # enters the sub-seed of every tensor
    layers: int
    n_seq: int
    n_kv_heads: int
    group: int                  # G: query heads per KV head
    window: int                 # W: recent queries per query head
    head_dim: int               # D = d_k = d_v
    dtype: str                  # "f32" | "bf16": dtype of Q, K, V and of the merged K, V
    # token count per sequence: ("fixed", n) or ("uniform", lo, hi) (inclusive, drawn per sequence)
    length: Tuple
    # budget per sequence: ("fixed", B) or ("fraction", num, den) -> floor(n * num / den)
    budget: Tuple
    # AR(1) coefficient of the Keys along tokens: ("fixed", rho) or ("uniform", lo, hi) per (seq, head)
    k_rho: Tuple
    k_outlier_channels: int = 0     # channels (drawn per unit) whose Keys are scaled
    k_outlier_scale: float = 1.0
    v_dist: str = "normal"          # "normal" | "student_t4" (scaled to unit variance)
    n_sink: int = 32
    n_recent: int = 0
    # Streaming regime: the rows are slots of an already merged cache.  fresh_tail = number of trailing
    # rows that are new tokens (cardinality 1, like the sinks); every other row stands for
    # 1 + Geometric(1 / mean_count) - 1 tokens (mean `mean_count`) and its Value row is the sum of that
    # many unit-variance draws.  mean_count = 0: plain tokens, no cardinalities.
    mean_count: float = 0.0
    fresh_tail: int = 0
    seed: int = 20260300907

    @property
    def n_units(self) -> int:
        return self.n_seq * self.n_kv_heads

    @property
    def q_rows(self) -> int:
        return self.group * self.window

    def scaled(self, **kw) -> "Workload":
        """A variant of the same recipe (e.g. fewer tokens) for quick tests."""
        return replace(self, **kw)


WORKLOADS = {
    # 1 layer, 1 KV head, 1 query head, head_dim 64, fp32; 1024 tokens, window 8, budget 512.
    "tiny": Workload(
        name="tiny", cfg_id=1, layers=1, n_seq=1, n_kv_heads=1, group=1, window=8,
        head_dim=64, dtype="f32", length=("fixed", 1024), budget=("fixed", 512),
        k_rho=("fixed", 0.9)),
    # one Llama-3.1-8B attention layer: 32 q heads / 8 KV heads / head_dim 128, bf16; 8192 -> 2048.
    "llama8b_8k": Workload(
        name="llama8b_8k", cfg_id=2, layers=1, n_seq=1, n_kv_heads=8, group=4, window=32,
        head_dim=128, dtype="bf16", length=("fixed", 8192), budget=("fixed", 2048),
        k_rho=("fixed", 0.9), k_outlier_channels=4, k_outlier_scale=8.0),
    # headline: same layout at 32768 tokens -> 4096, all 32 layers one after the other.
    "llama8b_32k": Workload(
        name="llama8b_32k", cfg_id=3, layers=32, n_seq=1, n_kv_heads=8, group=4, window=32,
        head_dim=128, dtype="bf16", length=("fixed", 32768), budget=("fixed", 4096),
        k_rho=("fixed", 0.9), k_outlier_channels=4, k_outlier_scale=8.0),
    # ragged batch: 16 sequences, lengths U{4096..65536}, budget 25 % of the length.
    "ragged16": Workload(
        name="ragged16", cfg_id=4, layers=1, n_seq=16, n_kv_heads=8, group=4, window=32,
        head_dim=128, dtype="bf16", length=("uniform", 4096, 65536), budget=("fraction", 1, 4),
        k_rho=("uniform", 0.7, 0.98)),
    # stress: 64 q heads over 8 KV heads, 131072 tokens -> 8192, window 64, heavy-tailed Values.
    "stress128k": Workload(
        name="stress128k", cfg_id=5, layers=1, n_seq=1, n_kv_heads=8, group=8, window=64,
        head_dim=128, dtype="bf16", length=("fixed", 131072), budget=("fixed", 8192),
        k_rho=("fixed", 0.95), v_dist="student_t4"),
    # streaming regime of Sec. 5: a cache of budget + chunk = 2048 + 512 slots is merged back to 2048;
    # the 2016 old non-sink slots stand for 4 tokens on average (about 8.6 K tokens seen so far).
    "stream2560": Workload(
        name="stream2560", cfg_id=6, layers=32, n_seq=1, n_kv_heads=8, group=4, window=32,
        head_dim=128, dtype="bf16", length=("fixed", 2560), budget=("fixed", 2048),
        k_rho=("fixed", 0.9), k_outlier_channels=4, k_outlier_scale=8.0, mean_count=4.0, fresh_tail=512),
    # Qwen2-7B layout (Sec. 5 evaluates it beside Llama-3.1-8B and Mistral-7B): 28 q heads over 4 KV heads, so a
    # window of 32 queries gives 224 query rows per unit (more than one pass of the 128-row score kernel).
    "qwen7b_32k": Workload(
        name="qwen7b_32k", cfg_id=7, layers=28, n_seq=1, n_kv_heads=4, group=7, window=32,
        head_dim=128, dtype="bf16", length=("fixed", 32768), budget=("fixed", 4096),
        k_rho=("fixed", 0.9), k_outlier_channels=4, k_outlier_scale=8.0),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]
