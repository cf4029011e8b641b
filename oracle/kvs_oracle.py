"""Plain fp64 CPU oracle of the KVSlimmer KV-cache merge step.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this module;
it exists so that the GPU library can be checked against an independent, slow
and obviously correct statement of what the step computes.  Only `tests/`,
`__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` use it.  It
shares no code with the HIP path and never rounds below fp64.

The method is a heuristic closed form, not a faster route to an independently
defined exact result, so the oracle is the algorithm itself, one step after the
other in the paper's notation, for one *unit* (one layer, one sequence, one KV
head):

  O1-O3  attention of every query row of the window over all cached Keys
         (Sec. 4.1, Eq. "attn_def_vec": e_i = q k_i^T / sqrt(d_k), alpha = softmax(e)),
         averaged over the R = G*W rows into one distribution alpha_bar.
  O4     o_bar = sum_t alpha_bar[t] V[t]            (same equation, with alpha_bar).
  O5-O6  adjacent pairs with the smallest accumulated attention mass are the
         merge candidates (App. C, paragraph (i)); edge score
         sigma[m] = alpha_bar[m] + alpha_bar[m+1]; the r = n - budget eligible edges
         with the smallest score are merged "in parallel", restoring the length
         to the budget in one step (Sec. 3.1, last paragraph).  The first n_sink
         tokens are always preserved (Sec. 5, implementation details).
  O7     consecutive selected edges chain into one output slot.
  O8     the forward-only vectors of Sec. 4.2 (Eqs. "c11_def"-"c12_def"):
         c_tt = alpha_t (1 - 2 alpha_t)(v_t - o),  c_{t,t+1} = -alpha_t alpha_{t+1}(v_t + v_{t+1} - 2o);
         A_t = ||c_tt||_2, C_t = ||c_{t,t+1}||_2.
  O9     merged Key: Eq. "kstar_final" for a pair,
         k* = [(A_m - C_m) k_m + (A_{m+1} - C_m) k_{m+1}] / (A_m - 2 C_m + A_{m+1});
         for a run of L > 2 tokens the same weight form (Eq. "kstar_weight_final_rewrite":
         w_a = sum_b g_ab / sum_ab g_ab) with the surrogate g_tt -> A_t,
         g_{t,t+1} -> -C_t of Eq. "cos_sign_relation_supp1" and only the diagonal and
         adjacent blocks kept.  Merged Value: the sum (Sec. 3.1, v* = v_m + v_{m+1}),
         with the slot's cardinality returned beside it.

Streaming regime (Sec. 3.1, last paragraph, and Sec. 5: the cache is compressed
again every time it exceeds the budget by a chunk): the input may itself be a
merged cache, every row a slot (k, V, c) that stands for c tokens sharing the Key
k whose Values add up to V (the "(k, k)" replacement of Sec. 3.1 carried along
with its cardinality).  For the attention output such a slot is exactly one token
with logit e + ln c and value V / c, and that is how every function below treats
it when `counts` is given: alpha_bar is then the slot's total mass, the residual
of O8 is V / c - o, merged Values stay sums and merged cardinalities add up.
Without `counts` every row is a plain token (c = 1).

Ablation rules for the merged Key (the paper's comparison of Sec. 3.1 / Sec. 4: what the off-diagonal
coupling buys): `rule="diagonal"` drops the coupling blocks (C_t := 0, the diagonal-only Hessian the
paper calls overlooked coupling), `rule="mean"` is the plain arithmetic mean of the run (over the tokens
the rows stand for).  Values, cardinalities and the partition are the same for every rule.

Per-query aggregation (an alternative to averaging the rows' attention first): Sec. 4 derives the
vectors c_tt, c_{t,t+1} for ONE query.  `per_query_norms` keeps every query row q of the window apart,
with its own alpha^{(q)} and its own output o^{(q)}, and averages the NORMS over the rows:
A_t = mean_q ||c_tt^{(q)}||, C_t = mean_q ||c_{t,t+1}^{(q)}||; `merge_compact(..., norms=(A, C))` then
uses them in the same weight form.  With one row it is the plain rule.  The partition still comes from
alpha_bar.

Causal window (`causal_window = W`): the paper does not say whether the window's queries see each other's
tokens.  With the mask, the W queries are those of the last W positions and each attends to the rows up
to its own position; without it (the default) every query row sees the whole cache.

Readings of points the paper leaves open (many query rows, ranking score, runs
longer than two, a non-positive denominator) are this module's and are listed
in the repository's design notes.

Parity pins (tests/test_oracle_pins.py): score / O8 / O9 are pinned by finite
differences of textbook attention, by brute-force minimisation of the
second-order objective, by the dense pseudo-inverse solution of Eq.
"optimal_k_cn", by identical-Key and lossless-Value special cases; select is
pinned by a brute-force sort and slot invariants; boundary_gap and conditioning (which decide what
seeded units the GPU tests accept) by worked examples and plain loops over explicit c-vectors.  The *choice* of the readings
P-1 (mean over query rows), P-2 (edge score) and P-3/P-4 (runs) is not fixed by
the paper: parity unpinned for those choices themselves.
"""

from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------- O1-O4
def attention_rows(Q: np.ndarray, K: np.ndarray, scale: Optional[float] = None,
                   counts: Optional[np.ndarray] = None, causal_window: int = 0) -> np.ndarray:
    """alpha[q, t] of Eq. "attn_def_vec" for every row q of Q [R, D] over K [n, D].

    With `counts`, row t of K stands for counts[t] tokens with that Key and alpha[q, t] is their total
    mass: c equal terms exp(e) in the softmax sums are one term exp(e + ln c).

    `causal_window = W > 0`: the rows of Q are [G, W] queries of the LAST W positions of the sequence,
    whose Keys are the last W rows of K; the query at window position w (row q with q mod W = w) sits
    at position n - W + w and attends to rows t <= n - W + w only (decoder attention)."""
    Q = np.asarray(Q, dtype=F64).reshape(-1, K.shape[-1])
    K = np.asarray(K, dtype=F64)
    if scale is None:
        scale = 1.0 / np.sqrt(K.shape[1])
    e = scale * (Q @ K.T)                                   # O1
    if counts is not None:
        e = e + np.log(np.asarray(counts, dtype=F64))[None, :]
    if causal_window:
        n, W = K.shape[0], int(causal_window)
        assert n >= W and Q.shape[0] % W == 0
        last_seen = n - W + (np.arange(Q.shape[0]) % W)
        e = np.where(np.arange(n)[None, :] <= last_seen[:, None], e, -np.inf)
    e = e - e.max(axis=1, keepdims=True)
    p = np.exp(e)
    return p / p.sum(axis=1, keepdims=True)                 # O2


def slot_values(V: np.ndarray, counts: Optional[np.ndarray]) -> np.ndarray:
    """The value a row contributes per unit of attention mass: V[t], or V[t] / counts[t] for a merged slot
    (its Values are a sum over counts[t] tokens)."""
    V = np.asarray(V, dtype=F64)
    if counts is None:
        return V
    return V / np.asarray(counts, dtype=F64)[:, None]


def score(Q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: Optional[float] = None,
          counts: Optional[np.ndarray] = None, causal_window: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """alpha_bar[n] (mean of the rows' attention) and o_bar[D] = sum_t alpha_bar[t] v[t]."""
    alpha = attention_rows(Q, K, scale, counts, causal_window)
    alpha_bar = alpha.mean(axis=0)                          # O3
    o_bar = alpha_bar @ slot_values(V, counts)              # O4
    return alpha_bar, o_bar


# --------------------------------------------------------------------------- O5-O7
def eligible_edges(n: int, n_sink: int, n_recent: int) -> Tuple[int, int]:
    """Edge m joins tokens m and m+1.  Eligible: n_sink <= m <= n - 2 - n_recent (inclusive)."""
    return n_sink, n - 2 - n_recent


def edge_scores(alpha_bar: np.ndarray, n_sink: int, n_recent: int, sigma_dtype=F64):
    n = alpha_bar.shape[0]
    lo, hi = eligible_edges(n, n_sink, n_recent)
    if hi < lo:
        return lo, hi, np.zeros(0, dtype=sigma_dtype)
    a = np.asarray(alpha_bar).astype(sigma_dtype)
    return lo, hi, a[lo:hi + 1] + a[lo + 1:hi + 2]          # O5, added in sigma_dtype


def select(alpha_bar: np.ndarray, budget: int, n_sink: int = 32, n_recent: int = 0,
           sigma_dtype=F64) -> Tuple[np.ndarray, np.ndarray]:
    """mask[n] (mask[m] = 1: token m+1 joins token m's slot) and slot[n].

    `sigma_dtype` is the precision in which the edge score is added and compared:
    fp64 for the oracle proper; float32 when a kernel that takes fp32 alpha_bar and
    decides in fp32 is checked in isolation (both sides then decide in the same precision).
    """
    n = alpha_bar.shape[0]
    mask = np.zeros(n, dtype=np.uint8)
    r = n - budget
    if r > 0:
        lo, hi, sigma = edge_scores(alpha_bar, n_sink, n_recent, sigma_dtype)
        if r > sigma.shape[0]:
            raise ValueError("budget below n_sink + 1 + n_recent: not enough eligible edges")
        order = np.argsort(sigma, kind="stable")            # ties -> smaller m      (O6)
        mask[lo + order[:r]] = 1
    starts = np.ones(n, dtype=np.int64)
    starts[1:] = 1 - mask[:-1].astype(np.int64)             # t starts a slot iff mask[t-1] = 0
    slot = (np.cumsum(starts) - 1).astype(np.int32)         # O7
    return mask, slot


def boundary_gap(alpha_bar: np.ndarray, budget: int, n_sink: int = 32, n_recent: int = 0) -> float:
    """Relative gap (sigma_(r+1) - sigma_(r)) / sigma_(r+1) at the budget boundary (inf if none)."""
    n = alpha_bar.shape[0]
    r = n - budget
    _, _, sigma = edge_scores(alpha_bar, n_sink, n_recent)
    if r <= 0 or r >= sigma.shape[0]:
        return float("inf")
    s = np.sort(sigma)
    return float((s[r] - s[r - 1]) / s[r])


# --------------------------------------------------------------------------- O8-O9
def token_and_edge_norms(alpha_bar: np.ndarray, V: np.ndarray, o_bar: np.ndarray,
                         counts: Optional[np.ndarray] = None):
    """A_t = ||c_tt||_2 for every token and C_t = ||c_{t,t+1}||_2 for every edge (Eqs. c11_def-c12_def)."""
    a = np.asarray(alpha_bar, dtype=F64)
    resid = slot_values(V, counts) - np.asarray(o_bar, dtype=F64)[None, :]        # r_t = v_t - o
    A = np.linalg.norm((a * (1.0 - 2.0 * a))[:, None] * resid, axis=1)
    C = np.linalg.norm(-(a[:-1] * a[1:])[:, None] * (resid[:-1] + resid[1:]), axis=1)
    return A, C


def per_query_norms(Q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: Optional[float] = None,
                    causal_window: int = 0, counts: Optional[np.ndarray] = None):
    """A_t and C_t with every query row kept apart: row q has its own attention alpha^{(q)} (Eq. attn_def_vec)
    and its own output o^{(q)}; the vectors of Eqs. c11_def-c12_def are formed per row and their norms are
    averaged over the rows.  Q [R, D] (or [G, W, D]), K, V [n, D]; returns A [n], C [n - 1].
    With `counts` the rows of K and V are slots of an already merged cache (streaming regime): every query row
    sees a slot as one token with logit e + ln c and value V / c, as everywhere else in this module."""
    alpha = attention_rows(Q, K, scale, counts, causal_window)
    values = slot_values(V, counts)
    R, n = alpha.shape
    A = np.zeros(n, dtype=F64)
    C = np.zeros(max(n - 1, 0), dtype=F64)
    for q in range(R):
        o_q = alpha[q] @ values                             # this row's attention output
        A_q, C_q = token_and_edge_norms(alpha[q], V, o_q, counts)
        A += A_q
        C += C_q
    return A / R, C / R


@dataclass
class MergeResult:
    K_out: np.ndarray        # [n_out, D] fp64
    V_out: np.ndarray        # [n_out, D] fp64
    counts: np.ndarray       # [n_out] int32: tokens the slot stands for
    n_rows: np.ndarray       # [n_out] int32: input rows merged into the slot
    U: np.ndarray            # [n_out] denominator of the Key weights (A_t for singletons)
    A_sum: np.ndarray        # [n_out] sum of A_t over the slot
    fallback: np.ndarray     # [n_out] bool: arithmetic-mean fallback taken


RULES = ("hessian", "diagonal", "mean")


def merge_compact(K: np.ndarray, V: np.ndarray, alpha_bar: np.ndarray, o_bar: np.ndarray,
                  mask: np.ndarray, slot: np.ndarray, counts_in: Optional[np.ndarray] = None,
                  rule: str = "hessian", norms=None) -> MergeResult:
    """`norms = (A, C)` replaces the norms computed from alpha_bar and o_bar (per-query aggregation);
    alpha_bar and o_bar are then not used.  With `counts_in` the rows are slots of a merged cache: cardinalities
    add up, Values stay sums, the fallback is the mean over the tokens the rows stand for."""
    assert rule in RULES
    K = np.asarray(K, dtype=F64)
    V = np.asarray(V, dtype=F64)
    n, D = K.shape
    c_in = np.ones(n, dtype=np.int64) if counts_in is None else np.asarray(counts_in, dtype=np.int64)
    if norms is None:
        A, C = token_and_edge_norms(alpha_bar, V, o_bar, counts_in)
    else:                                                   # (cardinalities then only enter the sums below)
        A, C = (np.asarray(x, dtype=F64) for x in norms)
    n_out = int(slot[-1]) + 1 if n else 0
    K_out = np.zeros((n_out, D), dtype=F64)
    V_out = np.zeros((n_out, V.shape[1]), dtype=F64)
    counts = np.zeros(n_out, dtype=np.int32)
    n_rows = np.zeros(n_out, dtype=np.int32)
    U_all = np.zeros(n_out, dtype=F64)
    A_sum = np.zeros(n_out, dtype=F64)
    fallback = np.zeros(n_out, dtype=bool)
    t = 0
    for S in range(n_out):
        t0 = t
        while t < n - 1 and mask[t]:
            t += 1
        t1 = t                                              # slot S = tokens t0..t1 inclusive
        t += 1
        assert slot[t0] == S and slot[t1] == S
        counts[S] = c_in[t0:t1 + 1].sum()                   # cardinalities add up
        n_rows[S] = t1 - t0 + 1
        V_out[S] = V[t0:t1 + 1].sum(axis=0)
        A_sum[S] = A[t0:t1 + 1].sum()
        if t1 == t0:
            K_out[S] = K[t0]
            U_all[S] = A[t0]
            continue
        if rule == "mean":
            u = c_in[t0:t1 + 1].astype(F64)                 # every token the rows stand for counts once
        else:
            u = A[t0:t1 + 1].copy()
            if rule == "hessian":
                u[:-1] -= C[t0:t1]                          # coupling with the next token
                u[1:] -= C[t0:t1]                           # coupling with the previous token
        U = u.sum()
        U_all[S] = U
        if np.isfinite(U) and U > 0.0:
            K_out[S] = (u[:, None] * K[t0:t1 + 1]).sum(axis=0) / U
        else:
            fallback[S] = True                              # mean over the tokens the rows stand for
            K_out[S] = (c_in[t0:t1 + 1, None] * K[t0:t1 + 1]).sum(axis=0) / c_in[t0:t1 + 1].sum()
    assert t == n
    return MergeResult(K_out, V_out, counts, n_rows, U_all, A_sum, fallback)


def conditioning(res: MergeResult) -> float:
    """min over merged slots of U / sum_t A_t (1 for an input without merged slots)."""
    multi = res.n_rows > 1
    if not multi.any():
        return 1.0
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = res.U[multi] / res.A_sum[multi]
    ratio = np.where(np.isfinite(ratio), ratio, -np.inf)
    return float(ratio.min())


# --------------------------------------------------------------------------- whole step
@dataclass
class StepResult:
    alpha_bar: np.ndarray
    o_bar: np.ndarray
    mask: np.ndarray
    slot: np.ndarray
    merged: MergeResult


def step(Q: np.ndarray, K: np.ndarray, V: np.ndarray, budget: int, n_sink: int = 32,
         n_recent: int = 0, scale: Optional[float] = None, counts: Optional[np.ndarray] = None,
         rule: str = "hessian", per_query: bool = False, causal_window: int = 0) -> StepResult:
    alpha_bar, o_bar = score(Q, K, V, scale, counts, causal_window)
    mask, slot = select(alpha_bar, budget, n_sink, n_recent)
    norms = per_query_norms(Q, K, V, scale, causal_window, counts) if per_query else None
    merged = merge_compact(K, V, alpha_bar, o_bar, mask, slot, counts, rule, norms)
    return StepResult(alpha_bar, o_bar, mask, slot, merged)


# --------------------------------------------------------------------------- consumer of the merged cache
def merged_attention(q: np.ndarray, K_out: np.ndarray, V_out: np.ndarray, counts: np.ndarray,
                     scale: Optional[float] = None) -> np.ndarray:
    """Attention of one query over a merged cache whose Values are sums.

    A slot (k', V', c) stands for c tokens that all carry the Key k' (the "(k, k)"
    replacement of Sec. 3.1) and whose Values add up to V':
    o = sum_S exp(e_S) V'_S / sum_S c_S exp(e_S).
    """
    q = np.asarray(q, dtype=F64)
    if scale is None:
        scale = 1.0 / np.sqrt(q.shape[-1])
    e = scale * (np.asarray(K_out, dtype=F64) @ q)
    w = np.exp(e - e.max())
    return (w @ np.asarray(V_out, dtype=F64)) / (w @ np.asarray(counts, dtype=F64))


def decode_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, counts: Optional[np.ndarray] = None,
                     scale: Optional[float] = None) -> np.ndarray:
    """merged_attention for every row of Q [..., D]: out [R, D].  counts = None: a plain cache (c = 1)."""
    K = np.asarray(K, dtype=F64)
    Q = np.asarray(Q, dtype=F64).reshape(-1, K.shape[1])
    c = np.ones(K.shape[0], dtype=F64) if counts is None else np.asarray(counts, dtype=F64)
    return np.stack([merged_attention(q, K, V, c, scale) for q in Q])
