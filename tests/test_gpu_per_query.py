"""GPU-vs-oracle parity of the per-query aggregation (kvs_sensitivity, kvs_merge_compact_norms,
kvs_step_per_query), called through the C ABI.

Bars: selected edges, slot maps and counts bit-exact; merged K / V within 1e-2 (bf16 I/O; 1e-5 for
kvs_merge_compact_norms with fp32 I/O) relative L2 error per output row; A_t and C_t within TOL_NORMS
relative.  TOL_NORMS: the kernels form alpha in fp32 (as the score sweeps, 3e-5), the attention outputs
o^{(q)} and the products v.o from bf16 operand pairs hi + lo (2^-17 relative per term), and the squared
distances by the expansion ||v||^2 - 2 v.o + ||o||^2 in fp32, whose cancellation is mild because
||o|| is well below ||v|| on every workload here.
"""

import numpy as np
import pytest

from oracle import kvs_oracle as O
from workloads import WORKLOADS, generate_unit

from helpers import DeviceBatch, accepted_unit_per_query, from_device
from test_gpu_parity import TOL_ALPHA, compare_outputs, merge_case, torch_sync, variant

pytestmark = pytest.mark.gpu

TOL_NORMS = 5e-5     # measured: at most 1.1e-5 over the cases below
# A_t carries the factor |1 - 2 alpha|, which vanishes at alpha = 1/2: there the rounding of a row's own attention
# weight (fp32 softmax, relative 1e-6) is all that is left of A_t, whatever the arithmetic.  Such a row's share is
# therefore held to its size without that factor, alpha ||v - o||, times this bound on alpha's relative error.
TOL_ALPHA_ROW = 4e-6


def per_query_buffers(batch):
    import torch
    p = batch.problem
    G = batch.GUARD
    a_tok = torch.full((p.rows_in + G,), -7.0, dtype=torch.float32, device="cuda")
    c_edge = torch.full((p.rows_in + G,), -7.0, dtype=torch.float32, device="cuda")
    ws = torch.empty(batch.kvs.kvs_per_query_workspace_size(p) + 256, dtype=torch.uint8, device="cuda")
    return a_tok, c_edge, ws


SENS_CASES = [
    # base, D, G, W, lengths
    ("llama8b_8k", 128, 4, 32, [2500]),              # one pass of 128 rows, ten chunks, ragged tail
    ("llama8b_8k", 128, 1, 20, [700, 33]),           # fewer rows than one wavefront's block; a 33-row unit
    ("llama8b_8k", 64, 2, 16, [900, 32]),            # head dim 64; a unit of exactly one tile
    ("llama8b_8k", 128, 5, 20, [1500]),              # 100 rows: the last wavefront's block is ragged
    ("llama8b_8k", 128, 5, 32, [1111, 300]),         # 160 rows: two passes
    ("stress128k", 128, 8, 40, [1200]),              # 320 rows: three passes
    ("ragged16", 128, 4, 32, [300, 5000, 9000]),     # chunks of different units in one launch
    ("llama8b_8k", 128, 1, 1, [257]),                # a single query row
]


# fp32 caches (vector-ALU kernels: any unit length, any number of rows)
SENS_CASES_F32 = [
    ("tiny", 64, 1, 8, [1024]),                      # the small configuration as it is
    ("tiny", 64, 2, 5, [300, 31, 2, 1]),             # units shorter than a tile, down to one token; ten rows
    ("tiny", 128, 4, 3, [700, 33]),                  # head dim 128; twelve rows: a ragged block of query rows
    ("llama8b_8k", 128, 4, 32, [1300, 600]),         # 128 rows, several chunks
]


# rows with input cardinalities (streaming regime): the recipe of the stream2560 workload at other shapes
SENS_CASES_COUNTS = [
    ("stream2560", 128, 4, 32, [2560, 700], "bf16"),   # the streaming configuration's own shape; a ragged second unit
    ("stream2560", 64, 2, 16, [900, 32], "bf16"),      # head dim 64; a unit of exactly one tile
    ("stream2560", 128, 5, 32, [1111], "bf16"),        # 160 rows: two passes
    ("stream2560", 64, 2, 5, [300, 31, 3], "f32"),     # fp32: units shorter than a tile
    ("stream2560", 128, 4, 8, [1300], "f32"),
]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("base,D,G,W,lens,dtype",
                         [c + ("bf16",) for c in SENS_CASES] + [c + ("f32",) for c in SENS_CASES_F32] +
                         SENS_CASES_COUNTS)
def test_sensitivity_matches_oracle(base, D, G, W, lens, dtype, causal):
    if causal:
        lens = [n for n in lens if n >= W]           # the window's own rows are part of the cache
    w = variant(base, dtype=dtype, head_dim=D, group=G, window=W, n_seq=len(lens), n_kv_heads=1)
    if w.mean_count > 0:
        w = w.scaled(fresh_tail=max(W, 8), n_sink=2)  # short units too have rows that stand for several tokens
    units = [generate_unit(w, 0, s, 0, n=n) for s, n in enumerate(lens)]
    batch = DeviceBatch(units, group=G, window=W, head_dim=D, dtype=dtype, n_sink=w.n_sink, gap_rows=3,
                        causal=causal)
    cw = W if causal else 0
    a_tok, c_edge, ws = per_query_buffers(batch)
    with_counts = units[0].counts is not None
    if with_counts:
        batch.kvs.kvs_sensitivity_counts(batch.problem, batch.Q, batch.K, batch.V, batch.counts_in, batch.alpha_bar,
                                         a_tok, c_edge, ws, stream=batch.stream())
    else:
        batch.kvs.kvs_sensitivity(batch.problem, batch.Q, batch.K, batch.V, batch.alpha_bar, a_tok, c_edge, ws,
                                  stream=batch.stream())
    torch_sync()
    batch.check_guards()
    p = batch.problem
    assert (a_tok[p.rows_in:] == -7.0).all() and (c_edge[p.rows_in:] == -7.0).all()
    alpha, A, C = from_device(batch.alpha_bar), from_device(a_tok), from_device(c_edge)
    for i, u in enumerate(units):
        n = lens[i]
        r0 = p.in_rows[i]
        ra, _ = O.score(u.Q, u.K, u.V, counts=u.counts, causal_window=cw)
        A_ref, C_ref = O.per_query_norms(u.Q, u.K, u.V, causal_window=cw, counts=u.counts)
        assert np.max(np.abs(alpha[r0:r0 + n] - ra) / ra) < TOL_ALPHA
        gA, gC = A[r0:r0 + n], C[r0:r0 + n - 1]
        assert np.isfinite(gA).all() and np.isfinite(gC).all()
        rows = O.attention_rows(u.Q, u.K, counts=u.counts, causal_window=cw)
        V64 = O.slot_values(u.V, u.counts)
        size = np.zeros(n)                           # mean over the rows of alpha ||v_t - o|| (no |1 - 2 alpha|)
        for a_q in rows:
            size += a_q * np.linalg.norm(V64 - a_q @ V64, axis=1)
        size /= rows.shape[0]
        den = A_ref + (TOL_ALPHA_ROW / TOL_NORMS) * size
        if n == 1:
            # a unit's only token has alpha = 1 and o = v: A is exactly zero, and what the kernel finds is the
            # rounding of o against v
            assert gA[0] <= 1e-5 * np.linalg.norm(V64[0])
            den = np.ones(1)
        eA = np.max(np.abs(gA - A_ref) / den)
        eC = np.max(np.abs(gC - C_ref) / C_ref) if n > 1 else 0.0
        assert eA < TOL_NORMS, (i, "A", eA)
        assert eC < TOL_NORMS, (i, "C", eC)
        assert C[r0 + n - 1] == 0.0                  # a unit's last row has no edge
    for i in range(len(units) - 1):                  # rows between units are never touched
        gap0 = p.in_rows[i] + lens[i]
        assert (A[gap0:gap0 + 3] == -7.0).all() and (C[gap0:gap0 + 3] == -7.0).all()


@pytest.mark.parametrize("rule", ["hessian", "diagonal"])
@pytest.mark.parametrize("base,dtype,D,lens,budgets", [
    ("tiny", "f32", 64, [1024, 300], [256, 100]),
    ("llama8b_8k", "bf16", 128, [3000, 777], [700, 300]),
    ("stream2560", "bf16", 128, [2560, 777], [2048, 300]),      # rows with input cardinalities
    ("stream2560", "f32", 64, [900], [400]),
])
def test_merge_compact_norms_matches_oracle(base, dtype, D, lens, budgets, rule):
    """The merge pass with A_t and C_t handed in (here the oracle's, rounded to fp32)."""
    import torch
    w, units = merge_case(base, dtype, D, lens, budgets)
    batch = DeviceBatch(units, group=w.group, window=w.window, head_dim=D, dtype=dtype, n_sink=w.n_sink,
                        key_rule=rule)
    p = batch.problem
    refs = []
    A_all = np.zeros(p.rows_in, dtype=np.float32)
    C_all = np.zeros(p.rows_in, dtype=np.float32)
    mask_all = np.zeros(p.rows_in, dtype=np.uint8)
    slot_all = np.zeros(p.rows_in, dtype=np.int32)
    for i, u in enumerate(units):
        n = u.K.shape[0]
        a, o = O.score(u.Q, u.K, u.V, counts=u.counts)
        mask, slot = O.select(a.astype(np.float32), u.budget, w.n_sink, 0, sigma_dtype=np.float32)
        A, C = O.per_query_norms(u.Q, u.K, u.V, counts=u.counts)
        A32, C32 = A.astype(np.float32), C.astype(np.float32)
        refs.append(O.merge_compact(u.K, u.V, a, o, mask, slot, counts_in=u.counts, rule=rule,
                                    norms=(A32.astype(np.float64), C32.astype(np.float64))))
        r0 = p.in_rows[i]
        A_all[r0:r0 + n] = A32
        C_all[r0:r0 + n - 1] = C32
        mask_all[r0:r0 + n] = mask
        slot_all[r0:r0 + n] = slot
    dev = [torch.from_numpy(x).cuda() for x in (A_all, C_all, mask_all, slot_all)]
    if units[0].counts is not None:
        batch.kvs.kvs_merge_compact_norms_counts(p, batch.K, batch.V, batch.counts_in, *dev, batch.K_out, batch.V_out,
                                                 batch.counts, stream=batch.stream())
    else:
        batch.kvs.kvs_merge_compact_norms(p, batch.K, batch.V, *dev, batch.K_out, batch.V_out, batch.counts,
                                          stream=batch.stream())
    torch_sync()
    batch.check_guards()
    compare_outputs(batch, refs, dtype)


def check_step_per_query(w, accepted, causal=False):
    batch = DeviceBatch([a.inputs for a in accepted], group=w.group, window=w.window, head_dim=w.head_dim,
                        dtype=w.dtype, n_sink=w.n_sink, n_recent=w.n_recent, causal=causal)
    _, _, ws = per_query_buffers(batch)
    if accepted[0].inputs.counts is not None:
        batch.kvs.kvs_step_per_query_counts(batch.problem, batch.Q, batch.K, batch.V, batch.counts_in, batch.K_out,
                                            batch.V_out, batch.counts, ws, slot_of_token_out=batch.slot,
                                            edge_mask_out=batch.mask, stream=batch.stream())
    else:
        batch.kvs.kvs_step_per_query(batch.problem, batch.Q, batch.K, batch.V, batch.K_out, batch.V_out,
                                     batch.counts, ws, slot_of_token_out=batch.slot, edge_mask_out=batch.mask,
                                     stream=batch.stream())
    torch_sync()
    batch.check_guards()
    p = batch.problem
    mask, slot = batch.mask.cpu().numpy(), batch.slot.cpu().numpy()
    for i, a in enumerate(accepted):
        r0, n = p.in_rows[i], a.inputs.n
        assert (mask[r0:r0 + n] == a.ref.mask).all(), f"unit {i}: selected edges differ (gap {a.gap:.2e})"
        assert (slot[r0:r0 + n] == a.ref.slot).all(), f"unit {i}: slot map differs"
    compare_outputs(batch, [a.ref.merged for a in accepted], w.dtype)
    return batch


def test_step_per_query_8k_config():
    w = WORKLOADS["llama8b_8k"]
    check_step_per_query(w, [accepted_unit_per_query(w, 0, 0, h) for h in range(3)])


def test_step_per_query_fp32_config():
    """The small fp32 configuration through the vector-ALU kernels, and a variant with more query rows."""
    w = WORKLOADS["tiny"]
    check_step_per_query(w, [accepted_unit_per_query(w, 0, 0, 0)])
    w = WORKLOADS["tiny"].scaled(group=3, window=6, length=("fixed", 700), budget=("fixed", 200))
    check_step_per_query(w, [accepted_unit_per_query(w, 0, 0, 0)])
    check_step_per_query(w, [accepted_unit_per_query(w, 0, 0, 0, causal=True)], causal=True)


def test_step_per_query_streaming_regime():
    """Caches of 2048 + 512 slots with input cardinalities, every query row kept apart: bf16 as configured, and the
    same recipe in fp32 at a smaller size; cardinalities of the merged slots bit-exact."""
    w = WORKLOADS["stream2560"]
    check_step_per_query(w, [accepted_unit_per_query(w, 0, 0, h) for h in range(2)])
    w = WORKLOADS["stream2560"].scaled(dtype="f32", group=2, window=8, length=("fixed", 900), budget=("fixed", 600),
                                       fresh_tail=64)
    check_step_per_query(w, [accepted_unit_per_query(w, 0, 0, 0)])


def test_step_per_query_with_causal_window():
    w = WORKLOADS["llama8b_8k"]
    check_step_per_query(w, [accepted_unit_per_query(w, 0, 0, h, causal=True) for h in range(2)], causal=True)


def test_step_per_query_32k_two_heads_full_length():
    """The headline shape (32768 -> 4096 tokens, 128 query rows), two of the layer's KV heads."""
    import torch
    w = WORKLOADS["llama8b_32k"]
    acc = [accepted_unit_per_query(w, 5, 0, h) for h in range(2)]
    b1 = check_step_per_query(w, acc)
    b2 = check_step_per_query(w, acc)
    assert torch.equal(b1.K_out.view(torch.int16), b2.K_out.view(torch.int16))     # run-to-run bitwise


def test_step_per_query_with_one_row_is_the_plain_step():
    """R = 1: the aggregation over query rows is the identity, the step equals kvs_step up to rounding."""
    w = WORKLOADS["llama8b_8k"].scaled(group=1, window=1, length=("fixed", 3000), budget=("fixed", 1000))
    acc = [accepted_unit_per_query(w, 0, 0, 0)]
    batch = check_step_per_query(w, acc)
    plain = DeviceBatch([a.inputs for a in acc], group=1, window=1, head_dim=w.head_dim, dtype=w.dtype,
                        n_sink=w.n_sink)
    plain.kvs.kvs_step(plain.problem, plain.Q, plain.K, plain.V, plain.K_out, plain.V_out, plain.counts, plain.ws,
                       stream=plain.stream())
    torch_sync()
    import torch
    assert torch.equal(batch.counts, plain.counts)
    assert torch.equal(batch.V_out.view(torch.int16), plain.V_out.view(torch.int16))
    n_out = plain.problem.rows_out
    d = (batch.K_out[:n_out].float() - plain.K_out[:n_out].float()).norm(dim=1) / plain.K_out[:n_out].float().norm(dim=1)
    assert float(d.max()) < 1e-2
