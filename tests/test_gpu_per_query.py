"""GPU-vs-oracle parity of the per-query aggregation (kvs_sensitivity, kvs_merge_compact_norms,
kvs_step_per_query), called through the C ABI.

Bars: selected edges, slot maps and counts bit-exact; merged K / V within 1e-2 (bf16 I/O; 1e-5 for
kvs_merge_compact_norms with fp32 I/O) relative L2 error per output row; A_t and C_t within TOL_NORMS
relative.  TOL_NORMS: the kernels form alpha in fp32 (as the score sweeps, 3e-5), the attention outputs
o^{(q)} and the products v.o from bf16 operand pairs hi + lo (2^-17 relative per term), and the squared
distances by the expansion ||v||^2 - 2 v.o + ||o||^2 in fp32 where that loses less than four bits to
cancellation, else from differences (test_sensitivity_concentrated_rows plants the cases that need it).
Two absolute terms join the bar where the relative one says nothing: see TOL_ALPHA_ROW and TOL_WEIGHT.
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
# weight is all that is left of A_t, whatever the arithmetic.  Such a row's share is therefore held to its size
# without that factor, alpha ||v - o||, times this bound on alpha's relative error.  The weights are exp2 of fp32
# logits, so their relative error is an absolute error of the logit, a few units in its last place: the bound holds
# for base-2 logits up to 32 in size (the generated workloads reach 20 to 36) and grows in proportion beyond
# (alpha_row_tol below; test_sensitivity_concentrated_rows reaches 150).
TOL_ALPHA_ROW = 4e-6
# The bf16 kernels hand o^{(q)} on as a bf16 pair hi + lo, relative 2^-18 per component: an absolute error of up to
# 2^-18 ||o^{(q)}|| in ||v_t - o|| (twice that in ||v_t + v_{t+1} - 2 o||), which the bars admit per query row.  It
# shows where o comes close to v_t (a row that puts nearly all its weight on one token, or Values that repeat) and
# the norm itself is small.  (The weights' own rounding does not show: o is formed as a convex combination with the
# rounded weights.)
TOL_WEIGHT = 2.0 ** -18


def alpha_row_tol(Q, K, counts, head_dim):
    """TOL_ALPHA_ROW, scaled up where the base-2 logits exceed 32 in size."""
    logit2 = (Q.reshape(-1, head_dim).astype(np.float64) @ K.astype(np.float64).T) / np.sqrt(head_dim) / np.log(2.0)
    if counts is not None:
        logit2 = logit2 + np.log2(counts.astype(np.float64))[None, :]
    return TOL_ALPHA_ROW * max(1.0, float(np.abs(logit2).max()) / 32.0)


def per_query_buffers(batch):
    import torch
    p = batch.problem
    G = batch.GUARD
    a_tok = torch.full((p.rows_in + G,), -7.0, dtype=torch.float32, device="cuda")
    c_edge = torch.full((p.rows_in + G,), -7.0, dtype=torch.float32, device="cuda")
    ws = torch.full((batch.kvs.kvs_per_query_workspace_size(p) + 256,), 0xFF, dtype=torch.uint8, device="cuda")
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
    check_sensitivity(w, units, lens, D, G, W, dtype, causal)


def check_sensitivity(w, units, lens, D, G, W, dtype, causal):
    """kvs_sensitivity(_counts) on `units` against the oracle."""
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
        onorm = np.linalg.norm(rows @ V64, axis=1)    # ||o^{(q)}|| of every row
        conc = (rows * onorm[:, None]).mean(axis=0)   # mean over the rows of alpha_t ||o||
        den = A_ref + (alpha_row_tol(u.Q, u.K, u.counts, D) / TOL_NORMS) * size + (TOL_WEIGHT / TOL_NORMS) * conc
        concC = 2.0 * (rows[:, :-1] * rows[:, 1:] * onorm[:, None]).mean(axis=0)
        if n == 1:
            # a unit's only token has alpha = 1 and o = v: A is exactly zero, and what the kernel finds is the
            # rounding of o against v
            assert gA[0] <= 1e-5 * np.linalg.norm(V64[0])
            den = np.ones(1)
        eA = np.max(np.abs(gA - A_ref) / den)
        eC = np.max(np.abs(gC - C_ref) / (C_ref + (TOL_WEIGHT / TOL_NORMS) * concC)) if n > 1 else 0.0
        assert eA < TOL_NORMS, (i, "A", eA)
        assert eC < TOL_NORMS, (i, "C", eC)
        assert C[r0 + n - 1] == 0.0                  # a unit's last row has no edge
    for i in range(len(units) - 1):                  # rows between units are never touched
        gap0 = p.in_rows[i] + lens[i]
        assert (A[gap0:gap0 + 3] == -7.0).all() and (C[gap0:gap0 + 3] == -7.0).all()


@pytest.mark.parametrize("dtype,G,W", [("bf16", 4, 1), ("f32", 1, 2)])
def test_sensitivity_at_the_maximum_length(dtype, G, W):
    """One unit of KVS_MAX_LEN = 2^22 rows, head dim 128 (with fp32 the longest rows there are: the last one ends one
    byte short of 2^31), few query rows so that the oracle stays quick; every A_t, C_t and alpha_bar is compared."""
    from workloads import gaussian_unit
    from workloads.generator import UnitInputs
    n, D = 1 << 22, 128
    Q, K, V = gaussian_unit(2, n, D, G, W, dtype, k_scale=1.0)
    u = UnitInputs(layer=0, seq=0, head=0, attempt=0, n=n, budget=n, rho=0.0, Q=Q, K=K, V=V)
    w = variant("llama8b_8k", dtype=dtype, head_dim=D, group=G, window=W, n_seq=1, n_kv_heads=1)
    check_sensitivity(w, [u], [n], D, G, W, dtype, False)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("counts", [False, True])
def test_sensitivity_with_values_that_repeat(counts, dtype):
    """Every token carries the same Value (per token it stands for), so every o^{(q)} equals it and A_t = C_t = 0: all
    that the kernels may leave is the rounding of o.  In the bf16 kernels every token takes the path that forms its
    norms from differences (5000 tokens: two of that kernel's spans, the second ragged).  A second unit has two
    Values that alternate in blocks of 40 tokens: norms of full size beside norms that cancel, in the same tiles."""
    D, G, W, n = 128, 3, 16, 5000
    base = "stream2560" if counts else "llama8b_8k"
    w = variant(base, dtype=dtype, head_dim=D, group=G, window=W, n_seq=2, n_kv_heads=1)
    if counts:
        w = w.scaled(fresh_tail=W, n_sink=2)
    units = [generate_unit(w, 0, s, 0, n=m) for s, m in enumerate([n, 700])]
    for u, period in zip(units, (0, 40)):
        c = np.ones(u.n) if u.counts is None else u.counts.astype(np.float64)
        two = u.V[:2].astype(np.float64) / c[:2, None]
        which = (np.arange(u.n) // period) % 2 if period else np.zeros(u.n, dtype=np.int64)
        # (cardinalities are small integers: for a bf16 vector v, c v is exact in fp32 and rounds once to bf16; the
        # oracle sees the rounded rows, so the per-token Values differ in the last bit and the norms are not exactly 0)
        u.V = _bf16(two[which] * c[:, None]) if dtype == "bf16" else (two[which] * c[:, None]).astype(np.float32)
    check_sensitivity(w, units, [n, 700], D, G, W, dtype, False)


def _bf16(x):
    from workloads import bf16_bits_to_f32, f32_to_bf16_bits
    return bf16_bits_to_f32(f32_to_bf16_bits(np.asarray(x, dtype=np.float32)))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("counts", [False, True])
@pytest.mark.parametrize("causal", [False, True])
def test_sensitivity_concentrated_rows(causal, counts, dtype):
    """Query rows that put (nearly) all their weight on one token, or share it between two adjacent ones.

    There o^{(q)} comes close to v_t, resp. to the mean of v_t and v_{t+1}, and ||v_t - o||, resp.
    ||v_t + v_{t+1} - 2 o||, is what is left when terms of size ||v|| cancel: the kernel has to form these norms
    from differences (the bf16 kernels do so for the tokens they find affected, the fp32 kernels always).  Tokens are planted inside a tile, at a tile's last row (31 rows are put out per tile) and in
    the unit's last rows; the rows of the second pass (160 query rows) get some as well.
    """
    D, G, W, n = 128, 5, 32, 1200
    base = "stream2560" if counts else "llama8b_8k"
    w = variant(base, dtype=dtype, head_dim=D, group=G, window=W, n_seq=1, n_kv_heads=1)
    if counts:
        w = w.scaled(fresh_tail=W, n_sink=2)
    u = generate_unit(w, 0, 0, 0, n=n)
    # two adjacent tokens with the same Key share a row's weight: alpha = 1/2 each, o = their mean
    Kd = u.K.copy()
    for t in (200, 216, 929):
        Kd[t + 1] = Kd[t]
    u.K = Kd
    K, Q = u.K.astype(np.float64), u.Q.reshape(G * W, D).astype(np.float64).copy()
    scale = 1.0 / np.sqrt(D)

    def aim(row, t, gap, pair=False):
        """Query row `row` := the multiple of (K^T K / n)^{-1} k_t whose logit on token t (and on t + 1, for a pair of
        equal Keys) lies `gap` above that of every other token (natural-log units)."""
        u_ = np.linalg.solve(K.T @ K / n + 1e-3 * np.eye(D), K[t])
        logit = K @ u_ * scale
        others = np.delete(logit, [t, t + 1] if pair else [t])
        assert logit[t] > others.max()
        Q[row] = _bf16(gap / (logit[t] - others.max()) * u_)

    aim(3, 500, 16.0)            # inside a tile: alpha within 1e-4 of 1
    aim(40, 30, 14.0)            # the last row a tile puts out
    aim(77, 31, 18.0)            # the first row of the next tile
    aim(130, 640, 9.0)           # a row of the second pass; alpha some 1e-2 below 1
    aim(159, n - 1, 16.0)        # the unit's last token (no edge behind it)
    aim(100, n - 2, 7.0)
    aim(8, 200, 16.0, pair=True)
    aim(140, 216, 16.0, pair=True)     # second pass
    aim(64, 929, 15.0, pair=True)      # the pair straddles two tiles (929 = 31 * 29 + 30)
    u.Q = Q.reshape(G, W, D).astype(np.float32)
    check_sensitivity(w, [u], [n], D, G, W, dtype, causal)


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


def test_streaming_loop_of_per_query_steps():
    """The loop of test_streaming_loop_of_steps with the per-query aggregation in every round."""
    from test_gpu_parity import streaming_loop
    streaming_loop(check_step_per_query, per_query=True)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_step_per_query_more_units_than_the_kernel_arguments_hold(dtype):
    """100 short units in one call: one launch group, its unit descriptors in the workspace."""
    w = WORKLOADS["llama8b_8k"].scaled(dtype=dtype, group=2, window=8, length=("fixed", 500), budget=("fixed", 150))
    check_step_per_query(w, [accepted_unit_per_query(w, h // 8, 0, h % 8, n=500 - 3 * (h % 11)) for h in range(100)])


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
