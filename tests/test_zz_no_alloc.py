"""kvs_step_static (the step for callers that cannot allocate: its workspace is a device array inside the library)
against kvs_step_counts with a caller-owned workspace, through the C ABI: same kernels, same launch geometry, so
every output must agree bit for bit; and against the oracle, to the bar of the other step tests.  Two calls in a
row, the second on a smaller problem (the array keeps the first call's contents)."""

import numpy as np
import pytest

from helpers import DeviceBatch, accepted_unit, from_device, rel_err_rows
from workloads import WORKLOADS

pytestmark = pytest.mark.gpu


def run_both(units, w):
    import torch
    import paper_2603_00907_amd as kvs
    a = DeviceBatch(units, group=w.group, window=w.window, head_dim=w.head_dim, dtype=w.dtype, n_sink=w.n_sink,
                    n_recent=w.n_recent)
    b = DeviceBatch(units, group=w.group, window=w.window, head_dim=w.head_dim, dtype=w.dtype, n_sink=w.n_sink,
                    n_recent=w.n_recent)
    assert kvs.kvs_workspace_size(a.problem) <= kvs.STATIC_SCRATCH_BYTES
    kvs.kvs_step_counts(a.problem, a.Q, a.K, a.V, a.counts_in, a.K_out, a.V_out, a.counts, a.ws,
                        slot_of_token_out=a.slot, edge_mask_out=a.mask, stream=a.stream())
    kvs.kvs_step_static(b.problem, b.Q, b.K, b.V, b.counts_in, b.K_out, b.V_out, b.counts,
                        slot_of_token_out=b.slot, edge_mask_out=b.mask, stream=b.stream())
    torch.cuda.synchronize()
    b.check_guards()
    for name in ("K_out", "V_out", "counts", "slot", "mask"):
        x, y = getattr(a, name), getattr(b, name)
        assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), name
    return b


def check_against_oracle(batch, accepted, tol):
    p = batch.problem
    for i, acc in enumerate(accepted):
        n, r0, o0, no = p.lens[i], p.in_rows[i], p.out_rows[i], p.n_out[i]
        assert (batch.slot[r0:r0 + n].cpu().numpy() == acc.ref.slot).all()
        assert (batch.mask[r0:r0 + n].cpu().numpy() == acc.ref.mask).all()
        assert (batch.counts[o0:o0 + no].cpu().numpy() == acc.ref.merged.counts).all()
        assert rel_err_rows(from_device(batch.K_out[o0:o0 + no]), acc.ref.merged.K_out) <= tol
        assert rel_err_rows(from_device(batch.V_out[o0:o0 + no]), acc.ref.merged.V_out) <= tol


def test_static_entry_matches_the_step_on_two_calls_in_a_row():
    # first call: two heads of the 8K bf16 configuration; second call: the tiny fp32 configuration
    w1 = WORKLOADS["llama8b_8k"]
    acc1 = [accepted_unit(w1, 0, 0, h) for h in range(2)]
    b1 = run_both([a.inputs for a in acc1], w1)
    check_against_oracle(b1, acc1, 1e-2)
    w2 = WORKLOADS["tiny"]
    acc2 = [accepted_unit(w2, 0, 0, 0)]
    b2 = run_both([a.inputs for a in acc2], w2)
    check_against_oracle(b2, acc2, 1e-5)
    # and the first problem again, after the smaller one
    b3 = run_both([a.inputs for a in acc1], w1)
    check_against_oracle(b3, acc1, 1e-2)


def test_static_entry_with_more_units_than_the_kernel_arguments_hold():
    """90 short fp32 units in one call: one launch group, whose unit descriptors go through the library's array as
    they go through a caller's workspace."""
    w = WORKLOADS["tiny"].scaled(group=2, window=3, length=("fixed", 300), budget=("fixed", 90), n_sink=4)
    acc = [accepted_unit(w, i, 0, 0, n=120 + 2 * i) for i in range(90)]
    b = run_both([a.inputs for a in acc], w)
    check_against_oracle(b, acc, 1e-5)


def test_static_entry_refuses_a_problem_beyond_its_array():
    import paper_2603_00907_amd as kvs
    w = WORKLOADS["tiny"]
    u = accepted_unit(w, 0, 0, 0).inputs
    small = DeviceBatch([u], group=w.group, window=w.window, head_dim=w.head_dim, dtype=w.dtype, n_sink=w.n_sink)
    big = kvs.Problem(lens=[3_000_000], budgets=[1_000_000], group=w.group, window=w.window, head_dim=w.head_dim,
                      dtype=w.dtype)
    assert kvs.kvs_workspace_size(big) > kvs.STATIC_SCRATCH_BYTES
    with pytest.raises(kvs.KvsError) as e:
        kvs.kvs_step_static(big, small.Q, small.K, small.V, None, small.K_out, small.V_out, small.counts)
    assert e.value.status == kvs.KVS_ERR_WORKSPACE
