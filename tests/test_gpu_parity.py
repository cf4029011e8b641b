"""GPU-vs-oracle parity of the HIP library, called through its C ABI.

Bars: selected edges, slot maps and counts bit-exact; merged K / V within 1e-5 (fp32 I/O) or
1e-2 (bf16 I/O) relative L2 error per output row.  alpha_bar within 3e-5 relative (fp32 dot products of
exact bf16 products: logit error about |e| 6e-8, one more rounding in the exponent's argument, the exponential
itself about 1 ulp, i.e. a few 1e-6 per (query, token), averaged over the rows), o_bar within 3e-5 of
sum_t alpha_bar[t] |V[t]|.
"""

import os

import numpy as np
import pytest

from oracle import kvs_oracle as O
from workloads import WORKLOADS, bf16_bits_to_f32, f32_to_bf16_bits, generate_unit, unit_budget, unit_lengths

from helpers import DeviceBatch, accepted_unit, from_device, rel_err_rows, to_device

pytestmark = pytest.mark.gpu

TOL_KV = {"f32": 1e-5, "bf16": 1e-2}
TOL_ALPHA = 3e-5


def torch_sync():
    import torch
    torch.cuda.synchronize()


def variant(base, **kw):
    return WORKLOADS[base].scaled(**kw)


class switch_override:
    """Sets one of the library's testing switches (include/kvs_debug.h) for the duration of a block."""

    def __init__(self, name, value):
        self.name, self.value = name, value

    def __enter__(self):
        import paper_2603_00907_amd as kvs
        self.old = kvs.kvs_debug_set(self.name, self.value)
        assert self.old >= 0

    def __exit__(self, *a):
        import paper_2603_00907_amd as kvs
        kvs.kvs_debug_set(self.name, self.old)


class switches:
    """Several testing switches at once."""

    def __init__(self, **kw):
        self.items = [switch_override(k, v) for k, v in kw.items()]

    def __enter__(self):
        for it in self.items:
            it.__enter__()

    def __exit__(self, *a):
        for it in reversed(self.items):
            it.__exit__(*a)


def score_path(path):
    """None: the library's own choice; "valu": the vector-ALU score kernels; "fuse": the pass over V carried along in
    sweep 1 (the library does that by itself only for large launches); "nofuse": never carried along; "onepass": the
    one-pass kernel that keeps K in LDS between its phases (windows of 65..128 bf16 rows; the library never picks it
    by itself); "defer": that kernel with a wait limit of zero, so that every work item whose unit is not complete
    at once goes to its second kernel; "narrow": more than 128 query rows with the kernel that keeps 64 rows per
    wavefront in registers (passes of 128 or 256 rows) instead of the one that reads blocks of 64 rows from LDS."""
    if path == "narrow":
        return switches(score_wide=1)
    if path == "fuse":
        return switches(fuse_obar=2)
    if path == "nofuse":
        return switches(fuse_obar=1)
    if path == "onepass":
        return switches(score_fused=2)
    if path == "defer":
        return switches(score_fused=2, fused_wait_us=1)
    return switches(score_path=1 if path == "valu" else 0)


# ------------------------------------------------------------------------------------------------
SCORE_CASES = [
    # base, dtype, D, G, W, lengths, path
    ("tiny", "f32", 64, 1, 8, [1024], None),
    ("tiny", "f32", 128, 2, 3, [777], None),
    ("tiny", "f32", 64, 3, 7, [1300, 64], None),
    ("tiny", "f32", 64, 1, 1, [257], None),
    # fp32 with four query rows or more: the fp32 matrix-core kernel (and the vector-ALU one on the same shapes)
    ("tiny", "f32", 128, 4, 32, [2100, 45], None),                    # 128 rows, a ragged last tile, a short unit
    ("tiny", "f32", 128, 4, 32, [2100], "valu"),
    ("tiny", "f32", 64, 4, 16, [1000, 32], None),                     # head_dim 64, a unit of exactly one tile
    ("tiny", "f32", 128, 5, 32, [1500], None),                        # 160 rows: two launches per sweep
    ("tiny", "f32", 64, 7, 40, [900], None),                          # 280 rows: three launches, the last of 24 rows
    ("tiny", "f32", 128, 1, 16, [5000], None),                        # 16 rows: half a block
    ("stream2560", "f32", 128, 4, 8, [2560, 700], None),              # with cardinalities
    ("stream2560", "f32", 128, 5, 32, [1300], None),                  # ... and two launches
    ("llama8b_8k", "bf16", 128, 4, 32, [2500], None),
    ("llama8b_8k", "bf16", 128, 4, 32, [2500], "valu"),
    # the one-pass kernel (K kept in LDS between the phases): ragged tiles, a last item of a few rows, a one-tile
    # unit, a unit longer than the grid can hold at once (its first items go to the second kernel), 100 query rows,
    # head dim 64, cardinalities, and the same with every wait given up at once
    ("llama8b_8k", "bf16", 128, 4, 32, [2500, 2565, 40, 32, 9000], "onepass"),
    ("llama8b_8k", "bf16", 128, 4, 32, [2500, 2565, 40, 32, 9000], "defer"),
    ("llama8b_8k", "bf16", 128, 4, 32, [300000], "onepass"),
    ("llama8b_8k", "bf16", 64, 4, 32, [1900, 1027], "onepass"),
    ("llama8b_8k", "bf16", 64, 3, 22, [5000, 100], "defer"),                  # 66 rows
    ("llama8b_8k", "bf16", 128, 5, 20, [1500], "onepass"),
    ("stream2560", "bf16", 128, 4, 32, [2560, 700], "onepass"),
    ("stream2560", "bf16", 128, 4, 32, [2560, 700], "defer"),
    ("llama8b_8k", "bf16", 128, 4, 32, [2500, 2053, 40], "fuse"),     # ragged tiles, a last chunk of 5 rows
    ("llama8b_8k", "bf16", 64, 4, 32, [1900], "fuse"),
    ("llama8b_8k", "bf16", 128, 5, 20, [1500], "fuse"),               # 100 query rows
    ("stream2560", "bf16", 128, 4, 32, [2560, 700], "fuse"),          # with cardinalities
    ("llama8b_8k", "bf16", 64, 2, 16, [900], None),
    ("llama8b_8k", "bf16", 128, 1, 20, [700, 33], None),
    ("llama8b_8k", "bf16", 128, 3, 20, [1111], None),
    ("llama8b_8k", "bf16", 128, 5, 20, [1500], None),
    ("llama8b_8k", "bf16", 128, 8, 32, [3000], None),
    ("qwen7b_32k", "bf16", 128, 7, 32, [2100, 100], None),            # 224 query rows in four blocks of 64
    ("qwen7b_32k", "bf16", 128, 7, 32, [2100, 100], "fuse"),
    ("qwen7b_32k", "bf16", 128, 7, 32, [2100], "narrow"),             # ... as two passes of 128 rows
    ("llama8b_8k", "bf16", 128, 5, 32, [1700, 40], "fuse"),           # 160 rows: three blocks
    ("llama8b_8k", "bf16", 128, 5, 29, [1700], None),                 # 145 rows
    ("llama8b_8k", "bf16", 64, 8, 32, [1900], "fuse"),                # 256 rows, head_dim 64
    ("llama8b_8k", "bf16", 128, 8, 32, [3000], "narrow"),
    ("stream2560", "bf16", 128, 7, 32, [2560, 700], "fuse"),          # 224 rows with cardinalities
    ("stress128k", "bf16", 128, 8, 64, [3000], None),                 # 512 rows: two launches of 256 per sweep
    ("stress128k", "bf16", 128, 8, 64, [3000, 77], "fuse"),
    ("stress128k", "bf16", 128, 8, 64, [3000], "narrow"),             # ... passes of 256 rows, four wavefronts a tile
    ("stress128k", "bf16", 128, 8, 100, [1200], None),                # 800 rows: four launches, the last of 32 rows
    ("stress128k", "bf16", 128, 8, 100, [1200], "narrow"),
    ("llama8b_8k", "bf16", 64, 1, 4, [500], None),
    # the vector-ALU kernels as the library's own choice: windows of one to three rows; units shorter than a tile
    ("llama8b_8k", "bf16", 128, 1, 3, [500, 33], None),
    ("llama8b_8k", "bf16", 64, 2, 1, [700], None),
    ("llama8b_8k", "bf16", 128, 4, 8, [20, 600], None),
    ("ragged16", "bf16", 128, 4, 32, [300, 5000, 33000], None),
    # rows that are slots of an already merged cache (cardinalities): every score kernel
    ("stream2560", "bf16", 128, 4, 32, [2560, 700], None),
    ("stream2560", "bf16", 128, 4, 32, [900], "valu"),
    ("stream2560", "bf16", 128, 1, 20, [1500], None),
    ("stream2560", "bf16", 64, 8, 40, [1100], None),
    ("stream2560", "bf16", 64, 8, 40, [1100, 300], "fuse"),           # 320 rows with cardinalities, two launches
    ("stream2560", "f32", 64, 2, 5, [600], None),
]


@pytest.mark.parametrize("base,dtype,D,G,W,lens,path", SCORE_CASES)
def test_score_matches_oracle(base, dtype, D, G, W, lens, path):
    w = variant(base, dtype=dtype, head_dim=D, group=G, window=W, n_seq=len(lens), n_kv_heads=1)
    units = [generate_unit(w, 0, s, 0, n=n) for s, n in enumerate(lens)]
    batch = DeviceBatch(units, group=G, window=W, head_dim=D, dtype=dtype, n_sink=w.n_sink, gap_rows=3)
    with score_path(path):
        if batch.counts_in is None:
            batch.kvs.kvs_score(batch.problem, batch.Q, batch.K, batch.V, batch.alpha_bar, batch.o_bar, batch.ws,
                                stream=batch.stream())
        else:
            batch.kvs.kvs_score_counts(batch.problem, batch.Q, batch.K, batch.V, batch.counts_in, batch.alpha_bar,
                                       batch.o_bar, batch.ws, stream=batch.stream())
        torch_sync()
    batch.check_guards()
    alpha = from_device(batch.alpha_bar)
    obar = from_device(batch.o_bar)
    for i, u in enumerate(units):
        ra, ro = O.score(u.Q, u.K, u.V, counts=u.counts)
        r0 = batch.problem.in_rows[i]
        got = alpha[r0:r0 + len(ra)]
        assert np.isfinite(got).all()
        assert np.max(np.abs(got - ra) / ra) < TOL_ALPHA, (i, np.max(np.abs(got - ra) / ra))
        bound = TOL_ALPHA * (ra @ np.abs(O.slot_values(u.V, u.counts))) + 1e-7
        assert (np.abs(obar[i] - ro) <= bound).all(), (i, np.max(np.abs(obar[i] - ro) / bound))
    # rows between units are never touched
    for i in range(len(units) - 1):
        gap0 = batch.problem.in_rows[i] + lens[i]
        assert (alpha[gap0:gap0 + 3] == -7.0).all()


# ------------------------------------------------------------------------------------------------
# How the selection is spread over workgroups (kvs_debug.h, KVS_DEBUG_SELECT_SPLIT): "none": no workspace is handed
# over, so every unit takes one workgroup; "auto": the library's own choice (several parts of at least 2048 keys
# per unit when the launch leaves compute units idle); "one": one workgroup per unit; "parts": as many parts as a
# unit can have (down to 64 keys each); "give_up": the same with a wait limit of zero, so that the parts leave at
# their first wait and part 0 selects the unit alone.
SPLIT_MODES = {"none": None, "auto": 0, "one": 1, "parts": 2, "give_up": 3}


def run_select(alphas, budgets, n_sink, n_recent, split="auto"):
    import torch
    import paper_2603_00907_amd as kvs
    lens = [len(a) for a in alphas]
    p = kvs.Problem(lens=lens, budgets=budgets, group=1, window=1, head_dim=64, dtype="f32",
                    n_sink=n_sink, n_recent=n_recent)
    flat = torch.from_numpy(np.concatenate(alphas).astype(np.float32)).cuda()
    mask = torch.full((p.rows_in + 64,), 9, dtype=torch.uint8, device="cuda")
    slot = torch.full((p.rows_in + 64,), -7, dtype=torch.int32, device="cuda")
    ws = None
    if SPLIT_MODES[split] is not None:
        # (filled with ones: the library must not rely on what a workspace holds)
        ws = torch.full((kvs.kvs_workspace_size(p),), 0xFF, dtype=torch.uint8, device="cuda")
    with switches(select_split=SPLIT_MODES[split] or 0):
        kvs.kvs_select(p, flat, mask, slot, ws=ws, stream=torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    assert (mask[p.rows_in:] == 9).all() and (slot[p.rows_in:] == -7).all()
    return p, mask.cpu().numpy(), slot.cpu().numpy()


def check_select(alphas, budgets, n_sink, n_recent, split="auto"):
    p, mask, slot = run_select(alphas, budgets, n_sink, n_recent, split)
    for i, a in enumerate(alphas):
        a32 = a.astype(np.float32)
        rm, rs = O.select(a32, budgets[i], n_sink, n_recent, sigma_dtype=np.float32)
        r0 = p.in_rows[i]
        assert (mask[r0:r0 + len(a)] == rm).all(), f"unit {i}: edge mask differs"
        assert (slot[r0:r0 + len(a)] == rs).all(), f"unit {i}: slot map differs"


@pytest.mark.parametrize("n,budget,s,nr,kind", [
    (1024, 512, 32, 0, "dirichlet"), (1000, 100, 32, 0, "lognormal"), (5000, 4999, 32, 0, "lognormal"),
    (5000, 33, 32, 0, "lognormal"), (4096, 1024, 0, 0, "ties"), (4096, 1024, 32, 100, "ties"),
    (3000, 700, 32, 0, "uniform"), (32801, 4096, 32, 0, "lognormal"), (32802, 4096, 32, 0, "lognormal"),
    (40000, 10000, 32, 0, "ties"), (131072, 8192, 32, 0, "lognormal"), (1 << 22, 1 << 20, 32, 0, "lognormal"),
    (70001, 9000, 4, 7, "uniform"), (50003, 25000, 0, 100, "zeros"), (100000, 97000, 1, 100, "ties"),
    (50, 50, 32, 0, "dirichlet"),
    (50, 80, 32, 0, "dirichlet"), (34, 33, 32, 0, "dirichlet"), (1, 1, 32, 0, "dirichlet"),
    (20, 6, 2, 3, "zeros")])
@pytest.mark.parametrize("split", list(SPLIT_MODES))
def test_select_bit_exact(n, budget, s, nr, kind, split):
    if n == 1 << 22 and split not in ("none", "auto"):
        pytest.skip("the longest unit's oracle sort is run for two modes only")
    rng = np.random.default_rng(n * 7 + budget)
    if kind == "dirichlet":
        a = rng.dirichlet(np.ones(n) * 0.5)
    elif kind == "lognormal":
        a = np.exp(4.0 * rng.standard_normal(n))
        a /= a.sum()
    elif kind == "ties":
        a = rng.integers(1, 5, size=n).astype(np.float64) / (2.5 * n)
    elif kind == "uniform":
        a = np.full(n, 1.0 / n)
    else:
        a = np.zeros(n)
    check_select([a], [budget], s, nr, split)


@pytest.mark.parametrize("split", list(SPLIT_MODES))
def test_select_many_ragged_units(split):
    rng = np.random.default_rng(5)
    lens = [int(x) for x in rng.integers(40, 9000, size=70)]       # more than one launch group
    alphas = []
    for n in lens:
        a = np.exp(3.0 * rng.standard_normal(n))
        alphas.append(a / a.sum())
    budgets = [max(33, n // 4) for n in lens]
    budgets[3] = lens[3] + 5                                         # pass-through unit
    check_select(alphas, budgets, 32, 0, split)


@pytest.mark.parametrize("split", ["auto", "parts", "give_up"])
def test_select_long_units_in_a_launch_of_many(split):
    """Forty units in one launch, a quarter of them too long for one workgroup's key cache (more than 32768 tokens),
    with and without parts (forced: more select workgroups than the chip holds at once, so late parts find their
    unit given up or wait for their turn)."""
    rng = np.random.default_rng(23)
    lens = [int(x) for x in rng.integers(3000, 9000, size=30)] + [40000, 65536, 33000, 70001, 50000, 32769 + 40,
                                                                  61000, 36000, 45000, 131072]
    order = rng.permutation(len(lens))
    lens = [lens[i] for i in order]
    alphas = []
    for n in lens:
        a = np.exp(3.0 * rng.standard_normal(n))
        alphas.append(a / a.sum())
    budgets = [max(40, n // 5) for n in lens]
    check_select(alphas, budgets, 32, 0, split)


@pytest.mark.parametrize("split", ["auto", "parts", "give_up"])
def test_select_split_units_of_one_launch_side_by_side(split):
    """Eight long units in one launch (the per-layer call's shape), each selected by several workgroups: heavy ties
    in one, a crowded threshold bin in another (more keys in it than the parts' list holds: every part leaves and
    part 0 selects alone), budgets from almost everything to almost nothing."""
    rng = np.random.default_rng(11)
    lens = [32768, 32768, 20000, 9000, 32768, 70000, 131072, 4200]
    alphas = []
    for i, n in enumerate(lens):
        if i == 1:
            a = rng.integers(1, 4, size=n).astype(np.float64)              # three distinct values: ties everywhere
        elif i == 4:
            a = 1.0 + 1e-7 * rng.integers(0, 3, size=n)                    # nearly constant: one bin holds most keys
        else:
            a = np.exp(3.0 * rng.standard_normal(n))
        alphas.append(a / a.sum())
    budgets = [4096, 4096, 19990, 40, 30000, 8192, 8192, 2100]
    check_select(alphas, budgets, 32, 0, split)


# ------------------------------------------------------------------------------------------------
def merge_case(base, dtype, D, lens, budgets=None, R=(1, 4), seed_layer=0):
    G, W = R
    w = variant(base, dtype=dtype, head_dim=D, group=G, window=W, n_seq=len(lens), n_kv_heads=1)
    units = [generate_unit(w, seed_layer, s, 0, n=n) for s, n in enumerate(lens)]
    if budgets is not None:
        for u, b in zip(units, budgets):
            u.budget = b
    return w, units


@pytest.mark.parametrize("base,dtype,D,lens,budgets", [
    ("tiny", "f32", 64, [1024], None),
    ("tiny", "f32", 128, [700, 41], [300, 35]),
    ("llama8b_8k", "bf16", 128, [3000, 257], [700, 100]),
    ("llama8b_8k", "bf16", 64, [2000], [1999]),
    ("tiny", "f32", 64, [600], [33]),            # one run swallows everything after the sinks
    ("tiny", "f32", 64, [300, 200], [300, 500]),  # pass-through
    ("stream2560", "bf16", 128, [2560, 300], None),          # rows with cardinalities
    ("stream2560", "f32", 64, [1200], [500]),
    ("stream2560", "bf16", 64, [900], [899]),
])
def test_merge_compact_matches_oracle(base, dtype, D, lens, budgets):
    check_merge_compact(base, dtype, D, lens, budgets, "hessian")


@pytest.mark.parametrize("rule", ["diagonal", "mean"])
@pytest.mark.parametrize("base,dtype,D,lens,budgets", [
    ("tiny", "f32", 64, [1024, 90], None),
    ("llama8b_8k", "bf16", 128, [3000], [700]),
    ("stream2560", "bf16", 128, [1300], [1000]),
    ("stream2560", "f32", 64, [700], [200]),
])
def test_merge_compact_ablation_rules(base, dtype, D, lens, budgets, rule):
    """The Key rule without the coupling blocks, and the plain mean, on the same ABI (kvs_problem.key_rule)."""
    check_merge_compact(base, dtype, D, lens, budgets, rule)


@pytest.mark.parametrize("with_ws", [False, True])
def test_merge_compact_more_units_than_the_kernel_arguments_hold(with_ws):
    """150 units of 40 to 330 rows in one kvs_merge_compact call.  Its workspace is optional: without one the units
    go out 64 per launch, with one in a single launch whose unit descriptors live in the workspace."""
    lens = [40 + (37 * i) % 291 for i in range(150)]
    check_merge_compact("llama8b_8k", "bf16", 128, lens, [max(36, n // 3) for n in lens], "hessian", with_ws=with_ws)


def check_merge_compact(base, dtype, D, lens, budgets, rule, with_ws=False):
    import torch
    w, units = merge_case(base, dtype, D, lens, budgets)
    batch = DeviceBatch(units, group=w.group, window=w.window, head_dim=D, dtype=dtype, n_sink=w.n_sink,
                        key_rule=rule)
    p = batch.problem
    refs = []
    alpha_all = np.zeros(p.rows_in, dtype=np.float32)
    mask_all = np.zeros(p.rows_in, dtype=np.uint8)
    slot_all = np.zeros(p.rows_in, dtype=np.int32)
    obar_all = np.zeros((len(units), D), dtype=np.float32)
    for i, u in enumerate(units):
        a, o = O.score(u.Q, u.K, u.V, counts=u.counts)
        a32, o32 = a.astype(np.float32), o.astype(np.float32)
        mask, slot = O.select(a32, u.budget, w.n_sink, 0, sigma_dtype=np.float32)
        refs.append(O.merge_compact(u.K, u.V, a32.astype(np.float64), o32.astype(np.float64), mask, slot,
                                    counts_in=u.counts, rule=rule))
        r0 = p.in_rows[i]
        alpha_all[r0:r0 + len(a)] = a32
        mask_all[r0:r0 + len(a)] = mask
        slot_all[r0:r0 + len(a)] = slot
        obar_all[i] = o32
    dev_args = (torch.from_numpy(alpha_all).cuda(), torch.from_numpy(obar_all).cuda(),
                torch.from_numpy(mask_all).cuda(), torch.from_numpy(slot_all).cuda())
    ws = batch.ws if with_ws else None
    if batch.counts_in is None:
        batch.kvs.kvs_merge_compact(p, batch.K, batch.V, *dev_args, batch.K_out, batch.V_out, batch.counts,
                                    ws=ws, stream=batch.stream())
    else:
        batch.kvs.kvs_merge_compact_counts(p, batch.K, batch.V, batch.counts_in, *dev_args, batch.K_out,
                                           batch.V_out, batch.counts, ws=ws, stream=batch.stream())
    torch_sync()
    batch.check_guards()
    compare_outputs(batch, refs, dtype)


def compare_outputs(batch, refs, dtype, strict_guard=True):
    p = batch.problem
    Ko, Vo, cnt = from_device(batch.K_out), from_device(batch.V_out), batch.counts.cpu().numpy()
    for i, ref in enumerate(refs):
        r0, n_out = p.out_rows[i], p.n_out[i]
        assert ref.K_out.shape[0] == n_out
        assert (cnt[r0:r0 + n_out] == ref.counts).all(), f"unit {i}: counts differ"
        ek = rel_err_rows(Ko[r0:r0 + n_out], ref.K_out)
        ev = rel_err_rows(Vo[r0:r0 + n_out], ref.V_out)
        assert ek <= TOL_KV[dtype], f"unit {i}: merged K rel err {ek:.3e}"
        assert ev <= TOL_KV[dtype], f"unit {i}: merged V rel err {ev:.3e}"
        single = ref.n_rows == 1
        assert (Ko[r0:r0 + n_out][single] == ref.K_out[single]).all(), f"unit {i}: singleton K not a copy"
        assert (Vo[r0:r0 + n_out][single] == ref.V_out[single]).all(), f"unit {i}: singleton V not a copy"


def test_merge_fallback_and_identical_keys():
    """Crafted inputs: (a) residuals exactly zero -> denominator 0 -> arithmetic mean on both sides;
    (b) identical Keys in a run merge to that Key."""
    import torch
    import paper_2603_00907_amd as kvs
    rng = np.random.default_rng(3)
    n, D = 96, 64
    K = rng.standard_normal((n, D)).astype(np.float32)
    V = rng.standard_normal((n, D)).astype(np.float32)
    obar = rng.standard_normal(D).astype(np.float32)
    V[10:14] = obar                       # zero residuals: A = C = 0 on the run 10..13
    K[40:45] = K[40]                      # identical Keys on the run 40..44
    alpha = rng.dirichlet(np.ones(n)).astype(np.float32)
    mask = np.zeros(n, dtype=np.uint8)
    mask[10:13] = 1
    mask[40:44] = 1
    mask[70] = 1
    starts = np.ones(n, dtype=np.int64)
    starts[1:] = 1 - mask[:-1]
    slot = (np.cumsum(starts) - 1).astype(np.int32)
    n_out = int(slot[-1]) + 1
    ref = O.merge_compact(K, V, alpha.astype(np.float64), obar.astype(np.float64), mask, slot)
    assert ref.fallback[10] and ref.fallback.sum() == 1
    p = kvs.Problem(lens=[n], budgets=[n_out], group=1, window=1, head_dim=D, dtype="f32", n_sink=4)
    Ko = torch.zeros((n_out, D), device="cuda")
    Vo = torch.zeros((n_out, D), device="cuda")
    cnt = torch.zeros(n_out, dtype=torch.int32, device="cuda")
    kvs.kvs_merge_compact(p, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda(), torch.from_numpy(alpha).cuda(),
                          torch.from_numpy(obar[None]).cuda(), torch.from_numpy(mask).cuda(),
                          torch.from_numpy(slot).cuda(), Ko, Vo, cnt)
    torch.cuda.synchronize()
    assert (cnt.cpu().numpy() == ref.counts).all()
    assert rel_err_rows(Ko.cpu().numpy(), ref.K_out) < 1e-5
    assert rel_err_rows(Vo.cpu().numpy(), ref.V_out) < 1e-5
    np.testing.assert_allclose(Ko.cpu().numpy()[10], K[10:14].mean(axis=0), rtol=1e-6)
    np.testing.assert_allclose(Ko.cpu().numpy()[37], K[40], rtol=2e-6)


def run_crafted_merge(K, V, alpha, obar, mask, dtype, counts=None, n_sink=0):
    """kvs_merge_compact(_counts) on one hand-made unit (fp32 arrays whose values the I/O dtype represents exactly);
    returns the oracle's result on the same inputs and the GPU outputs as fp32 arrays."""
    import torch
    import paper_2603_00907_amd as kvs
    n, D = K.shape
    starts = np.ones(n, dtype=np.int64)
    starts[1:] = 1 - mask[:-1]
    slot = (np.cumsum(starts) - 1).astype(np.int32)
    n_out = int(slot[-1]) + 1
    ref = O.merge_compact(K, V, alpha.astype(np.float64), obar.astype(np.float64), mask, slot, counts_in=counts)
    p = kvs.Problem(lens=[n], budgets=[n_out], group=1, window=1, head_dim=D, dtype=dtype, n_sink=n_sink)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    Ko = torch.full((n_out + 8, D), 512.0, dtype=tdt, device="cuda")
    Vo = torch.full((n_out + 8, D), 512.0, dtype=tdt, device="cuda")
    cnt = torch.full((n_out + 8,), -7, dtype=torch.int32, device="cuda")
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()  # noqa: E731
    args = (dev(alpha.astype(np.float32)), dev(obar.astype(np.float32)[None]), dev(mask), dev(slot), Ko, Vo, cnt)
    if counts is None:
        kvs.kvs_merge_compact(p, to_device(K, dtype), to_device(V, dtype), *args)
    else:
        kvs.kvs_merge_compact_counts(p, to_device(K, dtype), to_device(V, dtype), dev(counts.astype(np.int32)), *args)
    torch.cuda.synchronize()
    assert (Ko[n_out:].float() == 512.0).all() and (Vo[n_out:].float() == 512.0).all() and (cnt[n_out:] == -7).all()
    return ref, from_device(Ko[:n_out]), from_device(Vo[:n_out]), cnt[:n_out].cpu().numpy()


@pytest.mark.parametrize("with_counts", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_merge_with_attention_mass_at_and_above_one_half(dtype, with_counts):
    """The Key rule's two edge cases (App. C assumes merged Keys carry alpha < 1/2; Sec. 4.2, Eqs. c11_def-c12_def
    carry the factor 1 - 2 alpha): hand-made attention distributions put, inside merged runs, a token with
    alpha > 1/2 (the norm takes |1 - 2 alpha|), a token with alpha = 1/2 exactly (A_t = 0), and a pair whose
    weight denominator A_m - 2 C_m + A_{m+1} is negative (both masses just below 1/2: A nearly 0, C large), where
    both sides must take the arithmetic mean.  Three units, one per case (each distribution sums to one)."""
    rng = np.random.default_rng(17)
    n, D = 80, 64
    bf = lambda x: bf16_bits_to_f32(f32_to_bf16_bits(x.astype(np.float32)))  # noqa: E731
    for case in ("above", "exactly", "negative"):
        K = bf(rng.standard_normal((n, D)))
        V = bf(rng.standard_normal((n, D)))
        obar = (0.1 * rng.standard_normal(D)).astype(np.float32)
        counts = rng.integers(1, 5, size=n).astype(np.int32) if with_counts else None
        alpha = np.zeros(n, dtype=np.float64)
        mask = np.zeros(n, dtype=np.uint8)
        mask[20:23] = 1                                   # run 20..23
        mask[50] = 1                                      # pair 50, 51
        mask[60:62] = 1                                   # run 60..62 (ordinary masses)
        if case == "above":
            alpha[21] = 0.7                               # inside the run 20..23
            rest = 0.3
        elif case == "exactly":
            alpha[22] = 0.5
            rest = 0.5
            V[22] = bf(2.0 * obar - V[21] + 0.05 * rng.standard_normal(D))   # r_22 close to -r_21: C_21 stays small and
                                                                           # the denominator well away from zero
        else:
            alpha[50] = alpha[51] = 0.499                 # A_50, A_51 tiny, C_50 large: a negative denominator
            rest = 0.002
        free = np.array([t for t in range(n) if alpha[t] == 0.0])
        alpha[free] = rest * rng.dirichlet(np.ones(len(free)))
        alpha = alpha.astype(np.float32).astype(np.float64)   # what the kernel is given
        ref, Ko, Vo, cnt = run_crafted_merge(K, V, alpha, obar, mask, dtype, counts)
        pair_slot = 50 - 3                                # three edges selected before token 50
        if case == "negative":
            assert ref.fallback[pair_slot] and ref.U[pair_slot] < 0 and ref.fallback.sum() == 1
            c = np.ones(2) if counts is None else counts[50:52].astype(np.float64)
            mean = (c[:, None] * K[50:52]).sum(axis=0) / c.sum()
            np.testing.assert_allclose(Ko[pair_slot], mean, rtol=TOL_KV[dtype], atol=TOL_KV[dtype] * 0.1)
        else:
            assert not ref.fallback.any() and O.conditioning(ref) > 0.05, case
            run_slot = 20
            assert ref.n_rows[run_slot] == 4
        assert (cnt == ref.counts).all(), case
        assert rel_err_rows(Ko, ref.K_out) <= TOL_KV[dtype], (case, rel_err_rows(Ko, ref.K_out))
        assert rel_err_rows(Vo, ref.V_out) <= TOL_KV[dtype], case
        single = ref.n_rows == 1
        assert (Ko[single] == ref.K_out[single]).all() and (Vo[single] == ref.V_out[single]).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_merge_with_a_hand_made_mask_whose_last_byte_is_set(dtype):
    """An edge mask from outside the library: the byte of the unit's last token is set (there is no edge after it).
    The kernel reads it as 0, like the oracle, whose runs end with the unit: the last slot is the run that leads
    up to the last token, no row is written past the unit's outputs."""
    rng = np.random.default_rng(23)
    n, D = 300, 128
    bf = lambda x: bf16_bits_to_f32(f32_to_bf16_bits(x.astype(np.float32)))  # noqa: E731
    K, V = bf(rng.standard_normal((n, D))), bf(rng.standard_normal((n, D)))
    alpha = rng.dirichlet(np.ones(n))
    obar = (alpha @ V).astype(np.float32)
    mask = (rng.random(n) < 0.6).astype(np.uint8)
    mask[:4] = 0
    mask[n - 3:] = 1                                      # the last three tokens form a run, and the last byte is set
    ref, Ko, Vo, cnt = run_crafted_merge(K, V, alpha.astype(np.float32).astype(np.float64), obar, mask, dtype)
    assert ref.n_rows[-1] >= 3 and ref.counts.sum() == n
    assert (cnt == ref.counts).all()
    assert rel_err_rows(Ko, ref.K_out) <= TOL_KV[dtype] and rel_err_rows(Vo, ref.V_out) <= TOL_KV[dtype]


def test_merge_bf16_output_rounds_to_nearest_even():
    """Sums that fall exactly between two bf16 values go to the even one (one rounding, at the store)."""
    import torch
    import paper_2603_00907_amd as kvs
    n, D = 8, 64
    rng = np.random.default_rng(11)
    K = rng.integers(-3, 4, size=(n, D)).astype(np.float32)
    V = rng.integers(-3, 4, size=(n, D)).astype(np.float32)
    V[2], V[3] = 1.0, 2.0 ** -8              # 1.00390625: tie between 1.0 (even) and 1.0078125
    V[5], V[6] = 1.0078125, 2.0 ** -8        # 1.01171875: tie between 1.0078125 (odd) and 1.015625
    mask = np.array([0, 0, 1, 0, 0, 1, 0, 0], dtype=np.uint8)
    slot = np.array([0, 1, 2, 2, 3, 4, 4, 5], dtype=np.int32)
    alpha = np.full(n, 1.0 / n, dtype=np.float32)
    obar = np.zeros((1, D), dtype=np.float32)
    p = kvs.Problem(lens=[n], budgets=[6], group=1, window=1, head_dim=D, dtype="bf16", n_sink=0)
    dev = lambda x: torch.from_numpy(x).cuda()  # noqa: E731
    Ko = torch.zeros((6, D), dtype=torch.bfloat16, device="cuda")
    Vo = torch.zeros((6, D), dtype=torch.bfloat16, device="cuda")
    cnt = torch.zeros(6, dtype=torch.int32, device="cuda")
    kvs.kvs_merge_compact(p, dev(K).bfloat16(), dev(V).bfloat16(), dev(alpha), dev(obar), dev(mask), dev(slot),
                          Ko, Vo, cnt)
    torch.cuda.synchronize()
    Vg = Vo.float().cpu().numpy()
    assert (Vg[2] == 1.0).all() and (Vg[4] == 1.015625).all()
    assert cnt.cpu().numpy().tolist() == [1, 1, 2, 1, 2, 1]
    assert (Vg[0] == V[0]).all() and (Ko.float().cpu().numpy()[3] == K[4]).all()


CAUSAL_CASES = [
    # base, dtype, D, G, W, lengths, path: every score kernel, masked rows across tile and chunk borders
    ("tiny", "f32", 128, 4, 32, [2053, 40], None),              # fp32 matrix-core kernel, 128 rows
    ("tiny", "f32", 64, 5, 32, [900], None),                    # ... 160 rows in two launches
    ("tiny", "f32", 64, 2, 5, [777, 5], None),                  # vector-ALU kernel; a unit that is all window
    ("llama8b_8k", "bf16", 128, 1, 20, [700, 33], None),        # 20 rows in one MFMA block
    ("llama8b_8k", "bf16", 64, 2, 32, [900], None),             # 64 rows
    ("llama8b_8k", "bf16", 128, 4, 32, [2500, 2053], "fuse"),   # (with the pass over V carried along)
    ("llama8b_8k", "bf16", 128, 4, 32, [2500, 2053], None),     # 128 rows in one pass; a last chunk of 5 rows, all
    ("llama8b_8k", "bf16", 128, 4, 32, [2053], "valu"),         # of them masked for most rows
    ("llama8b_8k", "bf16", 128, 4, 32, [2500, 2053, 600], "onepass"),   # the one-pass kernel: an item of 5 rows that most
    ("llama8b_8k", "bf16", 128, 4, 32, [2500, 2053, 600], "defer"),     # query rows do not see at all
    ("llama8b_8k", "bf16", 64, 3, 22, [1500, 1029], "onepass"),         # 66 rows, head dim 64: items of 1024 rows, one of 5
    ("llama8b_8k", "bf16", 128, 8, 32, [3000], None),           # 256 rows in one pass (four blocks of 64)
    ("llama8b_8k", "bf16", 128, 8, 32, [3000, 2053], "fuse"),
    ("llama8b_8k", "bf16", 128, 8, 32, [3000], "narrow"),       # 256 rows, two wavefronts per pass
    ("qwen7b_32k", "bf16", 128, 5, 32, [2053, 40], None),       # 160 rows: three blocks
    ("stress128k", "bf16", 128, 8, 40, [1200], None),           # 320 rows, window 40 crosses two tiles
    ("stress128k", "bf16", 128, 8, 40, [1200, 45], "fuse"),
    ("stress128k", "bf16", 128, 8, 40, [1200], "narrow"),
    ("stream2560", "bf16", 128, 4, 32, [2560], None),           # with cardinalities (the tail rows are fresh tokens)
]


@pytest.mark.parametrize("base,dtype,D,G,W,lens,path", CAUSAL_CASES)
def test_score_with_causal_window_matches_oracle(base, dtype, D, G, W, lens, path):
    w = variant(base, dtype=dtype, head_dim=D, group=G, window=W, n_seq=len(lens), n_kv_heads=1)
    units = [generate_unit(w, 0, s, 0, n=n) for s, n in enumerate(lens)]
    batch = DeviceBatch(units, group=G, window=W, head_dim=D, dtype=dtype, n_sink=w.n_sink, gap_rows=3, causal=True)
    with score_path(path):
        batch.kvs.kvs_score_counts(batch.problem, batch.Q, batch.K, batch.V, batch.counts_in, batch.alpha_bar,
                                   batch.o_bar, batch.ws, stream=batch.stream())
        torch_sync()
    batch.check_guards()
    alpha = from_device(batch.alpha_bar)
    obar = from_device(batch.o_bar)
    for i, u in enumerate(units):
        ra, ro = O.score(u.Q, u.K, u.V, counts=u.counts, causal_window=W)
        plain, _ = O.score(u.Q, u.K, u.V, counts=u.counts)
        assert np.max(np.abs(plain - ra) / ra) > 1e-2            # the mask matters on this input
        r0 = batch.problem.in_rows[i]
        got = alpha[r0:r0 + len(ra)]
        assert np.isfinite(got).all()
        assert np.max(np.abs(got - ra) / ra) < TOL_ALPHA, (i, np.max(np.abs(got - ra) / ra))
        bound = TOL_ALPHA * (ra @ np.abs(O.slot_values(u.V, u.counts))) + 1e-7
        assert (np.abs(obar[i] - ro) <= bound).all(), (i, np.max(np.abs(obar[i] - ro) / bound))


# ------------------------------------------------------------------------------------------------
def run_step(w, accepted, path=None, causal=False):
    units = [a.inputs for a in accepted]
    batch = DeviceBatch(units, group=w.group, window=w.window, head_dim=w.head_dim, dtype=w.dtype,
                        n_sink=w.n_sink, n_recent=w.n_recent, causal=causal)
    with score_path(path):
        if batch.counts_in is None:
            batch.kvs.kvs_step(batch.problem, batch.Q, batch.K, batch.V, batch.K_out, batch.V_out, batch.counts,
                               batch.ws, slot_of_token_out=batch.slot, edge_mask_out=batch.mask,
                               stream=batch.stream())
        else:
            batch.kvs.kvs_step_counts(batch.problem, batch.Q, batch.K, batch.V, batch.counts_in, batch.K_out,
                                      batch.V_out, batch.counts, batch.ws, slot_of_token_out=batch.slot,
                                      edge_mask_out=batch.mask, stream=batch.stream())
        torch_sync()
    batch.check_guards()
    return batch


def check_step(w, accepted, path=None, causal=False):
    batch = run_step(w, accepted, path, causal)
    p = batch.problem
    mask, slot = batch.mask.cpu().numpy(), batch.slot.cpu().numpy()
    for i, a in enumerate(accepted):
        r0, n = p.in_rows[i], a.inputs.n
        assert (mask[r0:r0 + n] == a.ref.mask).all(), f"unit {i}: selected edges differ (gap {a.gap:.2e})"
        assert (slot[r0:r0 + n] == a.ref.slot).all(), f"unit {i}: slot map differs"
    compare_outputs(batch, [a.ref.merged for a in accepted], w.dtype)
    return batch


def test_step_tiny_config():
    w = WORKLOADS["tiny"]
    check_step(w, [accepted_unit(w, 0, 0, 0)])


def test_step_tiny_config_is_deterministic():
    w = WORKLOADS["tiny"]
    acc = [accepted_unit(w, 0, 0, 0)]
    b1 = run_step(w, acc)
    b2 = run_step(w, acc)
    import torch
    assert torch.equal(b1.K_out.view(torch.int32), b2.K_out.view(torch.int32))
    assert torch.equal(b1.V_out.view(torch.int32), b2.V_out.view(torch.int32))
    assert torch.equal(b1.counts, b2.counts)


@pytest.mark.parametrize("n_units,n", [(3, 3000), (100, 600)])
def test_step_replayed_from_a_hip_graph_equals_the_eager_step(n_units, n):
    """The library never allocates, memsets or synchronises, so a step can be captured as it is.  The graph is
    replayed three times, with the outputs scrubbed and other work on the device in between; every replay must
    reproduce the eager result bit for bit.  With 100 units the launch group's unit descriptors go through the
    workspace (which is scrubbed between the replays): the kernels that write them there are part of the graph."""
    import torch
    w = WORKLOADS["llama8b_8k"].scaled(length=("fixed", n), budget=("fixed", n // 4 + 50))
    acc = [accepted_unit(w, h // 8, 0, h % 8) for h in range(n_units)]
    eager = check_step(w, acc)
    batch = DeviceBatch([a.inputs for a in acc], group=w.group, window=w.window, head_dim=w.head_dim, dtype=w.dtype,
                        n_sink=w.n_sink)

    def step(stream):
        batch.kvs.kvs_step(batch.problem, batch.Q, batch.K, batch.V, batch.K_out, batch.V_out, batch.counts,
                           batch.ws, slot_of_token_out=batch.slot, edge_mask_out=batch.mask, stream=stream)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step(side.cuda_stream)                               # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step(torch.cuda.current_stream().cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    n_out = batch.problem.rows_out
    for replay in range(3):
        batch.K_out.fill_(512.0)                             # eager work between the replays
        batch.V_out.fill_(512.0)
        batch.counts.fill_(-7)
        batch.ws.zero_()
        scratch = torch.randn(1 << 20, device="cuda").sum()
        torch_sync()
        graph.replay()
        torch_sync()
        assert torch.isfinite(scratch)
        assert torch.equal(batch.K_out[:n_out].view(torch.int16), eager.K_out[:n_out].view(torch.int16)), replay
        assert torch.equal(batch.V_out[:n_out].view(torch.int16), eager.V_out[:n_out].view(torch.int16)), replay
        assert torch.equal(batch.counts[:n_out], eager.counts[:n_out]), replay
        assert torch.equal(batch.slot, eager.slot) and torch.equal(batch.mask, eager.mask)
        batch.check_guards()


@pytest.mark.parametrize("path", [None, "valu", "fuse", "onepass", "defer"])
def test_step_llama8b_8k_config(path):
    w = WORKLOADS["llama8b_8k"]
    heads = range(w.n_kv_heads) if path != "valu" else range(2)
    check_step(w, [accepted_unit(w, 0, 0, h) for h in heads], path)


@pytest.mark.parametrize("path", [None, "fuse", "narrow"])
def test_step_qwen_shape_reduced(path):
    """Qwen2-7B layout (7 query heads per KV head: 224 query rows, the one-pass score kernel with four blocks of 64
    rows), 8192 -> 2048 tokens."""
    w = WORKLOADS["qwen7b_32k"].scaled(length=("fixed", 8192), budget=("fixed", 2048))
    check_step(w, [accepted_unit(w, 0, 0, h) for h in range(2)], path)


def test_step_qwen_shape_full_size_two_heads():
    """The same layout at the headline's length, 32768 -> 4096 tokens, two KV heads of one layer."""
    w = WORKLOADS["qwen7b_32k"]
    check_step(w, [accepted_unit(w, 3, 0, h) for h in range(2)])


def test_step_fp32_on_the_llama_layout_reduced():
    """fp32 caches with a 128-row window (the fp32 matrix-core score kernel), 4096 -> 1024 tokens: the 1e-5 bar."""
    w = WORKLOADS["llama8b_8k"].scaled(dtype="f32", length=("fixed", 4096), budget=("fixed", 1024))
    check_step(w, [accepted_unit(w, 0, 0, h) for h in range(2)])
    check_step(w, [accepted_unit(w, 0, 0, 0)], "valu")


def random_step_case(rng):
    """One random but seeded shape of the step: dtype, head dim, GQA group, window, length, budget, sink and recent
    rows, cardinalities or the causal mask, the number of units and the score path."""
    dtype = str(rng.choice(["bf16", "bf16", "f32"]))
    D = int(rng.choice([64, 128]))
    G = int(rng.choice([1, 2, 4, 5, 7, 8]))
    W = int(rng.choice([1, 3, 8, 16, 32, 40]))
    counts = bool(rng.random() < 0.3)
    causal = bool(rng.random() < 0.25) and not counts
    n = int(rng.choice([rng.integers(300, 900), rng.integers(900, 3000), rng.integers(3000, 7000)]))
    n = max(n, 700 if counts else 0, W + 80)
    n_sink = int(rng.choice([0, 4, 32]))
    n_recent = int(rng.choice([0, 0, 16]))
    budget = max(int(n * float(rng.choice([0.125, 0.25, 0.5, 0.8]))), n_sink + n_recent + 8)
    kw = dict(dtype=dtype, head_dim=D, group=G, window=W, length=("fixed", n), budget=("fixed", budget),
              n_sink=n_sink, n_recent=n_recent)
    if counts:
        kw["fresh_tail"] = min(512, n // 5)
    w = WORKLOADS["stream2560" if counts else "llama8b_8k"].scaled(**kw)
    path = rng.choice([None, None, "fuse", "narrow"])
    return w, causal, int(rng.integers(1, 4)), path


@pytest.mark.parametrize("seed", range(16))
def test_step_random_shapes(seed):
    """Seeded random shapes (every score kernel, both dtypes, ragged tiles, sink and recent rows, budgets from an
    eighth to four fifths of the length), each unit accepted and compared like the named configurations."""
    rng = np.random.default_rng(1000 + seed)
    w, causal, n_units, path = random_step_case(rng)
    accepted = [accepted_unit(w, 0, 0, h, causal=causal) for h in range(n_units)]
    check_step(w, accepted, path, causal=causal)


@pytest.mark.parametrize("dtype,D,G,W,n,B,causal", [
    ("bf16", 128, 4, 32, 3000, 700, False), ("f32", 64, 2, 4, 1500, 300, False), ("bf16", 64, 4, 8, 5000, 1250, True)])
@pytest.mark.parametrize("zeroed", ["Q", "K"])
def test_step_with_uniform_attention(dtype, D, G, W, n, B, causal, zeroed):
    """Queries or Keys that are all zero: every logit is 0, every token has the same mass (under the causal mask:
    the same within the window's steps), so all edge scores tie and the selection is decided by the index alone.
    No acceptance rule applies (the gap is zero by construction): both sides must break the ties alike."""
    from helpers import AcceptedUnit
    w = WORKLOADS["llama8b_8k"].scaled(dtype=dtype, head_dim=D, group=G, window=W, length=("fixed", n),
                                       budget=("fixed", B))
    u = generate_unit(w, 0, 0, 0, n=n)
    if zeroed == "Q":
        u.Q = np.zeros_like(u.Q)
    else:
        u.K = np.zeros_like(u.K)
    ab, ob = O.score(u.Q, u.K, u.V, causal_window=W if causal else 0)
    mask, slot = O.select(ab.astype(np.float32), u.budget, w.n_sink, w.n_recent, sigma_dtype=np.float32)
    merged = O.merge_compact(u.K, u.V, ab, ob, mask, slot)
    check_step(w, [AcceptedUnit(u, O.StepResult(ab, ob, mask, slot, merged), 0.0, 1.0)], causal=causal)


def test_streaming_loop_of_steps():
    streaming_loop(check_step, per_query=False)


def streaming_loop(check, per_query):
    """The deployment loop of Sec. 3.1 / Sec. 5: a cache is merged down to the budget, a chunk of fresh tokens arrives,
    and the cache of budget + chunk rows is merged again: six rounds for two heads (2560 -> 2048, five times 2048 +
    512 -> 2048).  Every round's input is the GPU's own output of the round before, exactly as stored (merged Keys,
    Value sums, cardinalities), followed by the fresh rows; the oracle takes one step from that same input and the
    round is compared like any other step (partition bit for bit, cardinalities exact).  At the end every token that
    ever arrived is accounted for."""
    from helpers import AcceptedUnit, COND_MIN, GAP_MIN
    from workloads.generator import UnitInputs
    w = WORKLOADS["stream2560"]
    plain = WORKLOADS["llama8b_8k"]                  # the recipe of the arriving tokens (same shape and dtype)
    B, chunk, rounds, heads = 2048, 512, 6, 2
    total = B + chunk * rounds
    src = [generate_unit(plain, 0, 0, h, n=total) for h in range(heads)]
    state = [(u.K[:B + chunk], u.V[:B + chunk], np.ones(B + chunk, dtype=np.int32)) for u in src]
    for r in range(rounds):
        accepted = []
        for h, (K, V, c) in enumerate(state):
            for attempt in range(200):
                Q = generate_unit(plain, 1 + r, 0, h, attempt=attempt, n=64).Q          # a fresh window of queries
                u = UnitInputs(layer=r, seq=0, head=h, attempt=attempt, n=len(K), budget=B, rho=0.0, Q=Q, K=K, V=V,
                               counts=c)
                ab, ob = O.score(Q, K, V, counts=c)
                gap = O.boundary_gap(ab, B, w.n_sink, w.n_recent)
                if gap < GAP_MIN:
                    continue
                mask, slot = O.select(ab, B, w.n_sink, w.n_recent)
                norms = O.per_query_norms(Q, K, V, counts=c) if per_query else None
                merged = O.merge_compact(K, V, ab, ob, mask, slot, counts_in=c, norms=norms)
                if O.conditioning(merged) >= COND_MIN:
                    break
            else:
                raise RuntimeError("no accepted attempt found")
            accepted.append(AcceptedUnit(u, O.StepResult(ab, ob, mask, slot, merged), gap, 1.0))
        batch = check(w, accepted)
        p = batch.problem
        Ko, Vo, cnt = from_device(batch.K_out), from_device(batch.V_out), batch.counts.cpu().numpy()
        state = []
        for h in range(heads):
            r0 = p.out_rows[h]
            assert cnt[r0:r0 + B].sum() == B + chunk * (r + 1)           # no token lost, none counted twice
            if r + 1 == rounds:
                continue
            lo = B + chunk * (r + 1)
            fresh = slice(lo, lo + chunk)
            state.append((np.concatenate([Ko[r0:r0 + B], src[h].K[fresh]]),
                          np.concatenate([Vo[r0:r0 + B], src[h].V[fresh]]),
                          np.concatenate([cnt[r0:r0 + B], np.ones(chunk, dtype=np.int32)]).astype(np.int32)))


def test_step_with_causal_window():
    """The whole step with the causal mask inside the window, bf16 (MFMA score) and fp32 (vector-ALU score)."""
    w = WORKLOADS["llama8b_8k"]
    check_step(w, [accepted_unit(w, 0, 0, h, causal=True) for h in range(2)], causal=True)
    w = WORKLOADS["tiny"]
    check_step(w, [accepted_unit(w, 0, 0, 0, causal=True)], causal=True)


def test_step_llama8b_32k_one_layer_full_size():
    """The headline workload's launch configuration: one layer, 8 KV heads x 32768 tokens -> 4096."""
    w = WORKLOADS["llama8b_32k"]
    batch = check_step(w, [accepted_unit(w, 5, 0, h) for h in range(w.n_kv_heads)])
    import torch
    b2 = run_step(w, [accepted_unit(w, 5, 0, h) for h in range(w.n_kv_heads)])
    assert torch.equal(batch.K_out.view(torch.int16), b2.K_out.view(torch.int16))     # run-to-run bitwise


def test_step_headline_workload_in_the_launch_configuration_of_the_bench():
    """All 32 layers x 8 KV heads of the headline workload the way bench.py times them: two kvs_step calls of 16
    layers (128 units, launch groups of 64 units = 8 layers) on two streams, each with its own workspace.  EVERY one
    of the 256 units is compared with the oracle like any other unit (its accepted Query redraw comes from the
    manifest, so the oracle runs once per unit, sixteen units side by side on the host); a unit for which no redraw
    is accepted would be held to the invariants that hold for any selection (none occurs)."""
    import torch
    from concurrent.futures import ThreadPoolExecutor
    from threadpoolctl import threadpool_limits
    import paper_2603_00907_amd as kvs
    from helpers import to_device
    from workloads import unit_budget
    w = WORKLOADS["llama8b_32k"]
    H, D, R, n = w.n_kv_heads, w.head_dim, w.q_rows, unit_lengths(w)[0]
    B = unit_budget(w, n)
    nu = w.layers * H
    K = torch.empty((nu * n, D), dtype=torch.bfloat16, device="cuda")
    V = torch.empty_like(K)
    Q = torch.empty((nu, R, D), dtype=torch.bfloat16, device="cuda")
    refs = [None] * nu

    def unit(i):
        try:
            a = accepted_unit(w, i // H, 0, i % H)
        except RuntimeError:                                  # no accepted redraw: invariants only
            return generate_unit(w, i // H, 0, i % H), None
        m = a.ref.merged
        return a.inputs, (a.ref.mask, a.ref.slot, m.counts, m.K_out, m.V_out, m.n_rows, a.gap)

    with threadpool_limits(limits=1), ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
        for i, (u, ref) in enumerate(pool.map(unit, range(nu))):
            K[i * n:(i + 1) * n] = to_device(u.K, "bf16")
            V[i * n:(i + 1) * n] = to_device(u.V, "bf16")
            Q[i] = to_device(u.Q.reshape(R, D), "bf16")
            refs[i] = ref
    half = nu // 2
    p = kvs.Problem(lens=[n] * half, budgets=[B] * half, group=w.group, window=w.window, head_dim=D, dtype="bf16",
                    n_sink=w.n_sink, n_recent=w.n_recent)
    K_out = torch.empty((nu * B, D), dtype=torch.bfloat16, device="cuda")
    V_out = torch.empty_like(K_out)
    counts = torch.empty(nu * B, dtype=torch.int32, device="cuda")
    mask = torch.empty(nu * n, dtype=torch.uint8, device="cuda")
    slot = torch.empty(nu * n, dtype=torch.int32, device="cuda")
    main = torch.cuda.current_stream()
    streams = [main, torch.cuda.Stream()]
    streams[1].wait_stream(main)
    wss = [torch.full((kvs.kvs_workspace_size(p),), 0xFF, dtype=torch.uint8, device="cuda") for _ in streams]
    for c, st in enumerate(streams):
        u0, u1 = c * half, (c + 1) * half
        kvs.kvs_step(p, Q[u0:u1], K[u0 * n:u1 * n], V[u0 * n:u1 * n], K_out[u0 * B:u1 * B], V_out[u0 * B:u1 * B],
                     counts[u0 * B:u1 * B], wss[c], slot_of_token_out=slot[u0 * n:u1 * n],
                     edge_mask_out=mask[u0 * n:u1 * n], stream=st.cuda_stream)
    main.wait_stream(streams[1])
    torch_sync()
    # every unit: r edges selected, none in the sink, slots numbered 0 .. B-1, cardinalities add up to n
    m2, s2, c2 = mask.view(nu, n), slot.view(nu, n), counts.view(nu, B)
    assert (m2.sum(dim=1) == n - B).all()
    assert (m2[:, :w.n_sink] == 0).all() and (m2[:, -1] == 0).all()
    assert (s2[:, 0] == 0).all() and (s2[:, -1] == B - 1).all()
    assert (c2.sum(dim=1) == n).all() and (c2 >= 1).all()
    assert torch.isfinite(K_out.float()).all() and torch.isfinite(V_out.float()).all()
    m_host, s_host, c_host = m2.cpu().numpy(), s2.cpu().numpy(), c2.cpu().numpy()
    compared = 0
    for i, ref in enumerate(refs):
        if ref is None:
            continue
        r_mask, r_slot, r_counts, r_K, r_V, r_rows, gap = ref
        assert (m_host[i] == r_mask).all(), f"unit {i}: selected edges differ (gap {gap:.2e})"
        assert (s_host[i] == r_slot).all(), f"unit {i}: slot map differs"
        assert (c_host[i] == r_counts).all(), f"unit {i}: cardinalities differ"
        Ko, Vo = from_device(K_out[i * B:(i + 1) * B]), from_device(V_out[i * B:(i + 1) * B])
        ek, ev = rel_err_rows(Ko, r_K), rel_err_rows(Vo, r_V)
        assert ek <= TOL_KV["bf16"] and ev <= TOL_KV["bf16"], (i, ek, ev)
        single = r_rows == 1
        assert (Ko[single] == r_K[single]).all() and (Vo[single] == r_V[single]).all(), f"unit {i}: a single row is a copy"
        compared += 1
    assert compared == nu, f"{nu - compared} units had no accepted Query redraw"


def test_step_ragged_batch_reduced():
    """Ragged batch recipe (lengths and rho drawn per sequence) on 5 of the 16 sequences, 2 heads each, capped
    at 20000 tokens so the oracle finishes in seconds; more than 64 units are covered by the select test."""
    w = WORKLOADS["ragged16"]
    lens = unit_lengths(w)
    accepted = []
    for s in (0, 3, 7, 11, 15):
        n = min(lens[s], 20000 + 37 * s)
        for h in (0, 5):
            a = accepted_unit(w, 0, s, h, n=n)
            accepted.append(a)
    check_step(w, accepted)


def check_whole_batch_in_one_call(w, layer, sampled_ids):
    """Every (sequence, KV head) of a workload's layer as the units of ONE kvs_step call.  The units named in
    `sampled_ids` are accepted units and are compared with the oracle like any other; every unit must satisfy the
    invariants that hold at any size (r edges selected, none in the sink, consecutive slot numbers, cardinalities
    adding up)."""
    import torch
    from concurrent.futures import ThreadPoolExecutor
    import paper_2603_00907_amd as kvs
    D, R, H = w.head_dim, w.q_rows, w.n_kv_heads
    seq_lens = unit_lengths(w)
    ids = [(s, h) for s in range(w.n_seq) for h in range(H)]
    lens = [seq_lens[s] for s, _ in ids]
    budgets = [unit_budget(w, n) for n in lens]
    sampled = {sh: accepted_unit(w, layer, sh[0], sh[1]) for sh in sampled_ids}
    p = kvs.Problem(lens=lens, budgets=budgets, group=w.group, window=w.window, head_dim=D, dtype="bf16",
                    n_sink=w.n_sink, n_recent=w.n_recent)
    K = torch.empty((p.rows_in, D), dtype=torch.bfloat16, device="cuda")
    V = torch.empty_like(K)
    Q = torch.empty((len(ids), R, D), dtype=torch.bfloat16, device="cuda")

    def unit(sh):
        a = sampled.get(sh)
        return a.inputs if a is not None else generate_unit(w, layer, sh[0], sh[1])

    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
        for i, u in enumerate(pool.map(unit, ids)):
            r0 = p.in_rows[i]
            K[r0:r0 + lens[i]] = to_device(u.K, "bf16")
            V[r0:r0 + lens[i]] = to_device(u.V, "bf16")
            Q[i] = to_device(u.Q.reshape(R, D), "bf16")
    K_out = torch.empty((p.rows_out, D), dtype=torch.bfloat16, device="cuda")
    V_out = torch.empty_like(K_out)
    counts = torch.empty(p.rows_out, dtype=torch.int32, device="cuda")
    mask = torch.empty(p.rows_in, dtype=torch.uint8, device="cuda")
    slot = torch.empty(p.rows_in, dtype=torch.int32, device="cuda")
    ws = torch.full((kvs.kvs_workspace_size(p),), 0xFF, dtype=torch.uint8, device="cuda")
    kvs.kvs_step(p, Q, K, V, K_out, V_out, counts, ws, slot_of_token_out=slot, edge_mask_out=mask,
                 stream=torch.cuda.current_stream().cuda_stream)
    torch_sync()
    assert torch.isfinite(K_out.float()).all() and torch.isfinite(V_out.float()).all()
    mask_h, slot_h, counts_h = mask.cpu().numpy(), slot.cpu().numpy(), counts.cpu().numpy()
    for i, (n, B) in enumerate(zip(lens, budgets)):
        r0, o0 = p.in_rows[i], p.out_rows[i]
        m, s, c = mask_h[r0:r0 + n], slot_h[r0:r0 + n], counts_h[o0:o0 + B]
        assert m.sum() == n - B and not m[:w.n_sink].any() and m[-1] == 0, i
        assert s[0] == 0 and s[-1] == B - 1 and (np.diff(s) == 1 - m[:-1]).all(), i
        assert c.sum() == n and (c >= 1).all(), i
    for (sq, h), a in sampled.items():
        i = sq * H + h
        n, B, r0, o0 = lens[i], budgets[i], p.in_rows[i], p.out_rows[i]
        assert (mask_h[r0:r0 + n] == a.ref.mask).all(), f"unit {i}: selected edges differ (gap {a.gap:.2e})"
        assert (slot_h[r0:r0 + n] == a.ref.slot).all(), f"unit {i}: slot map differs"
        ref = a.ref.merged
        assert (counts_h[o0:o0 + B] == ref.counts).all()
        ek = rel_err_rows(from_device(K_out[o0:o0 + B]), ref.K_out)
        ev = rel_err_rows(from_device(V_out[o0:o0 + B]), ref.V_out)
        assert ek <= TOL_KV["bf16"] and ev <= TOL_KV["bf16"], (i, ek, ev)


def test_step_ragged_batch_full_size_in_one_call():
    """The ragged batch at its full size: 16 sequences of 4096..65536 tokens, 8 KV heads each, all 128 units in ONE
    kvs_step call (two launch groups, units longer than the select kernel's key cache among them).  Sampled for the
    oracle: the longest sequence, the shortest, the first unit of the second launch group."""
    w = WORKLOADS["ragged16"]
    seq_lens = unit_lengths(w)
    check_whole_batch_in_one_call(w, 0, [(int(np.argmax(seq_lens)), 3), (int(np.argmin(seq_lens)), 0), (8, 0)])


def test_step_stress_full_size_all_heads_in_one_call():
    """The stress configuration as it is benchmarked: 8 KV heads of 131072 tokens -> 8192 with 512 query rows
    (two launches of 256 rows per score sweep, the selection of units four times the key cache) in one call; head 0
    is compared with the oracle."""
    check_whole_batch_in_one_call(WORKLOADS["stress128k"], 0, [(0, 0)])


@pytest.mark.parametrize("group_units", [0, 64, 100, 7])
def test_step_more_units_than_the_kernel_arguments_hold(group_units):
    """150 short units of the headline shape (bf16, 128 query rows) in ONE call.  The library makes one launch group
    of them, whose unit descriptors go through the workspace (the kernel arguments hold 64); with the groups limited
    to 64 units there are three groups with descriptors in the arguments, with 100 one of each kind, with 7 many
    small ones.  Every unit is checked like any other; all four ways select the same edges and sum the same Values
    (the merged Keys agree to the tolerance: the score chunks follow the size of the call's first group, and with
    them the order in which a row's softmax sums are added)."""
    import torch
    w = WORKLOADS["llama8b_32k"].scaled(length=("fixed", 1500), budget=("fixed", 400))
    accepted = [accepted_unit(w, layer, 0, layer % w.n_kv_heads, n=1500 - 13 * (layer % 7)) for layer in range(150)]
    with switches(group_units=group_units):
        batch = check_step(w, accepted)
    if group_units:
        ref = check_step(w, accepted)
        assert torch.equal(batch.V_out.view(torch.int16), ref.V_out.view(torch.int16))
        assert torch.equal(batch.counts, ref.counts) and torch.equal(batch.slot, ref.slot)


def test_step_more_units_than_one_launch_group_takes():
    """1100 units of 40 to 167 rows (fp32, six query rows): more than the 1024 units a launch group may have, so two
    groups, both with their descriptors in the workspace, the second written over the first."""
    w = WORKLOADS["tiny"].scaled(group=2, window=3, length=("fixed", 167), budget=("fixed", 60), n_sink=4)
    accepted = [accepted_unit(w, i, 0, 0, n=40 + i % 128) for i in range(1100)]
    check_step(w, accepted)


@pytest.mark.parametrize("path", [None, "fuse", "onepass"])
def test_step_streaming_regime_full_size(path):
    """Sec. 5's streaming regime at full size: 8 KV heads, each a merged cache of 2048 + 512 slots (the old
    slots stand for 4 tokens on average) merged back to 2048; cardinalities must add up bit-exactly."""
    w = WORKLOADS["stream2560"]
    batch = check_step(w, [accepted_unit(w, 0, 0, h) for h in range(w.n_kv_heads)], path)
    total_in = sum(int(u.counts.sum()) for u in batch.units)
    assert int(batch.counts[:batch.problem.rows_out].sum().item()) == total_in


def test_step_streaming_regime_fp32_and_small_window():
    w = WORKLOADS["stream2560"].scaled(dtype="f32", head_dim=64, group=2, window=5, length=("fixed", 1500),
                                       budget=("fixed", 1100), fresh_tail=300, k_outlier_channels=0)
    check_step(w, [accepted_unit(w, 0, 0, h) for h in range(2)])


def test_counts_of_one_are_the_plain_step():
    """Cardinalities of one select the same edges and give the same cache as the plain entry point (the
    logits take one more rounding on that path, so merged rows agree to the tolerance, not bit for bit)."""
    import torch
    w = WORKLOADS["llama8b_8k"].scaled(length=("fixed", 3000), budget=("fixed", 800))
    acc = [accepted_unit(w, 0, 0, h) for h in range(2)]
    plain = run_step(w, acc)
    for a in acc:
        a.inputs.counts = np.ones(a.inputs.n, dtype=np.int32)
    ones = run_step(w, acc)
    for a in acc:
        a.inputs.counts = None
    assert torch.equal(plain.counts, ones.counts) and torch.equal(plain.slot, ones.slot)
    n_out = plain.problem.rows_out
    assert torch.equal(plain.V_out.view(torch.int16), ones.V_out.view(torch.int16))      # sums of the same rows
    assert rel_err_rows(from_device(ones.K_out)[:n_out], from_device(plain.K_out)[:n_out].astype(np.float64)) <= 1e-2


def test_step_stress_reduced():
    """Stress recipe (512 query rows, Student-t Values, rho 0.95) at 16384 tokens -> 1024, two heads."""
    w = WORKLOADS["stress128k"].scaled(length=("fixed", 16384), budget=("fixed", 1024))
    check_step(w, [accepted_unit(w, 0, 0, h) for h in range(2)])


def test_step_stress_full_size_one_head():
    """131072 tokens -> 8192 with 512 query rows, one KV head, full size."""
    w = WORKLOADS["stress128k"]
    check_step(w, [accepted_unit(w, 0, 0, 0)])


def test_step_passthrough_and_single_token_units():
    w = WORKLOADS["tiny"].scaled(n_seq=3)
    units = [generate_unit(w, 0, 0, 0, n=40), generate_unit(w, 0, 1, 0, n=1), generate_unit(w, 0, 2, 0, n=600)]
    units[0].budget, units[1].budget, units[2].budget = 64, 1, 600
    batch = DeviceBatch(units, group=w.group, window=w.window, head_dim=w.head_dim, dtype=w.dtype, n_sink=w.n_sink)
    batch.kvs.kvs_step(batch.problem, batch.Q, batch.K, batch.V, batch.K_out, batch.V_out, batch.counts, batch.ws,
                       slot_of_token_out=batch.slot, edge_mask_out=batch.mask, stream=batch.stream())
    torch_sync()
    batch.check_guards()
    Ko, Vo, cnt = from_device(batch.K_out), from_device(batch.V_out), batch.counts.cpu().numpy()
    for i, u in enumerate(units):
        r0 = batch.problem.out_rows[i]
        assert (Ko[r0:r0 + u.n] == u.K).all() and (Vo[r0:r0 + u.n] == u.V).all()
        assert (cnt[r0:r0 + u.n] == 1).all()


@pytest.mark.parametrize("dtype,D", [("bf16", 64), ("f32", 128)])
def test_step_at_the_maximum_length(dtype, D):
    """One unit of KVS_MAX_LEN = 2^22 rows (16 query rows) merged to a quarter: bf16 with head dim 64, and fp32 with
    head dim 128, the longest rows there are (512 bytes: the last row ends one byte short of 2^31).  At this length
    neighbouring edge scores at the budget boundary differ by less than fp32 resolves, so the selected set is not
    unique: it is checked for validity (the right number of edges, none of the selected scores above an
    unselected one beyond the tolerance of alpha_bar), slot map and cardinalities must follow from it exactly,
    merged Values are compared for every slot and merged Keys on windows the oracle merges with the same edges."""
    import torch
    import paper_2603_00907_amd as kvs
    from helpers import to_device
    from workloads import gaussian_unit
    n, G, W, n_sink = 1 << 22, 4, 4, 32
    B = n // 4
    Q, K, V = gaussian_unit(1, n, D, G, W, dtype)
    p = kvs.Problem(lens=[n], budgets=[B], group=G, window=W, head_dim=D, dtype=dtype, n_sink=n_sink)
    Kd, Vd, Qd = to_device(K, dtype), to_device(V, dtype), to_device(Q.reshape(1, G * W, D), dtype)
    K_out = torch.empty((B, D), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    V_out = torch.empty_like(K_out)
    counts = torch.empty(B, dtype=torch.int32, device="cuda")
    mask_d = torch.empty(n, dtype=torch.uint8, device="cuda")
    slot_d = torch.empty(n, dtype=torch.int32, device="cuda")
    ws = torch.full((kvs.kvs_workspace_size(p),), 0xFF, dtype=torch.uint8, device="cuda")
    kvs.kvs_step(p, Qd, Kd, Vd, K_out, V_out, counts, ws, slot_of_token_out=slot_d, edge_mask_out=mask_d,
                 stream=torch.cuda.current_stream().cuda_stream)
    torch_sync()
    mask, slot, cnt = mask_d.cpu().numpy(), slot_d.cpu().numpy(), counts.cpu().numpy()
    # the selection is a valid one
    alpha_bar, o_bar = O.score(Q, K, V)
    sigma = alpha_bar[:-1] + alpha_bar[1:]
    sel = mask[:-1] == 1
    assert sel.sum() == n - B and mask[-1] == 0 and not sel[:n_sink].any()
    assert sigma[sel].max() <= sigma[n_sink:][~sel[n_sink:]].min() * (1 + 4 * TOL_ALPHA)
    # slot map and cardinalities follow from the edges
    starts = np.ones(n, dtype=np.int64)
    starts[1:] = 1 - mask[:-1]
    assert (slot == np.cumsum(starts) - 1).all()
    first = np.flatnonzero(starts)
    assert len(first) == B
    assert (cnt == np.diff(np.append(first, n))).all()
    # every merged Value row is the sum of its run
    Vo = from_device(V_out)
    want_v = np.add.reduceat(V.astype(np.float64), first, axis=0)
    assert rel_err_rows(Vo, want_v) <= TOL_KV[dtype]
    # merged Keys on windows of whole slots: head of the cache, two places inside, the tail
    Ko = from_device(K_out)
    for s0 in (0, B // 3, (2 * B) // 3 + 7, B - 700):
        s1 = s0 + 700
        a, b = first[s0], (first[s1] if s1 < B else n)
        ref = O.merge_compact(K[a:b], V[a:b], alpha_bar[a:b], o_bar, mask[a:b] * (np.arange(a, b) < b - 1),
                              slot[a:b] - s0)
        assert (cnt[s0:s1] == ref.counts).all()
        assert rel_err_rows(Ko[s0:s1], ref.K_out) <= TOL_KV[dtype], s0
        single = ref.n_rows == 1
        assert (Ko[s0:s1][single] == ref.K_out[single]).all()


# ------------------------------------------------------------------------------------------------
# the consumer: decode attention over a (merged) cache
@pytest.mark.parametrize("base,dtype,D,G,W,lens,path", [
    ("tiny", "f32", 64, 1, 1, [1024], None),
    ("tiny", "f32", 128, 3, 2, [700, 41, 5000], None),
    ("llama8b_8k", "bf16", 128, 4, 1, [2048, 300], "mfma"),          # MFMA kernel, plain tokens
    ("llama8b_8k", "bf16", 128, 4, 1, [2048, 300], None),            # (four rows: the vector-ALU kernel)
    ("stream2560", "bf16", 128, 4, 1, [2560, 2049], "mfma"),         # with cardinalities; a chunk of one row
    ("stream2560", "bf16", 128, 4, 1, [2560, 2049], None),
    ("stream2560", "bf16", 64, 4, 3, [1111, 32, 33], None),          # head dim 64; units of one tile and one row more
    ("stream2560", "bf16", 64, 4, 3, [1111], "valu"),
    ("stream2560", "bf16", 128, 8, 5, [777], None),                  # 40 query rows: two blocks of 32
    ("stream2560", "bf16", 128, 8, 8, [40000], None),                # 64 query rows; chunks longer than 256 rows
    ("llama8b_8k", "bf16", 128, 4, 1, [500, 31], None),              # a unit below 32 rows: the vector-ALU kernel
    ("stream2560", "f32", 64, 2, 5, [2300], None),
])
def test_decode_attention_matches_oracle(base, dtype, D, G, W, lens, path):
    w = variant(base, dtype=dtype, head_dim=D, group=G, window=W, n_seq=len(lens), n_kv_heads=1)
    units = [generate_unit(w, 0, s, 0, n=n) for s, n in enumerate(lens)]
    check_decode(units, dtype, D, G, W, path)


@pytest.mark.parametrize("dtype,G,path", [("f32", 2, None), ("bf16", 8, "mfma"), ("bf16", 4, "valu")])
def test_decode_attention_more_units_than_the_kernel_arguments_hold(dtype, G, path):
    """130 caches of 33 to 400 rows in one call: one launch group whose unit descriptors live in the decode workspace."""
    lens = [33 + (53 * i) % 368 for i in range(130)]
    w = variant("stream2560", dtype=dtype, head_dim=128, group=G, window=1, n_seq=len(lens), n_kv_heads=1)
    w = w.scaled(fresh_tail=8, n_sink=2)
    units = [generate_unit(w, 0, s, 0, n=n) for s, n in enumerate(lens)]
    check_decode(units, dtype, 128, G, 1, path)


@pytest.mark.parametrize("dtype,G,path", [("f32", 2, None), ("bf16", 8, "mfma"), ("bf16", 2, "valu")])
def test_decode_attention_at_the_maximum_length(dtype, G, path):
    """A cache of KVS_MAX_LEN = 2^22 rows with head dim 128 (fp32: the longest rows there are), with cardinalities."""
    from workloads import gaussian_unit
    from workloads.generator import UnitInputs
    n, D = 1 << 22, 128
    Q, K, V = gaussian_unit(3, n, D, G, 1, dtype, k_scale=1.0)
    counts = np.random.default_rng(5).integers(1, 9, n).astype(np.int32)
    u = UnitInputs(layer=0, seq=0, head=0, attempt=0, n=n, budget=n, rho=0.0, Q=Q, K=K, V=V, counts=counts)
    check_decode([u], dtype, D, G, 1, path)


def check_decode(units, dtype, D, G, W, path):
    import torch
    lens = [u.n for u in units]
    batch = DeviceBatch(units, group=G, window=W, head_dim=D, dtype=dtype, n_sink=0, budgets=lens, gap_rows=2)
    p = batch.problem
    R = G * W
    out = torch.full((len(units) + 1, R, D), -7.0, dtype=torch.float32, device="cuda")
    ws = torch.full((batch.kvs.kvs_decode_workspace_size(p),), 0xFF, dtype=torch.uint8, device="cuda")
    with switch_override("decode_path", {None: 0, "valu": 1, "mfma": 2}[path]):
        batch.kvs.kvs_decode_attention(p, batch.Q, batch.K, batch.V, batch.counts_in, out, ws, stream=batch.stream())
        torch_sync()
    assert (out[len(units):] == -7.0).all()
    got = out.cpu().numpy()
    for i, u in enumerate(units):
        want = O.decode_attention(u.Q, u.K, u.V, u.counts)
        # every weight carries the relative error of a softmax weight; bound the sum term by term
        c = np.ones(u.n) if u.counts is None else u.counts
        alpha = O.attention_rows(u.Q, u.K, counts=c)                    # [R, n] masses of the rows
        bound = TOL_ALPHA * (alpha @ np.abs(O.slot_values(u.V, c))) + 1e-7
        assert np.isfinite(got[i]).all()
        assert (np.abs(got[i] - want) <= bound).all(), (i, np.max(np.abs(got[i] - want) / bound))


def test_decode_attention_over_the_output_of_a_step():
    """End to end: merge a cache, then attend over (K', V', counts) with fresh queries; the GPU result equals
    the oracle's attention over the oracle's merged cache (both within their tolerances)."""
    import torch
    w = WORKLOADS["llama8b_8k"].scaled(length=("fixed", 4000), budget=("fixed", 1000))
    acc = [accepted_unit(w, 0, 0, h) for h in range(2)]
    batch = check_step(w, acc)
    p = batch.problem
    rng = np.random.default_rng(5)
    G = w.group
    qn = rng.standard_normal((len(acc), G, 1, w.head_dim)).astype(np.float32)
    from workloads import bf16_bits_to_f32, f32_to_bf16_bits
    qn = bf16_bits_to_f32(f32_to_bf16_bits(qn)).reshape(qn.shape)
    dp = batch.kvs.Problem(lens=p.n_out, budgets=p.n_out, group=G, window=1, head_dim=w.head_dim, dtype=w.dtype,
                           n_sink=0, in_rows=p.out_rows)
    from helpers import to_device
    Qd = to_device(qn.reshape(len(acc), G, w.head_dim), w.dtype)
    out = torch.empty((len(acc), G, w.head_dim), dtype=torch.float32, device="cuda")
    ws = torch.full((batch.kvs.kvs_decode_workspace_size(dp),), 0xFF, dtype=torch.uint8, device="cuda")
    batch.kvs.kvs_decode_attention(dp, Qd, batch.K_out, batch.V_out, batch.counts, out, ws, stream=batch.stream())
    torch_sync()
    got = out.cpu().numpy()
    for i, a in enumerate(acc):
        m = a.ref.merged
        want = O.decode_attention(qn[i], m.K_out, m.V_out, m.counts)
        err = np.linalg.norm(got[i] - want, axis=1) / np.linalg.norm(want, axis=1)
        assert err.max() < 2e-2, err.max()       # the merged rows themselves carry the bf16 tolerance
