"""CPU-only checks of the C ABI: the library loads, exports what include/kvs.h declares, and every
argument error is reported on the host before anything is launched (so no GPU is needed here)."""

import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2603_00907_amd as kvs
from paper_2603_00907_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(kvs_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = kvs.load_library()
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None
    assert kvs.kvs_version() == 300
    assert kvs.status_str(kvs.KVS_OK) == "ok"
    for code in range(1, 7):
        assert kvs.status_str(code) not in ("ok", "unknown status")


def problem(**kw):
    base = dict(lens=[1024, 500], budgets=[512, 600], group=2, window=4, head_dim=64, dtype="f32")
    base.update(kw)
    return kvs.Problem(**base)


def status_of(fn, *a, **k):
    try:
        fn(*a, **k)
    except kvs.KvsError as e:
        return e.status
    return kvs.KVS_OK


def test_workspace_size_grows_with_the_problem():
    small = kvs.kvs_workspace_size(problem())
    big = kvs.kvs_workspace_size(problem(lens=[100000, 500]))
    assert small % 256 == 0 and big > small
    # pieces: chunk statistics, row normalisers, chunk o_bar, alpha_bar, o_bar, edge mask, slot map, and the
    # exchange area of the selection by several workgroups (6208 ints per unit of a launch)
    rows, nu, R, D = 1524, 2, 8, 64
    lower = nu * 64 * R * 8 + nu * R * 4 + nu * 64 * D * 4 + rows * 4 + nu * D * 4 + rows + rows * 4 + nu * 6208 * 4
    assert lower <= small <= lower + 8 * 256


@pytest.mark.parametrize("kw,want", [
    (dict(head_dim=96), kvs.KVS_ERR_INVALID_ARG),
    (dict(group=0), kvs.KVS_ERR_INVALID_ARG),
    (dict(group=64, window=32), kvs.KVS_ERR_INVALID_ARG),          # G*W above KVS_MAX_Q_ROWS
    (dict(lens=[0, 5]), kvs.KVS_ERR_INVALID_ARG),
    (dict(lens=[(1 << 22) + 1, 5], budgets=[1 << 21, 5]), kvs.KVS_ERR_INVALID_ARG),   # above KVS_MAX_LEN
    (dict(lens=[1 << 22, 5], budgets=[1 << 21, 5]), kvs.KVS_OK),
    (dict(n_sink=-1), kvs.KVS_ERR_INVALID_ARG),
    (dict(key_rule=3), kvs.KVS_ERR_INVALID_ARG),
    (dict(key_rule="mean"), kvs.KVS_OK),
    (dict(scale=float("nan")), kvs.KVS_ERR_INVALID_ARG),
    (dict(dtype=7), kvs.KVS_ERR_DTYPE),
    (dict(budgets=[20, 600]), kvs.KVS_ERR_BUDGET),                 # must merge but budget < n_sink + 1
    (dict(budgets=[32, 600], n_sink=30, n_recent=2), kvs.KVS_ERR_BUDGET),
    (dict(budgets=[0, 600]), kvs.KVS_ERR_BUDGET),
    (dict(in_rows=[0, 1000]), kvs.KVS_ERR_INVALID_ARG),            # input rows of the units overlap
    (dict(out_rows=[0, 100]), kvs.KVS_ERR_INVALID_ARG),            # output rows overlap
    (dict(budgets=[33, 600]), kvs.KVS_OK),
    (dict(budgets=[33, 600], n_recent=1), kvs.KVS_ERR_BUDGET),
])
def test_problem_validation(kw, want):
    assert status_of(kvs.kvs_workspace_size, problem(**kw)) == want


class FakeBuf:
    """An address range that is never dereferenced: validation happens before any launch."""

    def __init__(self, addr, nbytes):
        self.addr, self.nbytes = addr, nbytes

    def data_ptr(self):
        return self.addr

    def numel(self):
        return self.nbytes

    def element_size(self):
        return 1


def fake_buffers(p, D=64, elt=4):
    a = 1 << 30
    out = {}
    for name, nbytes in [("Q", len(p.lens) * p.group * p.window * D * elt), ("K", p.rows_in * D * elt),
                         ("V", p.rows_in * D * elt), ("K_out", p.rows_out * D * elt),
                         ("V_out", p.rows_out * D * elt), ("counts", p.rows_out * 4),
                         ("alpha", p.rows_in * 4), ("obar", len(p.lens) * D * 4), ("mask", p.rows_in),
                         ("slot", p.rows_in * 4), ("ws", kvs.kvs_workspace_size(p))]:
        out[name] = FakeBuf(a, nbytes)
        a += (nbytes + 4095) // 4096 * 4096
    return out


def test_pointer_workspace_and_alias_errors_are_host_side():
    p = problem()
    b = fake_buffers(p)
    step = lambda **o: status_of(  # noqa: E731
        kvs.kvs_step, p, o.get("Q", b["Q"]), o.get("K", b["K"]), o.get("V", b["V"]), o.get("K_out", b["K_out"]),
        o.get("V_out", b["V_out"]), o.get("counts", b["counts"]), o.get("ws", b["ws"]),
        slot_of_token_out=o.get("slot"), edge_mask_out=o.get("mask"), ws_bytes=o.get("ws_bytes"))
    assert step(K=None) == kvs.KVS_ERR_INVALID_ARG
    assert step(K=FakeBuf(b["K"].addr + 4, 16)) == kvs.KVS_ERR_INVALID_ARG           # misaligned
    assert step(ws=None, ws_bytes=0) == kvs.KVS_ERR_WORKSPACE
    assert step(ws=FakeBuf(b["ws"].addr + 16, b["ws"].nbytes)) == kvs.KVS_ERR_WORKSPACE
    assert step(ws_bytes=b["ws"].nbytes - 1) == kvs.KVS_ERR_WORKSPACE
    assert step(K_out=b["K"]) == kvs.KVS_ERR_ALIAS
    assert step(V_out=b["K_out"]) == kvs.KVS_ERR_ALIAS
    assert step(counts=FakeBuf(b["ws"].addr + 256, 64)) == kvs.KVS_ERR_ALIAS
    assert step(slot=b["V"]) == kvs.KVS_ERR_ALIAS
    assert step(mask=FakeBuf(b["K_out"].addr + 16, 64)) == kvs.KVS_ERR_ALIAS
    # inputs may alias each other (K used as V is legal, if odd)
    bad = status_of(kvs.kvs_score, p, b["Q"], b["K"], b["K"], b["alpha"], b["K"], b["ws"])
    assert bad == kvs.KVS_ERR_ALIAS
    assert status_of(kvs.kvs_select, p, b["alpha"], b["alpha"], b["slot"]) == kvs.KVS_ERR_ALIAS
    assert status_of(kvs.kvs_merge_compact, p, b["K"], b["V"], b["alpha"], b["obar"], b["mask"], b["slot"],
                     b["K_out"], b["K_out"], b["counts"]) == kvs.KVS_ERR_ALIAS
    assert status_of(kvs.kvs_merge_compact, p, b["K"], b["V"], b["alpha"], b["obar"], None, b["slot"],
                     b["K_out"], b["V_out"], b["counts"]) == kvs.KVS_ERR_INVALID_ARG


def test_static_entry_refuses_large_problems_and_bad_pointers_before_any_device_call():
    """kvs_step_static brings its own workspace of KVS_STATIC_SCRATCH_BYTES: a problem that needs more is refused,
    and so is every pointer error, on the host (no GPU is touched before those checks)."""
    p = problem()
    b = fake_buffers(p)
    assert kvs.kvs_workspace_size(p) <= kvs.STATIC_SCRATCH_BYTES
    st = lambda pr=p, **o: status_of(  # noqa: E731
        kvs.kvs_step_static, pr, b["Q"], o.get("K", b["K"]), b["V"], None, o.get("K_out", b["K_out"]), b["V_out"],
        b["counts"])
    assert st(K=None) == kvs.KVS_ERR_INVALID_ARG
    assert st(K_out=b["V"]) == kvs.KVS_ERR_ALIAS
    big = problem(lens=[2_000_000, 500], budgets=[1_000_000, 600])
    assert kvs.kvs_workspace_size(big) > kvs.STATIC_SCRATCH_BYTES
    assert st(big) == kvs.KVS_ERR_WORKSPACE
    header = open(os.path.join(ROOT, "include", "kvs.h")).read()
    assert re.search(r"#define KVS_STATIC_SCRATCH_BYTES \(16u << 20\)", header) and kvs.STATIC_SCRATCH_BYTES == 16 << 20


def test_debug_switches_are_process_state_without_environment_lookups():
    for name, idx in kvs.DEBUG_SWITCHES.items():
        old = kvs.kvs_debug_get(name)
        assert old >= 0
        assert kvs.kvs_debug_set(name, 2) == old and kvs.kvs_debug_get(idx) == 2
        assert kvs.kvs_debug_set(name, old) == 2
    assert kvs.kvs_debug_set(len(kvs.DEBUG_SWITCHES), 1) == -1          # unknown switch
    assert kvs.kvs_debug_set("verbose", -3) == -1 and kvs.kvs_debug_get(99) == -1
    # the environment is read when the library is loaded, not by the calls
    os.environ["KVS_SCORE_PATH"] = "valu"
    try:
        assert kvs.kvs_debug_get("score_path") == 0
    finally:
        del os.environ["KVS_SCORE_PATH"]
    for src in os.listdir(os.path.join(ROOT, "paper_2603_00907_amd", "csrc")):
        text = open(os.path.join(ROOT, "paper_2603_00907_amd", "csrc", src)).read()
        assert "getenv" not in text or src == "kvs_api.hip", src


def test_null_problem_and_null_tables():
    lib = kvs.load_library()
    out = C.c_size_t(0)
    assert lib.kvs_workspace_size(None, C.byref(out)) == kvs.KVS_ERR_INVALID_ARG
    p = problem()
    assert lib.kvs_workspace_size(p.ref, None) == kvs.KVS_ERR_INVALID_ARG
    p.struct.len = None
    assert lib.kvs_workspace_size(p.ref, C.byref(out)) == kvs.KVS_ERR_INVALID_ARG


def test_generator_is_order_independent_and_rounds_once():
    from workloads import WORKLOADS, bf16_bits_to_f32, f32_to_bf16_bits, generate_unit
    w = WORKLOADS["llama8b_8k"].scaled(length=("fixed", 300))
    a = generate_unit(w, 0, 0, 3)
    _ = generate_unit(w, 0, 0, 1)
    b = generate_unit(w, 0, 0, 3)
    assert (a.K == b.K).all() and (a.V == b.V).all() and (a.Q == b.Q).all()
    c = generate_unit(w, 0, 0, 3, attempt=1, kv_from=a)
    assert (c.K == a.K).all() and not (c.Q == a.Q).all()
    assert (bf16_bits_to_f32(f32_to_bf16_bits(a.K)) == a.K).all()           # already representable
    # round-to-nearest-even on a tie
    x = np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8], dtype=np.float32)
    assert bf16_bits_to_f32(f32_to_bf16_bits(x)).tolist() == [1.0, 1.0 + 2 ** -6]
    # four outlier channels, scaled 8x
    var = a.K.var(axis=0)
    assert (var > 20 * np.median(var)).sum() == 4


def test_decode_and_counts_entry_points_validate_on_the_host():
    p = problem()
    b = fake_buffers(p)
    dws = FakeBuf(b["ws"].addr, kvs.kvs_decode_workspace_size(p))
    out = FakeBuf(1 << 40, len(p.lens) * p.group * p.window * 64 * 4)
    cin = FakeBuf((1 << 40) + (1 << 30), p.rows_in * 4)
    dec = lambda **o: status_of(  # noqa: E731
        kvs.kvs_decode_attention, p, o.get("Q", b["Q"]), b["K"], b["V"], o.get("counts", cin), o.get("out", out),
        o.get("ws", dws), ws_bytes=o.get("ws_bytes"))
    assert dec(Q=None) == kvs.KVS_ERR_INVALID_ARG
    assert dec(out=b["K"]) == kvs.KVS_ERR_ALIAS
    assert dec(ws_bytes=dws.nbytes - 1) == kvs.KVS_ERR_WORKSPACE
    assert dec(counts=FakeBuf(cin.addr + 2, 16)) == kvs.KVS_ERR_INVALID_ARG          # misaligned
    wide = problem(group=9, window=8)                                                # 72 rows > KVS_MAX_DECODE_ROWS
    assert status_of(kvs.kvs_decode_workspace_size, wide) == kvs.KVS_ERR_INVALID_ARG
    # cardinalities that overlap an output are an alias error like any other input
    assert status_of(kvs.kvs_step_counts, p, b["Q"], b["K"], b["V"], b["K_out"], b["K_out"], b["V_out"], b["counts"],
                     b["ws"]) == kvs.KVS_ERR_ALIAS


def test_per_query_entry_points_validate_on_the_host():
    assert status_of(kvs.kvs_per_query_workspace_size, problem()) == kvs.KVS_OK                 # fp32: any length
    assert status_of(kvs.kvs_per_query_workspace_size, problem(lens=[1024, 31], budgets=[512, 31])) == kvs.KVS_OK
    assert status_of(kvs.kvs_per_query_workspace_size,
                     problem(dtype="bf16", lens=[1024, 31], budgets=[512, 31])) == kvs.KVS_ERR_INVALID_ARG
    assert kvs.kvs_per_query_workspace_size(problem()) > kvs.kvs_workspace_size(problem())
    p = problem(dtype="bf16")
    need = kvs.kvs_per_query_workspace_size(p)
    assert need % 256 == 0 and need > kvs.kvs_workspace_size(p)
    b = fake_buffers(p, elt=2)
    ws = FakeBuf(b["ws"].addr, need)
    a_tok = FakeBuf(1 << 40, p.rows_in * 4)
    c_edge = FakeBuf((1 << 40) + (1 << 30), p.rows_in * 4)
    sens = lambda **o: status_of(  # noqa: E731
        kvs.kvs_sensitivity, p, b["Q"], o.get("K", b["K"]), b["V"], b["alpha"], o.get("a_tok", a_tok), c_edge,
        o.get("ws", ws), ws_bytes=o.get("ws_bytes"))
    assert sens(K=None) == kvs.KVS_ERR_INVALID_ARG
    assert sens(a_tok=c_edge) == kvs.KVS_ERR_ALIAS
    assert sens(ws_bytes=need - 256) == kvs.KVS_ERR_WORKSPACE
    assert sens(ws=FakeBuf(ws.addr + 16, need)) == kvs.KVS_ERR_WORKSPACE
    step = lambda **o: status_of(  # noqa: E731
        kvs.kvs_step_per_query, p, b["Q"], b["K"], b["V"], o.get("K_out", b["K_out"]), b["V_out"], b["counts"],
        o.get("ws", ws), ws_bytes=o.get("ws_bytes"))
    assert step(K_out=b["V"]) == kvs.KVS_ERR_ALIAS
    assert step(ws_bytes=kvs.kvs_workspace_size(p)) == kvs.KVS_ERR_WORKSPACE
    norms = lambda **o: status_of(  # noqa: E731
        kvs.kvs_merge_compact_norms, p, b["K"], b["V"], o.get("a_tok", a_tok), c_edge, b["mask"], b["slot"],
        b["K_out"], o.get("V_out", b["V_out"]), b["counts"])
    assert norms(a_tok=None) == kvs.KVS_ERR_INVALID_ARG
    assert norms(V_out=b["K_out"]) == kvs.KVS_ERR_ALIAS


def test_causal_flag_is_validated_on_the_host():
    assert status_of(kvs.kvs_workspace_size, problem(causal=True)) == kvs.KVS_OK
    assert status_of(kvs.kvs_workspace_size, problem(causal=2)) == kvs.KVS_ERR_INVALID_ARG
    # the window's own rows are part of the cache: a unit shorter than the window cannot be masked
    assert status_of(kvs.kvs_workspace_size, problem(causal=True, lens=[1024, 3], budgets=[512, 3])) \
        == kvs.KVS_ERR_INVALID_ARG
    assert status_of(kvs.kvs_workspace_size, problem(lens=[1024, 3], budgets=[512, 3])) == kvs.KVS_OK


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; any other --gpus value ends with a message and a non-zero status before
    anything touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
