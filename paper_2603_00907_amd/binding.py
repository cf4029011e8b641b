"""ctypes binding of libkvs.so: argument marshalling only.

The functions carry the names of the C ABI (include/kvs.h) and take anything that
exposes `data_ptr()` (torch tensors on the GPU) or a raw integer address.  Nothing is
computed here; if the shared library is missing the import of this module's functions
fails loudly instead of falling back to anything else.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libkvs.so")

KVS_OK = 0
KVS_ERR_INVALID_ARG, KVS_ERR_DTYPE, KVS_ERR_BUDGET, KVS_ERR_WORKSPACE, KVS_ERR_ALIAS, KVS_ERR_DEVICE = range(1, 7)
KVS_F32, KVS_BF16 = 0, 1
DTYPES = {"f32": KVS_F32, "bf16": KVS_BF16}

EXPORTS = ["kvs_workspace_size", "kvs_score", "kvs_select", "kvs_merge_compact", "kvs_step",
           "kvs_score_counts", "kvs_merge_compact_counts", "kvs_step_counts", "kvs_decode_workspace_size",
           "kvs_decode_attention", "kvs_per_query_workspace_size", "kvs_sensitivity", "kvs_merge_compact_norms",
           "kvs_step_per_query", "kvs_sensitivity_counts", "kvs_merge_compact_norms_counts",
           "kvs_step_per_query_counts", "kvs_step_static", "kvs_status_str", "kvs_version", "kvs_debug_set",
           "kvs_debug_get"]

STATIC_SCRATCH_BYTES = 16 << 20
# testing switches of include/kvs_debug.h
DEBUG_SWITCHES = {"score_path": 0, "score_wide": 1, "fuse_obar": 2, "decode_path": 3, "score_chunk": 4, "verbose": 5,
                  "score_fused": 6, "select_split": 7, "fused_wait_us": 8, "fused_stagger": 9, "group_units": 10}


KEY_RULES = {"hessian": 0, "diagonal": 1, "mean": 2}


class KvsProblemStruct(C.Structure):
    _fields_ = [
        ("n_units", C.c_int32), ("group", C.c_int32), ("window", C.c_int32), ("head_dim", C.c_int32),
        ("n_sink", C.c_int32), ("n_recent", C.c_int32), ("io_dtype", C.c_int), ("scale", C.c_float),
        ("len", C.POINTER(C.c_int32)), ("budget", C.POINTER(C.c_int32)),
        ("in_row", C.POINTER(C.c_int64)), ("out_row", C.POINTER(C.c_int64)),
        ("key_rule", C.c_int), ("causal", C.c_int32),
    ]


class KvsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_str(status)} (kvs_status {status})")


_lib = None


def load_library(path: Optional[str] = None):
    """dlopen libkvs.so and declare the prototypes.  Raises if it has not been built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or os.environ.get("KVS_LIB") or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: build it with `python -m paper_2603_00907_amd.build` (hipcc, gfx950)")
    # The device pointers handed to the library come from PyTorch, so both must talk to ONE HIP runtime:
    # torch's.  torch bundles its own libamdhip64 under the same SONAME as the system's; whichever is
    # loaded first serves both, and with the system's loaded first the library's launches find no device.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(path)
    P, vp, sz = C.POINTER(KvsProblemStruct), C.c_void_p, C.c_size_t
    lib.kvs_workspace_size.argtypes = [P, C.POINTER(sz)]
    lib.kvs_score.argtypes = [P, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_select.argtypes = [P, vp, vp, vp, vp, sz, vp]
    lib.kvs_merge_compact.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_step.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_score_counts.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_merge_compact_counts.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_step_counts.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_decode_workspace_size.argtypes = [P, C.POINTER(sz)]
    lib.kvs_decode_attention.argtypes = [P, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_per_query_workspace_size.argtypes = [P, C.POINTER(sz)]
    lib.kvs_sensitivity.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_merge_compact_norms.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_step_per_query.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_sensitivity_counts.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_merge_compact_norms_counts.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_step_per_query_counts.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_step_static.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.kvs_debug_set.argtypes = [C.c_int, C.c_int]
    lib.kvs_debug_get.argtypes = [C.c_int]
    for name in ("kvs_workspace_size", "kvs_score", "kvs_select", "kvs_merge_compact", "kvs_step",
                 "kvs_score_counts", "kvs_merge_compact_counts", "kvs_step_counts", "kvs_decode_workspace_size",
                 "kvs_decode_attention", "kvs_per_query_workspace_size", "kvs_sensitivity",
                 "kvs_merge_compact_norms", "kvs_step_per_query", "kvs_sensitivity_counts",
                 "kvs_merge_compact_norms_counts", "kvs_step_per_query_counts", "kvs_step_static", "kvs_debug_set",
                 "kvs_debug_get"):
        getattr(lib, name).restype = C.c_int
    lib.kvs_status_str.argtypes = [C.c_int]
    lib.kvs_status_str.restype = C.c_char_p
    lib.kvs_version.argtypes = []
    lib.kvs_version.restype = C.c_int
    _lib = lib
    return lib


def status_str(status: int) -> str:
    return load_library().kvs_status_str(int(status)).decode()


def kvs_version() -> int:
    return int(load_library().kvs_version())


class Problem:
    """Host-side kvs_problem.  Keeps the arrays the struct points to alive."""

    def __init__(self, *, lens: Sequence[int], budgets: Sequence[int], group: int, window: int, head_dim: int,
                 dtype: str, n_sink: int = 32, n_recent: int = 0, scale: float = 0.0,
                 in_rows: Optional[Sequence[int]] = None, out_rows: Optional[Sequence[int]] = None,
                 key_rule=0, causal: bool = False):
        n = len(lens)
        if in_rows is None:
            in_rows, acc = [], 0
            for l in lens:
                in_rows.append(acc)
                acc += int(l)
        if out_rows is None:
            out_rows, acc = [], 0
            for l, b in zip(lens, budgets):
                out_rows.append(acc)
                acc += min(int(l), int(b))
        self.lens = [int(x) for x in lens]
        self.budgets = [int(x) for x in budgets]
        self.in_rows = [int(x) for x in in_rows]
        self.out_rows = [int(x) for x in out_rows]
        self.n_out = [min(l, b) for l, b in zip(self.lens, self.budgets)]
        self.rows_in = max(r + l for r, l in zip(self.in_rows, self.lens)) if n else 0
        self.rows_out = max(r + o for r, o in zip(self.out_rows, self.n_out)) if n else 0
        self._len = (C.c_int32 * n)(*self.lens)
        self._budget = (C.c_int32 * n)(*self.budgets)
        self._in = (C.c_int64 * n)(*self.in_rows)
        self._out = (C.c_int64 * n)(*self.out_rows)
        self.n_units = n
        self.group, self.window, self.head_dim, self.dtype = group, window, head_dim, dtype
        self.struct = KvsProblemStruct(
            n_units=n, group=group, window=window, head_dim=head_dim, n_sink=n_sink, n_recent=n_recent,
            io_dtype=DTYPES[dtype] if isinstance(dtype, str) else int(dtype), scale=float(scale),
            len=self._len, budget=self._budget, in_row=self._in, out_row=self._out,
            key_rule=KEY_RULES[key_rule] if isinstance(key_rule, str) else int(key_rule), causal=int(causal))

    @property
    def ref(self):
        return C.byref(self.struct)


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _nbytes(x) -> int:
    return int(x.numel() * x.element_size())


def _check(status: int, where: str):
    if status != KVS_OK:
        raise KvsError(status, where)


def kvs_workspace_size(problem: Problem) -> int:
    out = C.c_size_t(0)
    _check(load_library().kvs_workspace_size(problem.ref, C.byref(out)), "kvs_workspace_size")
    return int(out.value)


def kvs_score(problem: Problem, Q, K, V, alpha_bar, o_bar, ws, stream: int = 0, ws_bytes: Optional[int] = None):
    _check(load_library().kvs_score(problem.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(alpha_bar), _ptr(o_bar),
                                    _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes, stream), "kvs_score")


def kvs_select(problem: Problem, alpha_bar, edge_mask, slot_of_token, ws=None, stream: int = 0):
    _check(load_library().kvs_select(problem.ref, _ptr(alpha_bar), _ptr(edge_mask), _ptr(slot_of_token),
                                     _ptr(ws), _nbytes(ws) if ws is not None else 0, stream), "kvs_select")


def kvs_merge_compact(problem: Problem, K, V, alpha_bar, o_bar, edge_mask, slot_of_token, K_out, V_out, counts_out,
                      ws=None, stream: int = 0):
    _check(load_library().kvs_merge_compact(
        problem.ref, _ptr(K), _ptr(V), _ptr(alpha_bar), _ptr(o_bar), _ptr(edge_mask), _ptr(slot_of_token),
        _ptr(K_out), _ptr(V_out), _ptr(counts_out), _ptr(ws), _nbytes(ws) if ws is not None else 0, stream),
        "kvs_merge_compact")


def kvs_step(problem: Problem, Q, K, V, K_out, V_out, counts_out, ws, slot_of_token_out=None, edge_mask_out=None,
             stream: int = 0, ws_bytes: Optional[int] = None):
    _check(load_library().kvs_step(
        problem.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(K_out), _ptr(V_out), _ptr(counts_out),
        _ptr(slot_of_token_out), _ptr(edge_mask_out), _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes,
        stream), "kvs_step")


def kvs_score_counts(problem: Problem, Q, K, V, counts_in, alpha_bar, o_bar, ws, stream: int = 0,
                     ws_bytes: Optional[int] = None):
    _check(load_library().kvs_score_counts(
        problem.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(counts_in), _ptr(alpha_bar), _ptr(o_bar), _ptr(ws),
        _nbytes(ws) if ws_bytes is None else ws_bytes, stream), "kvs_score_counts")


def kvs_merge_compact_counts(problem: Problem, K, V, counts_in, alpha_bar, o_bar, edge_mask, slot_of_token, K_out,
                             V_out, counts_out, ws=None, stream: int = 0):
    _check(load_library().kvs_merge_compact_counts(
        problem.ref, _ptr(K), _ptr(V), _ptr(counts_in), _ptr(alpha_bar), _ptr(o_bar), _ptr(edge_mask),
        _ptr(slot_of_token), _ptr(K_out), _ptr(V_out), _ptr(counts_out), _ptr(ws),
        _nbytes(ws) if ws is not None else 0, stream), "kvs_merge_compact_counts")


def kvs_step_counts(problem: Problem, Q, K, V, counts_in, K_out, V_out, counts_out, ws, slot_of_token_out=None,
                    edge_mask_out=None, stream: int = 0, ws_bytes: Optional[int] = None):
    _check(load_library().kvs_step_counts(
        problem.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(counts_in), _ptr(K_out), _ptr(V_out), _ptr(counts_out),
        _ptr(slot_of_token_out), _ptr(edge_mask_out), _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes,
        stream), "kvs_step_counts")


def kvs_decode_workspace_size(problem: Problem) -> int:
    out = C.c_size_t(0)
    _check(load_library().kvs_decode_workspace_size(problem.ref, C.byref(out)), "kvs_decode_workspace_size")
    return int(out.value)


def kvs_decode_attention(problem: Problem, Q, K, V, counts, out, ws, stream: int = 0, ws_bytes: Optional[int] = None):
    _check(load_library().kvs_decode_attention(
        problem.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(counts), _ptr(out), _ptr(ws),
        _nbytes(ws) if ws_bytes is None else ws_bytes, stream), "kvs_decode_attention")


def kvs_per_query_workspace_size(problem: Problem) -> int:
    out = C.c_size_t(0)
    _check(load_library().kvs_per_query_workspace_size(problem.ref, C.byref(out)), "kvs_per_query_workspace_size")
    return int(out.value)


def kvs_sensitivity(problem: Problem, Q, K, V, alpha_bar, a_tok, c_edge, ws, stream: int = 0,
                    ws_bytes: Optional[int] = None):
    _check(load_library().kvs_sensitivity(
        problem.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(alpha_bar), _ptr(a_tok), _ptr(c_edge), _ptr(ws),
        _nbytes(ws) if ws_bytes is None else ws_bytes, stream), "kvs_sensitivity")


def kvs_sensitivity_counts(problem: Problem, Q, K, V, counts_in, alpha_bar, a_tok, c_edge, ws, stream: int = 0,
                           ws_bytes: Optional[int] = None):
    _check(load_library().kvs_sensitivity_counts(
        problem.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(counts_in), _ptr(alpha_bar), _ptr(a_tok), _ptr(c_edge), _ptr(ws),
        _nbytes(ws) if ws_bytes is None else ws_bytes, stream), "kvs_sensitivity_counts")


def kvs_merge_compact_norms(problem: Problem, K, V, a_tok, c_edge, edge_mask, slot_of_token, K_out, V_out,
                            counts_out, ws=None, stream: int = 0):
    _check(load_library().kvs_merge_compact_norms(
        problem.ref, _ptr(K), _ptr(V), _ptr(a_tok), _ptr(c_edge), _ptr(edge_mask), _ptr(slot_of_token),
        _ptr(K_out), _ptr(V_out), _ptr(counts_out), _ptr(ws), _nbytes(ws) if ws is not None else 0, stream),
        "kvs_merge_compact_norms")


def kvs_merge_compact_norms_counts(problem: Problem, K, V, counts_in, a_tok, c_edge, edge_mask, slot_of_token, K_out,
                                   V_out, counts_out, ws=None, stream: int = 0):
    _check(load_library().kvs_merge_compact_norms_counts(
        problem.ref, _ptr(K), _ptr(V), _ptr(counts_in), _ptr(a_tok), _ptr(c_edge), _ptr(edge_mask),
        _ptr(slot_of_token), _ptr(K_out), _ptr(V_out), _ptr(counts_out), _ptr(ws),
        _nbytes(ws) if ws is not None else 0, stream), "kvs_merge_compact_norms_counts")


def kvs_step_per_query_counts(problem: Problem, Q, K, V, counts_in, K_out, V_out, counts_out, ws,
                              slot_of_token_out=None, edge_mask_out=None, stream: int = 0,
                              ws_bytes: Optional[int] = None):
    _check(load_library().kvs_step_per_query_counts(
        problem.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(counts_in), _ptr(K_out), _ptr(V_out), _ptr(counts_out),
        _ptr(slot_of_token_out), _ptr(edge_mask_out), _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes,
        stream), "kvs_step_per_query_counts")


def kvs_step_per_query(problem: Problem, Q, K, V, K_out, V_out, counts_out, ws, slot_of_token_out=None,
                       edge_mask_out=None, stream: int = 0, ws_bytes: Optional[int] = None):
    _check(load_library().kvs_step_per_query(
        problem.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(K_out), _ptr(V_out), _ptr(counts_out),
        _ptr(slot_of_token_out), _ptr(edge_mask_out), _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes,
        stream), "kvs_step_per_query")


def kvs_step_static(problem: Problem, Q, K, V, counts_in, K_out, V_out, counts_out, slot_of_token_out=None,
                    edge_mask_out=None, stream: int = 0):
    _check(load_library().kvs_step_static(
        problem.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(counts_in), _ptr(K_out), _ptr(V_out), _ptr(counts_out),
        _ptr(slot_of_token_out), _ptr(edge_mask_out), stream), "kvs_step_static")


def kvs_debug_set(which, value: int) -> int:
    """Sets a testing switch (name from DEBUG_SWITCHES or its number); returns the previous value."""
    idx = DEBUG_SWITCHES[which] if isinstance(which, str) else int(which)
    return int(load_library().kvs_debug_set(idx, int(value)))


def kvs_debug_get(which) -> int:
    idx = DEBUG_SWITCHES[which] if isinstance(which, str) else int(which)
    return int(load_library().kvs_debug_get(idx))
