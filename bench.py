#!/usr/bin/env python3
"""Benchmark of the merge step on the headline workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama8b_32k]

One *step* is one pass of the whole hot path (score -> select -> merge_compact) over every layer of
the workload, inputs resident in HBM.  A (layer, sequence, KV head) cache is one independent unit of
the library, so the layers are simply more units of the same kvs_step call (--layers-per-call, all of
them by default; the library launches its kernels over groups of units: 64 of the headline's).
Prints ONE JSON line: whole-job merged KV tokens/s, the roofline of the whole step (with the phases' and the
dominant kernel's own figures as flat fields beside it, timed live with events on the launch stream) and the
fp64 oracle's rate on the host cores of this machine.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth


def launch_groups(lens):
    """The units (cache lengths, in call order) that each launch of the library covers: 64 units, and more as long
    as they have fewer than 2 M tokens (64 units of 32768), up to 1024 units.  Returns the groups' sizes."""
    groups, count, tokens = [], 0, 0
    for n in lens:
        count += 1
        tokens += n
        if (count >= 64 and tokens >= 64 * 32768) or count == 1024:
            groups.append(count)
            count = tokens = 0
    if count:
        groups.append(count)
    return groups


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama8b_32k")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (0 = workload's)")
    ap.add_argument("--layers-per-call", type=int, default=0,
                    help="layers handed to one kvs_step call (0 = all; 1 = one call per layer)")
    ap.add_argument("--streams", type=int, default=None,
                    help="deal the kvs_step calls of a step round-robin to this many streams (default 2: the layers go "
                         "to two calls on two streams, whose kernels fill each other's idle resources; 1 when all units "
                         "of the step fit ONE launch of the library, which then beats two half-size calls)")
    ap.add_argument("--no-per-layer-calls", action="store_true", help="skip the one-call-per-layer comparison loop")
    ap.add_argument("--io-dtype", default=None, choices=["bf16", "f32"],
                    help="run the workload's recipe with this I/O dtype instead of its own (fp32: the fp32 kernels at size)")
    ap.add_argument("--key-rule", default="hessian", choices=["hessian", "diagonal", "mean"],
                    help="rule for the merged Key (the ablations run the same kernels)")
    ap.add_argument("--decode", action="store_true",
                    help="also time kvs_decode_attention (one new query per query head) over the merged caches")
    ap.add_argument("--per-query", action="store_true",
                    help="also time the step with per-query aggregation of the norms (kvs_step_per_query, bf16 only)")
    ap.add_argument("--one-pass-score", action="store_true",
                    help="take the one-pass score kernel (K kept in LDS between its phases) where it applies; the library "
                         "does not pick it by itself (measured slower than the two sweeps)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true", help="replay the step from a HIP graph instead of launching from the host")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (known HBM bytes) for scaling rocprofv3 byte counters")
    return ap.parse_args()


def phase_bytes(n, B, R, D, b, with_counts=False):
    """Algorithmic HBM bytes of one unit, per phase (each tensor counted once per phase that needs it)."""
    c = 4 * n if with_counts else 0                            # input cardinalities (streaming regime)
    score = 2 * n * D * b + R * D * b + 4 * n + 4 * D + c      # read K, V, Q; write alpha_bar, o_bar
    select = 4 * n + n + 4 * n                                 # read alpha_bar; write edge mask, slot map
    merge = 2 * n * D * b + 9 * n + 4 * D + 2 * B * D * b + 4 * B + c   # read K, V, alpha, mask, slot, o_bar; write K', V', counts
    return {"score": score, "select": select, "merge_compact": merge}


def measured_traffic(workload):
    """HBM-side bytes per launch of each phase, from the committed rocprofv3 counter summary (None if absent)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    try:
        for line in open(path):
            if line.startswith("bench-traffic-bytes-per-launch:"):
                return {k: float(v) for k, v in (kv.split("=") for kv in line.split(":", 1)[1].split())}
    except OSError:
        pass
    return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (units are independent: more GPUs would each take a share "
              "of the KV heads, with nothing to exchange); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2603_00907_amd as kvs
    from workloads import WORKLOADS, f32_to_bf16_bits, generate_unit, unit_budget, unit_lengths

    kvs.load_library()
    if args.one_pass_score:
        kvs.kvs_debug_set("score_fused", 2)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    w = WORKLOADS[args.workload]
    if args.io_dtype and args.io_dtype != w.dtype:
        w = w.scaled(dtype=args.io_dtype)
    layers = args.layers or w.layers
    lens_seq = unit_lengths(w)
    lens = [lens_seq[s] for s in range(w.n_seq) for _ in range(w.n_kv_heads)]       # the units of one layer
    budgets = [unit_budget(w, n) for n in lens]
    D, R = w.head_dim, w.q_rows
    b = 4 if w.dtype == "f32" else 2
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    if args.streams is None:
        args.streams = 1 if len(launch_groups(lens * layers)) == 1 else 2
    # launch shape: by default the layers are split evenly into one kvs_step call per stream
    lpc = args.layers_per_call or -(-layers // max(1, min(args.streams, layers)))
    batches = [list(range(l0, min(layers, l0 + lpc))) for l0 in range(0, layers, lpc)]
    problems = {}
    for nl in {len(bt) for bt in batches}:
        problems[nl] = kvs.Problem(lens=lens * nl, budgets=budgets * nl, group=w.group, window=w.window, head_dim=D,
                                   dtype=w.dtype, n_sink=w.n_sink, n_recent=w.n_recent, key_rule=args.key_rule)
    rows_layer = sum(lens)

    # ---- synthetic inputs, one independent draw per (layer, sequence, head), uploaded once
    t_gen = time.time()
    workers = min(16, os.cpu_count() or 1)
    keep_host = {}                     # units kept on the host for the oracle sample
    n_keep_layers = 0 if args.no_cpu_baseline else layers       # fp32 copies on the host, 34 MB per unit

    def upload(x32):
        if w.dtype == "f32":
            return torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).to(dev)
        return torch.from_numpy(f32_to_bf16_bits(x32).view(np.int16)).to(dev).view(torch.bfloat16)

    Ks, Vs, Qs, Cs = [], [], [], []    # one tensor per batch of layers (Cs: row cardinalities or None)
    with ThreadPoolExecutor(max_workers=workers) as pool:
        for bt in batches:
            Kb = torch.empty((rows_layer * len(bt), D), dtype=tdt, device=dev)
            Vb = torch.empty_like(Kb)
            Qb = torch.empty((len(lens) * len(bt), R, D), dtype=tdt, device=dev)
            Cb = torch.ones(rows_layer * len(bt), dtype=torch.int32, device=dev) if w.mean_count > 0 else None
            for i, layer in enumerate(bt):
                ids = [(s, h) for s in range(w.n_seq) for h in range(w.n_kv_heads)]
                units = list(pool.map(lambda sh: generate_unit(w, layer, sh[0], sh[1]), ids))
                Kb[i * rows_layer:(i + 1) * rows_layer] = upload(np.concatenate([u.K for u in units]))
                Vb[i * rows_layer:(i + 1) * rows_layer] = upload(np.concatenate([u.V for u in units]))
                Qb[i * len(lens):(i + 1) * len(lens)] = upload(np.stack([u.Q.reshape(R, D) for u in units]))
                if Cb is not None:
                    Cb[i * rows_layer:(i + 1) * rows_layer] = torch.from_numpy(np.concatenate([u.counts for u in units])).to(dev)
                if layer < n_keep_layers:
                    keep_host[layer] = units
            Ks.append(Kb)
            Vs.append(Vb)
            Qs.append(Qb)
            Cs.append(Cb)
    t_gen = time.time() - t_gen

    probs = [problems[len(bt)] for bt in batches]
    K_out = [torch.empty((pr.rows_out, D), dtype=tdt, device=dev) for pr in probs]
    V_out = [torch.empty((pr.rows_out, D), dtype=tdt, device=dev) for pr in probs]
    counts = [torch.empty(pr.rows_out, dtype=torch.int32, device=dev) for pr in probs]
    big = probs[0]                                               # the first batch is the largest
    ws = torch.empty(kvs.kvs_workspace_size(big), dtype=torch.uint8, device=dev)
    alpha = torch.empty(big.rows_in, dtype=torch.float32, device=dev)
    obar = torch.empty((big.n_units, D), dtype=torch.float32, device=dev)
    mask = torch.empty(big.rows_in, dtype=torch.uint8, device=dev)
    slot = torch.empty(big.rows_in, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream

    n_streams = 1 if args.graph else max(1, min(args.streams, len(batches)))
    side_streams = [torch.cuda.Stream() for _ in range(n_streams - 1)]
    wss = [ws] + [torch.empty_like(ws) for _ in side_streams]

    def one_step():
        if n_streams == 1:
            for i, pr in enumerate(probs):
                kvs.kvs_step_counts(pr, Qs[i], Ks[i], Vs[i], Cs[i], K_out[i], V_out[i], counts[i], ws, stream=stream)
            return
        # calls dealt round-robin to several streams (each with its own workspace): independent calls overlap
        main = torch.cuda.current_stream()
        for st in side_streams:
            st.wait_stream(main)
        for i, pr in enumerate(probs):
            j = i % n_streams
            sj = stream if j == 0 else side_streams[j - 1].cuda_stream
            kvs.kvs_step_counts(pr, Qs[i], Ks[i], Vs[i], Cs[i], K_out[i], V_out[i], counts[i], wss[j], stream=sj)
        for st in side_streams:
            main.wait_stream(st)

    # Optionally the launches of one step (4 kernels per layer) are captured once into a HIP graph and
    # replayed: the library never allocates, synchronises or memsets, so a step is capturable as it is.
    # (Measured: no gain here, the kernels are long enough for the host to run ahead.)
    run_step = one_step
    graph = None
    if args.graph:
        one_step()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            stream = side.cuda_stream
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                one_step()
        torch.cuda.current_stream().wait_stream(side)
        stream = torch.cuda.current_stream().cuda_stream
        run_step = graph.replay

    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        run_step()
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = ev0.elapsed_time(ev1)
    ms_per_step = max(wall_ms, gpu_ms) / args.steps
    tokens_per_step = layers * sum(lens_seq)          # one token = the K and V rows of all KV heads at one position
    value = tokens_per_step / (ms_per_step * 1e-3)

    # ---- for comparison: the same step as one kvs_step call per layer, layer after layer on the same stream
    seq_ms = None
    if lpc != 1 and not args.graph and not args.no_per_layer_calls:
        one = kvs.Problem(lens=lens, budgets=budgets, group=w.group, window=w.window, head_dim=D, dtype=w.dtype,
                          n_sink=w.n_sink, n_recent=w.n_recent, key_rule=args.key_rule)
        nu = len(lens)

        def layer_calls():
            for i, bt in enumerate(batches):
                for j in range(len(bt)):
                    r0, r1, o0, o1 = j * rows_layer, (j + 1) * rows_layer, j * one.rows_out, (j + 1) * one.rows_out
                    kvs.kvs_step_counts(one, Qs[i][j * nu:(j + 1) * nu], Ks[i][r0:r1], Vs[i][r0:r1],
                                        None if Cs[i] is None else Cs[i][r0:r1], K_out[i][o0:o1], V_out[i][o0:o1],
                                        counts[i][o0:o1], ws, stream=stream)

        layer_calls()
        torch.cuda.synchronize()
        n_rep = max(1, min(args.steps, 5))
        ev0.record()
        for _ in range(n_rep):
            layer_calls()
        ev1.record()
        torch.cuda.synchronize()
        seq_ms = ev0.elapsed_time(ev1) / n_rep

    # ---- per-phase timing, same inputs, the three entry points one after the other with events between
    phases = ["score", "select", "merge_compact"]
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in probs]
    reps = max(1, min(args.steps, 5))
    phase_ms = {p: 0.0 for p in phases}
    for rep in range(reps + 1):
        for i, pr in enumerate(probs):
            evs[i][0].record()
            kvs.kvs_score_counts(pr, Qs[i], Ks[i], Vs[i], Cs[i], alpha, obar, ws, stream=stream)
            evs[i][1].record()
            kvs.kvs_select(pr, alpha, mask, slot, ws=ws, stream=stream)    # (with the workspace, as inside kvs_step)
            evs[i][2].record()
            kvs.kvs_merge_compact_counts(pr, Ks[i], Vs[i], Cs[i], alpha, obar, mask, slot, K_out[i], V_out[i], counts[i],
                                         ws=ws, stream=stream)
            evs[i][3].record()
        torch.cuda.synchronize()
        if rep == 0:
            continue                                   # warm-up of the stand-alone entry points
        for i in range(len(probs)):
            for j, p in enumerate(phases):
                phase_ms[p] += evs[i][j].elapsed_time(evs[i][j + 1])
    # One kernel launch of the library covers one group of units (64 of the headline's; all 256 caches of the
    # streaming workload); the figures below are per such launch.
    groups = [g for bt in batches for g in launch_groups(lens * len(bt))]
    UNITS_PER_LAUNCH = max(groups)
    launches = reps * len(groups)
    layers_per_launch = layers * reps / launches
    phase_ms = {p: v / launches for p, v in phase_ms.items()}
    pb = {p: 0 for p in phases}                       # bytes of one layer's units
    for n, B in zip(lens, budgets):
        for p, v in phase_bytes(n, min(n, B), R, D, b, w.mean_count > 0).items():
            pb[p] += v
    step_bytes = sum(pb.values())
    pb = {p: v * layers_per_launch for p, v in pb.items()}     # ... of one launch's units
    # The dominant KERNEL of the path is merge_kernel (kvs_merge_compact is exactly that kernel; kvs_score runs
    # two sweeps and two small kernels, each shorter than it): its algorithmic bytes over its launch time, timed
    # live above.  The roofline object's own figures are those of the WHOLE STEP (what the target is stated on).
    kernel = "merge_compact"
    kernel_gbs = pb[kernel] / (phase_ms[kernel] * 1e-3) / 1e9
    step_gbs = step_bytes * layers / (ms_per_step * 1e-3) / 1e9
    frac = {p: pb[p] / (phase_ms[p] * 1e-3) / 1e9 / HBM_PEAK_GBS for p in phases}
    traffic = measured_traffic(w.name)                 # per launch of 64 units, from the committed counter summary
    traffic_step = None if traffic is None else sum(traffic.values()) / 8.0        # per layer of 8 units
    flops_score = 2 * 2.0 * R * D * sum(lens)          # both sweeps' Q K^T products, one layer
    mfma_peak = 2500.0 if w.dtype == "bf16" else 157.3

    result = {
        "metric": ("merged KV tokens/s and achieved HBM GB/s (% of peak), 8B-shape 32K merge step"
                   if w.name == "llama8b_32k" else f"merged KV cache rows/s and achieved HBM GB/s (% of peak), {w.name}"),
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "layers": layers, "kv_heads": w.n_kv_heads, "q_heads": w.group * w.n_kv_heads,
                   "head_dim": D, "window": w.window, "tokens": lens_seq if w.n_seq > 1 else lens_seq[0],
                   "budget": budgets[0] if w.n_seq == 1 else "25% of length", "n_sink": w.n_sink,
                   "key_rule": args.key_rule, "io_dtype": w.dtype, "accumulate": "f32", "layers_per_call": lpc,
                   "streams": n_streams, "launch": "hip graph replay" if args.graph else "host",
                   "score_kernels": "one pass" if args.one_pass_score else "two sweeps",
                   "us_per_layer": ms_per_step * 1e3 / layers,
                   "us_per_layer_one_call_per_layer": None if seq_ms is None else seq_ms * 1e3 / layers,
                   "value_one_call_per_layer": None if seq_ms is None else tokens_per_step / (seq_ms * 1e-3),
                   "input_generation_s": round(t_gen, 1)},
        # scope "step": algorithmic bytes of score + select + merge_compact of all layers over the timed step
        "roofline": {"bound": "hbm", "scope": "step", "achieved": step_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": step_gbs / HBM_PEAK_GBS, "target_frac": 0.60,
                     "traffic": traffic_step, "traffic_source": "committed rocprofv3 counter summary under profiles/"
                     if traffic else None,
                     "algorithmic_bytes_per_layer": step_bytes, "step_frac": step_gbs / HBM_PEAK_GBS,
                     "kernel": "merge_kernel (kvs_merge_compact)", "kernel_achieved": kernel_gbs,
                     "kernel_frac": kernel_gbs / HBM_PEAK_GBS, "kernel_us_per_launch": phase_ms[kernel] * 1e3,
                     "kernel_algorithmic_bytes_per_launch": pb[kernel],
                     "kernel_traffic": (traffic or {}).get(kernel),
                     "units_per_launch": min(UNITS_PER_LAUNCH, big.n_units),
                     "score_us_per_launch": phase_ms["score"] * 1e3, "select_us_per_launch": phase_ms["select"] * 1e3,
                     "merge_compact_us_per_launch": phase_ms["merge_compact"] * 1e3,
                     "score_frac": frac["score"], "select_frac": frac["select"], "merge_compact_frac": frac["merge_compact"],
                     "score_traffic_ratio": None if traffic is None else traffic["score"] / pb["score"],
                     "merge_compact_traffic_ratio": None if traffic is None else traffic["merge_compact"] / pb["merge_compact"],
                     # the score phase's matrix work against the dense MFMA peak of its dtype (it matters for windows
                     # of several hundred rows: the stress configuration)
                     "score_mfma_frac": flops_score * layers_per_launch / (phase_ms["score"] * 1e-3) / 1e12 / mfma_peak},
    }

    if args.decode:
        # the consumer: every query head's next query attends over its KV head's merged cache (K', V', counts)
        dec = {}
        t_ms, nbytes = 0.0, 0
        reps = max(1, min(args.steps, 5))
        for i, pr in enumerate(probs):
            dp = kvs.Problem(lens=pr.n_out, budgets=pr.n_out, group=w.group, window=1, head_dim=D, dtype=w.dtype,
                             n_sink=0, in_rows=pr.out_rows)
            Qd = Qs[i][:, :w.group].contiguous()                     # [units, G, D]: one row per query head
            out = torch.empty((dp.n_units, w.group, D), dtype=torch.float32, device=dev)
            dws = torch.empty(kvs.kvs_decode_workspace_size(dp), dtype=torch.uint8, device=dev)
            for rep in range(reps + 1):
                if rep == 1:
                    ev0.record()
                kvs.kvs_decode_attention(dp, Qd, K_out[i], V_out[i], counts[i], out, dws, stream=stream)
            ev1.record()
            torch.cuda.synchronize()
            t_ms += ev0.elapsed_time(ev1) / reps
            nbytes += sum(pr.n_out) * (2 * D * b + 4) + dp.n_units * w.group * D * (b + 4)
        result["decode_attention"] = {"ms": t_ms, "us_per_layer": t_ms * 1e3 / layers, "algorithmic_bytes": nbytes,
                                      "achieved": nbytes / (t_ms * 1e-3) / 1e9, "unit": "GB/s",
                                      "frac": nbytes / (t_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                      "query_rows_per_unit": w.group}

    if args.per_query:
        # the same step with the norms aggregated per query row: four MFMA products per (token, query row)
        # instead of the streaming passes, so this leg is priced against the matrix cores, not HBM
        pws = torch.empty(kvs.kvs_per_query_workspace_size(big), dtype=torch.uint8, device=dev)
        a_tok = torch.empty(big.rows_in, dtype=torch.float32, device=dev)
        c_edge = torch.empty(big.rows_in, dtype=torch.float32, device=dev)
        reps = max(1, min(args.steps, 5))

        def timed(fn):
            fn()
            torch.cuda.synchronize()
            ev0.record()
            for _ in range(reps):
                fn()
            ev1.record()
            torch.cuda.synchronize()
            return ev0.elapsed_time(ev1) / reps

        def pq_step():
            for i, pr in enumerate(probs):
                kvs.kvs_step_per_query(pr, Qs[i], Ks[i], Vs[i], K_out[i], V_out[i], counts[i], pws, stream=stream)

        def pq_sens():
            for i, pr in enumerate(probs):
                kvs.kvs_sensitivity(pr, Qs[i], Ks[i], Vs[i], alpha, a_tok, c_edge, pws, stream=stream)

        step_ms, sens_ms = timed(pq_step), timed(pq_sens)
        # algorithmic work of kvs_sensitivity: K Q^T in both score sweeps and in both per-query kernels, P V and
        # V O^T once, 2 n R D flops each
        flops = layers * sum(12.0 * n * R * D for n in lens)
        result["per_query"] = {
            "ms_per_step": step_ms, "us_per_layer": step_ms * 1e3 / layers, "value": tokens_per_step / (step_ms * 1e-3),
            "unit": "tokens/s", "sensitivity_ms": sens_ms,
            "roofline": {"bound": "mfma", "call": "kvs_sensitivity", "algorithmic_flops": flops,
                         "achieved": flops / (sens_ms * 1e-3) / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                         "frac": flops / (sens_ms * 1e-3) / 1e12 / 2500.0}}

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, keep_host, args.cpu_seconds, workers, args.key_rule)
    print(json.dumps(result))


def cpu_baseline(w, keep_host, target_s, workers, rule="hessian"):
    """The fp64 oracle as it stands, on this machine's host cores, over a bounded sample of the same units."""
    from threadpoolctl import threadpool_limits

    from oracle import kvs_oracle as O

    units = [u for layer in sorted(keep_host) for u in keep_host[layer]]
    if not units:
        return None

    def run(u):
        O.step(u.Q, u.K, u.V, u.budget, w.n_sink, w.n_recent, counts=u.counts, rule=rule)
        return u.n

    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        run(units[0])
        one = time.perf_counter() - t0
        # as many units as fit the time target when `workers` of them run side by side
        n_units = int(min(len(units), max(workers, target_s / max(one, 1e-3) * workers * 0.5)))
        sample = units[:n_units]
        t0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=workers) as pool:
            done = sum(pool.map(run, sample))
        dt = time.perf_counter() - t0
    # a token counts K and V rows of ALL KV heads of a layer: n_kv_heads units make one token-layer row
    tokens = done / w.n_kv_heads
    return {"value": tokens / dt, "unit": "tokens/s", "cores": workers, "kind": "oracle",
            "sample": f"{len(sample)} units (layer 0.., {w.n_kv_heads} KV heads per layer) of the same workload; the oracle "
                      f"is numpy fp64 (not a tuned C++/OpenMP program), one BLAS thread per unit, {workers} units side "
                      f"by side on {workers} of the {os.cpu_count()} host threads the box reports, {dt:.1f} s"}


if __name__ == "__main__":
    main()
