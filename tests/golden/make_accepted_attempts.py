"""Writes tests/golden/accepted_attempts.json: for every unit the parity tests use, the first Query
attempt that passes the acceptance rule of tests/helpers.py (boundary gap >= 1e-4 relative, weight
denominators well conditioned).  Calls only the seeded generator and the fp64 oracle.

    python tests/golden/make_accepted_attempts.py
"""

import json
import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from helpers import MANIFEST, accepted_unit, load_manifest, manifest_key  # noqa: E402
from workloads import WORKLOADS, unit_lengths  # noqa: E402


def wanted():
    w = WORKLOADS["tiny"]
    yield w, 0, 0, 0, None
    w = WORKLOADS["llama8b_8k"]
    for h in range(w.n_kv_heads):
        yield w, 0, 0, h, None
    w = WORKLOADS["llama8b_32k"]
    for layer in range(w.layers):                  # every unit of the headline workload (the full-size step test)
        for h in range(w.n_kv_heads):
            yield w, layer, 0, h, None
    w = WORKLOADS["ragged16"]
    lens = unit_lengths(w)
    for s in (0, 3, 7, 11, 15):
        for h in (0, 5):
            yield w, 0, s, h, min(lens[s], 20000 + 37 * s)
    w = WORKLOADS["stress128k"].scaled(length=("fixed", 16384), budget=("fixed", 1024))
    for h in range(2):
        yield w, 0, 0, h, None
    w = WORKLOADS["stress128k"]
    yield w, 0, 0, 0, None


def one(args):
    w, layer, seq, head, n = args
    t = time.time()
    a = accepted_unit(w, layer, seq, head, n=n, manifest={})
    key = manifest_key(w, layer, seq, head, a.inputs.n)
    return key, a.inputs.attempt, f"{key}: attempt {a.inputs.attempt} gap {a.gap:.2e} cond {a.cond:.3f} ({time.time() - t:.1f}s)"


def main():
    from multiprocessing import Pool
    manifest = {}
    with Pool(int(os.environ.get("KVS_MANIFEST_WORKERS", "6"))) as pool:
        for key, attempt, line in pool.imap_unordered(one, list(wanted())):
            manifest[key] = attempt
            print(line, flush=True)
    with open(MANIFEST, "w") as f:
        json.dump(manifest, f, indent=1, sort_keys=True)


if __name__ == "__main__":
    main()
