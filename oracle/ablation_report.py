"""What the Key rule buys, measured with the fp64 oracle alone (test infrastructure, CPU only).

    python -m oracle.ablation_report [workload] [n_units]

For units of a synthetic workload it merges the cache with each Key rule ("hessian": Eq. kstar_final
with the off-diagonal coupling; "diagonal": coupling dropped; "mean": arithmetic mean) and reports how far
the cardinality-normalised attention output over the merged cache (Sec. 3.1) is from attention over the
full cache, for the window's own queries and for fresh queries of the same distribution.  For caches of
plain tokens it adds the hessian rule with per-query aggregation of the norms ("per_query": every query row
with its own attention and output, norms averaged over the rows).
"""

import sys

import numpy as np

from oracle import kvs_oracle as O
from workloads import WORKLOADS, generate_unit


def full_attention(q, K, V, counts=None):
    return O.score(q[None, :], K, V, counts=counts)[1]


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "llama8b_8k"
    n_units = int(sys.argv[2]) if len(sys.argv) > 2 else 4
    w = WORKLOADS[name]
    rng = np.random.default_rng(7)
    rules = list(O.RULES) + (["per_query"] if w.mean_count == 0 else [])
    err = {r: {"window": [], "fresh": []} for r in rules}
    dk = {r: [] for r in rules if r != "hessian"}
    for h in range(n_units):
        u = generate_unit(w, 0, 0, h % w.n_kv_heads)
        ab, ob = O.score(u.Q, u.K, u.V, counts=u.counts)
        mask, slot = O.select(ab, u.budget, w.n_sink, w.n_recent)
        merged = {r: O.merge_compact(u.K, u.V, ab, ob, mask, slot, counts_in=u.counts, rule=r) for r in O.RULES}
        if "per_query" in rules:
            merged["per_query"] = O.merge_compact(u.K, u.V, ab, ob, mask, slot, norms=O.per_query_norms(u.Q, u.K, u.V))
        queries = {"window": u.Q.reshape(-1, w.head_dim)[:16].astype(np.float64),
                   "fresh": rng.standard_normal((16, w.head_dim))}
        for kind, Qs in queries.items():
            for q in Qs:
                want = full_attention(q, u.K, u.V, u.counts)
                for r, m in merged.items():
                    got = O.merged_attention(q, m.K_out, m.V_out, m.counts)
                    err[r][kind].append(np.linalg.norm(got - want) / np.linalg.norm(want))
        multi = merged["hessian"].n_rows > 1
        for r in dk:
            d = np.linalg.norm(merged[r].K_out[multi] - merged["hessian"].K_out[multi], axis=1)
            dk[r].append((d / np.linalg.norm(merged["hessian"].K_out[multi], axis=1)).mean())
    print(f"workload {name}, {n_units} units, {w.length[1]} -> {w.budget[1]} rows")
    for r in rules:
        print(f"  rule {r:9s} attention-output error vs the full cache: window queries "
              f"{np.mean(err[r]['window']):.4e}, fresh queries {np.mean(err[r]['fresh']):.4e}")
    for r, v in dk.items():
        print(f"  merged Keys of rule {r:9s} differ from the hessian rule's by {np.mean(v):.3e} (mean relative L2)")


if __name__ == "__main__":
    main()
