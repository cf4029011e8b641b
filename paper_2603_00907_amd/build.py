"""Builds libkvs.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc.

    python -m paper_2603_00907_amd.build [--report] [--incremental]

Every source is compiled to an object of its own (side by side), then linked.  `--report` prints registers,
LDS and occupancy of every kernel as the compiler sees them; `--incremental` recompiles only the sources that
are newer than their objects (or older than a header).
"""

from __future__ import annotations

import glob
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvs.so")
OBJ = os.path.join(HERE, "_build")

SOURCES = ["kvs_api.hip", "kvs_score_valu.hip", "kvs_score_mfma.hip", "kvs_score_fused.hip", "kvs_select.hip", "kvs_merge.hip", "kvs_decode.hip",
           "kvs_perquery.hip", "kvs_perquery_f32.hip", "kvs_table.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # hipcc must not form packed-fp32 instructions on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _stale(src: str, obj: str) -> bool:
    if not os.path.exists(obj):
        return True
    deps = [src] + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return any(os.path.getmtime(d) > os.path.getmtime(obj) for d in deps)


def build(report: bool = False, defines=(), out: str = LIB, incremental: bool = False, jobs: int = 8) -> str:
    """Compiles every source (all of them unless `incremental`) and links `out`."""
    tag = ("_" + re.sub(r"\W+", "_", "_".join(defines))) if defines else ""
    os.makedirs(OBJ, exist_ok=True)
    base = [hipcc()] + FLAGS + (["-Rpass-analysis=kernel-resource-usage"] if report else [])
    base += ["-D" + d for d in defines]
    noise = "is not a recognized feature for this target"

    def compile_one(name):
        src = os.path.join(CSRC, name)
        obj = os.path.join(OBJ, os.path.splitext(name)[0] + tag + ".o")
        if incremental and not report and not _stale(src, obj):
            return obj, ""
        proc = subprocess.run(base + ["-c", src, "-o", obj], capture_output=True, text=True)
        err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
        if proc.returncode != 0:
            raise RuntimeError(f"hipcc failed on {name}:\n" + err)
        return obj, err

    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(SOURCES)))) as pool:
        done = list(pool.map(compile_one, SOURCES))
    err = "\n".join(e for _, e in done if e)
    proc = subprocess.run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + [o for o, _ in done],
                          capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("link failed:\n" + proc.stderr)
    if report:
        print(_summarise(err))
    elif err.strip() and "warning" in err:
        sys.stderr.write(err + "\n")
    return out


def _summarise(text: str) -> str:
    rows, cur = [], None
    for line in text.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            name = subprocess.run(["c++filt", m.group(1)], capture_output=True, text=True).stdout.strip()
            name = name.replace("(anonymous namespace)::", "").replace("void ", "")
            cur = {"name": re.sub(r"\(.*", "", name)}
            rows.append(cur)
            continue
        m = re.search(r"remark:\s+(VGPRs|AGPRs|VGPRs Spill|LDS Size \[bytes/block\]|Occupancy \[waves/SIMD\]): (\d+)", line)
        if m and cur is not None:
            cur[m.group(1)] = int(m.group(2))
    out = [f"{'kernel':70s} {'VGPR':>5s} {'AGPR':>5s} {'spill':>5s} {'LDS':>7s} {'occ':>3s}"]
    for r in rows:
        out.append(f"{r['name'][:70]:70s} {r.get('VGPRs', 0):5d} {r.get('AGPRs', 0):5d} {r.get('VGPRs Spill', 0):5d} "
                   f"{r.get('LDS Size [bytes/block]', 0):7d} {r.get('Occupancy [waves/SIMD]', 0):3d}")
    return "\n".join(out)


if __name__ == "__main__":
    print(build(report="--report" in sys.argv, incremental="--incremental" in sys.argv))
