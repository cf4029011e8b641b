"""Builds libkvs.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc.

    python -m paper_2603_00907_amd.build [--report]

`--report` prints registers, LDS and occupancy of every kernel as the compiler sees them.
"""

from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvs.so")

SOURCES = ["kvs_api.hip", "kvs_score_valu.hip", "kvs_score_mfma.hip", "kvs_select.hip", "kvs_merge.hip", "kvs_decode.hip",
           "kvs_perquery.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # hipcc must not form packed-fp32 instructions on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(report: bool = False, defines=(), out: str = LIB) -> str:
    cmd = [hipcc()] + FLAGS + (["-Rpass-analysis=kernel-resource-usage"] if report else [])
    cmd += ["-D" + d for d in defines]
    cmd += ["-o", out] + [os.path.join(CSRC, s) for s in SOURCES]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
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
    print(build(report="--report" in sys.argv))
