"""Build the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libguard_hip.so")
SOURCES = ["api.hip", "score.hip", "score_z.hip", "window.hip", "topk.hip", "severity.hip", "sweep.hip", "ledger.hip", "membership.hip"]

# One rounding per written operation (no FMA contraction), IEEE divide,
# denormals kept, and no packed-fp32 instructions.
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off", "-fno-fast-math", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    # the compiler's own account of registers, spills and LDS per kernel (kept as text
    # beside the objects and checked below)
    "-Rpass-analysis=kernel-resource-usage",
]

# The scoring kernel keeps a whole column in registers and is laid out for 16 waves per
# CU: every instantiation must stay within 128 vector registers and spill none of them.
VGPR_BUDGET = 128


def resource_file(src: str) -> str:
    return os.path.join(HERE, "_build", src.replace(".hip", ".resources.txt"))


def parse_resources(text: str) -> dict:
    """{kernel symbol: {field: int}} from -Rpass-analysis=kernel-resource-usage remarks."""
    out, cur = {}, None
    for line in text.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z][A-Za-z /\[\]]*?):\s+(-?\d+|True|False)\s", line)
        if m and cur is not None:
            v = m.group(2)
            cur[m.group(1).strip()] = int(v) if v.lstrip("-").isdigit() else (v == "True")
    return out


def tiling_of(symbol: str):
    """(NT, ROWS, LOG_NB, FULL, SPLIT, WANT_Z) of a mangled score_kernel<...> symbol, or None."""
    m = re.search(r"score_kernelILi(\d+)ELi(\d+)ELi(\d+)ELb([01])ELb([01])ELb([01])E", symbol)
    return tuple(int(g) for g in m.groups()) if m else None


# Ragged tilings (rank counts that do not fill the register tile: bounds checks on every
# row), the one-wave tilings of up to 1 024 ranks (launch-bound) and the per-column route
# of short batches (latency-bound: one column per workgroup) may keep a few registers in
# scratch memory; the exact-fit batch tilings of 256 threads and more may not.
RAGGED_SCRATCH_LIMIT = 128     # bytes per lane


def check_register_budget(resources: dict) -> list:
    """Violations among the score_kernel instantiations (empty = within budget)."""
    bad = []
    for name, r in resources.items():
        t = tiling_of(name)
        if t is None:
            continue
        full = bool(t[3]) and t[0] >= 256 and not t[4]
        if r.get("VGPRs", 0) + r.get("AGPRs", 0) > VGPR_BUDGET:
            bad.append(f"{name}: {r.get('VGPRs')} VGPRs + {r.get('AGPRs')} AGPRs > {VGPR_BUDGET}")
        scratch = r.get("ScratchSize [bytes/lane]", 0)
        if r.get("Dynamic Stack", False) or scratch > (0 if full else RAGGED_SCRATCH_LIMIT) or \
                (full and r.get("VGPRs Spill", 0)):
            bad.append(f"{name}: {r.get('VGPRs Spill')} vector registers spilled, {scratch} bytes of scratch per lane")
        if r.get("Occupancy [waves/SIMD]", 0) < 4:
            bad.append(f"{name}: occupancy {r.get('Occupancy [waves/SIMD]')} waves per SIMD < 4")
    return bad


def build(verbose: bool = False, extra=()) -> str:
    """Compile every source and link libguard_hip.so; always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(HERE, "_build", src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stderr=subprocess.PIPE, text=True)))
        objs.append(obj)
    for src, p in procs:
        _, err = p.communicate()
        remarks = [l for l in err.splitlines() if "-Rpass-analysis=kernel-resource-usage" in l]
        with open(resource_file(src), "w") as f:
            f.write("\n".join(remarks) + "\n")
        err = "\n".join(l for l in err.splitlines()
                        if "packed-fp32-ops" not in l and "-Rpass-analysis=kernel-resource-usage" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
    bad = []
    for src in ("score.hip", "score_z.hip"):
        with open(resource_file(src)) as f:
            res = parse_resources(f.read())
        if not any(tiling_of(k) for k in res):
            bad.append(f"{src}: the compiler reported no score_kernel instantiation")
        bad += check_register_budget(res)
    if bad:
        raise RuntimeError("register budget of the scoring kernel exceeded:\n  " + "\n  ".join(bad))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
