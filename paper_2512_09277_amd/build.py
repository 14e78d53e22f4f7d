"""Builds libmetro.so (the C-ABI HIP library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmetro.so")
SOURCES = ["route.hip", "permute.hip", "ffn.hip", "unpermute.hip", "gate.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]


RESOURCES: dict = {}        # kernel symbol -> {"VGPRs": .., "AGPRs": .., "Occupancy": .., "LDS": .., "Scratch": ..} of the last build


def build(verbose: bool = False, extra=()) -> str:
    """Compile the library; fails if any kernel spills registers to scratch memory (a spill in a
    streaming loop costs more HBM traffic than the kernel is allowed to waste)."""
    cmd = ["hipcc", *FLAGS, "-Rpass-analysis=kernel-resource-usage", *extra, "-I", os.path.join(ROOT, "include"),
           "-I", CSRC, *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    name, report, spilled = "?", [], []
    for line in proc.stderr.splitlines():
        if "remark:" not in line:
            if "packed-fp32-ops" not in line and "kernel-resource-usage" not in line and line.strip() not in ("^", ""):
                if not re.match(r"^\s*(\d+ )?\|", line):
                    print(line, file=sys.stderr)
            continue
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"(VGPRs|AGPRs|Occupancy \[waves/SIMD\]|ScratchSize \[bytes/lane\]|LDS Size \[bytes/block\]): (\d+)", line)
        if m:
            short = {"VGPRs": "VGPRs", "AGPRs": "AGPRs", "Occupancy [waves/SIMD]": "Occupancy",
                     "ScratchSize [bytes/lane]": "Scratch", "LDS Size [bytes/block]": "LDS"}[m.group(1)]
            RESOURCES.setdefault(name, {})[short] = int(m.group(2))
            report.append((name, m.group(1), int(m.group(2))))
            if m.group(1).startswith("Scratch") and int(m.group(2)) > 0:
                spilled.append((name, int(m.group(2))))
    if proc.returncode != 0:
        raise subprocess.CalledProcessError(proc.returncode, cmd)
    if verbose:
        for name, key, val in report:
            if key == "VGPRs":
                print(f"  {name[:70]:70s} VGPRs {val}")
    if spilled:
        raise RuntimeError(f"kernels spill to scratch: {spilled}")
    return LIB


def resources_markdown() -> str:
    """The compiler's per-kernel resource report of the last build() as a markdown table."""
    rows = ["| kernel | VGPRs | AGPRs | static LDS bytes | scratch | occupancy (waves/SIMD, compiler) |", "|---|---|---|---|---|---|"]
    demangle = subprocess.run(["c++filt"], input="\n".join(RESOURCES), stdout=subprocess.PIPE, text=True).stdout.splitlines()
    for sym, pretty in zip(RESOURCES, demangle):
        r = RESOURCES[sym]
        pretty = pretty.replace("metro::(anonymous namespace)::", "").replace("void ", "").split("(")[0]
        m = re.match(r"_ZN5metro12_GLOBAL__N_1\d+([a-z_]+)I", pretty)      # __bf16 instantiations are not demangled
        if m:
            pretty = m.group(1) + "<__bf16>"
        rows.append(f"| {pretty} | {r.get('VGPRs')} | {r.get('AGPRs')} | {r.get('LDS')} | {r.get('Scratch')} | {r.get('Occupancy')} |")
    return "\n".join(rows)


if __name__ == "__main__":
    args = [a for a in sys.argv[1:] if a != "--resources"]
    print(build(verbose="--resources" not in sys.argv, extra=args))
    if "--resources" in sys.argv:
        print(resources_markdown())
