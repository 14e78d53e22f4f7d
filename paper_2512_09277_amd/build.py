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
                if not re.match(r"^\s*\d+ \|", line):
                    print(line, file=sys.stderr)
            continue
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"(VGPRs|ScratchSize \[bytes/lane\]|LDS Size \[bytes/block\]): (\d+)", line)
        if m:
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


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
