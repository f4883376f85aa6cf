"""Build liblory.so (the HIP library behind include/lory.h) for gfx950.

Usage: python -m paper_2405_03133_amd.build
The library is built in-tree next to this file so that it travels with the
source tree; nothing is installed.
"""
from __future__ import annotations

import glob
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblory.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    "-fgpu-rdc" if False else "-fno-gpu-rdc",
    # keep the compiler from forming packed fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"),
    "-I", CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


RESOURCES = os.path.join(HERE, "_build", "kernel_resources.txt")
_REMARK = re.compile(r"remark:\s+(Function Name|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|LDS Size \[bytes/block\]): (\S+)")


def _run(cmd, verbose):
    """Run one compiler command; returns the kernels' resource usage it reported:
    [(name, vgprs, agprs, scratch bytes per lane, static LDS bytes)]."""
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    kernels, other = [], []
    for ln in proc.stdout.splitlines():
        m = _REMARK.search(ln)
        if m:
            key, val = m.group(1), m.group(2)
            if key == "Function Name":
                kernels.append({"name": val})
            elif kernels:
                kernels[-1][key.split(" ")[0]] = int(val)
        elif "packed-fp32-ops" not in ln and "-Rpass-analysis" not in ln and not re.match(r"^\s*(\d+ \|.*|\|\s*\^)\s*$", ln):
            other.append(ln)
    out = "\n".join(other)
    if verbose and out.strip():
        print(out)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return [(k["name"], k.get("VGPRs", -1), k.get("AGPRs", -1), k.get("ScratchSize", -1), k.get("LDS", -1))
            for k in kernels]


def build(verbose: bool = True, jobs: int = 8) -> str:
    """Compile every csrc/*.hip to an object (in parallel) and link liblory.so.

    The compiler's per-kernel resource report goes to _build/kernel_resources.txt, and the build
    fails if any kernel needs scratch memory (spilled registers): the kernels that count their own
    outstanding memory operations are written for code without spills."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    objs = []
    cmds = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        cmds.append([hipcc] + flags + ["-Rpass-analysis=kernel-resource-usage", "-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        reports = list(pool.map(lambda c: _run(c, verbose), cmds))
    kernels = sorted(k for rep in reports for k in rep)
    with open(RESOURCES, "w") as f:
        f.write("# kernel  VGPRs  AGPRs  scratch_bytes_per_lane  static_LDS_bytes\n")
        for k in kernels:
            f.write("%s %d %d %d %d\n" % k)
    spilling = [k for k in kernels if k[3] != 0]
    if spilling or not kernels:
        raise RuntimeError("kernels that need scratch memory (or no resource report at all): %r" % spilling)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc"] + objs + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
