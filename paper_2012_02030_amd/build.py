"""Build the gfx950 shared library (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libap_mi355x.so")
RESOURCES = os.path.join(PKG, "libap_mi355x.resources.txt")   # per-kernel registers, spills, LDS

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # leading scalar kernel arguments (up to 16 dwords) arrive in registers when a wavefront starts
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-Wall", "-Wno-unused-command-line-argument",
    # the LDS-direct load helper names M0 as clobbered; the compiler remarks that M0 is a reserved
    # register (it never keeps a value of its own live in it across a statement)
    "-Wno-inline-asm",
    "-Rpass-analysis=kernel-resource-usage", "-fno-caret-diagnostics",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def kernel_resources(compiler_output: str) -> list:
    """Per-kernel figures from the compiler's resource-usage remarks: one dict per kernel."""
    kernels, cur = [], None
    for line in compiler_output.splitlines():
        if "remark:" not in line:
            continue
        text = line.split("remark:", 1)[1].split("[-Rpass", 1)[0].strip()
        if text.startswith("Function Name:"):
            cur = {"name": text.split(":", 1)[1].strip()}
            kernels.append(cur)
        elif cur is not None and ":" in text:
            key, val = text.split(":", 1)
            cur[key.strip()] = val.strip()
    return kernels


def build(verbose: bool = False, extra=()) -> str:
    """Compile every HIP source into libap_mi355x.so next to this file and return its path.

    Writes the per-kernel register, spill and LDS figures next to the library and warns if any
    kernel spills vector registers: spilled values travel through the same in-order vector memory
    path as the tile loads, and a reload inside a tile loop then waits for the tiles in flight
    (tests/test_abi.py asserts that there is none)."""
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, *FLAGS, *extra, *sources(), "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the device-only target feature and says so; drop that line
    out = "\n".join(line for line in proc.stdout.splitlines() if "packed-fp32-ops" not in line)
    if proc.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("hipcc failed:\n" + out)
    kernels = kernel_resources(out)
    out = "\n".join(line for line in out.splitlines() if "-Rpass-analysis=kernel-resource-usage" not in line)
    if verbose and out.strip():
        print(out)
    with open(RESOURCES, "w") as f:
        for k in kernels:
            f.write("%s  VGPRs %s  AGPRs %s  spilled VGPRs %s  spilled SGPRs %s  waves/SIMD %s  LDS %s\n" % (
                k["name"], k.get("VGPRs", "?"), k.get("AGPRs", "?"), k.get("VGPRs Spill", "?"),
                k.get("SGPRs Spill", "?"), k.get("Occupancy [waves/SIMD]", "?"),
                k.get("LDS Size [bytes/block]", "?")))
    spilling = [k["name"] for k in kernels if k.get("VGPRs Spill", "0") != "0"]
    if spilling:                                             # the library still works; the tests flag it
        print("WARNING: kernels that spill vector registers: " + ", ".join(spilling), flush=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
