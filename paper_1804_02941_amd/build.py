"""Build step: compile the HIP sources into the in-tree shared library for gfx950.

    python -m paper_1804_02941_amd.build

hipcc cross-compiles without a GPU.  The library is written next to the sources
(``paper_1804_02941_amd/libdab_hip.so``); nothing is installed.
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdab_hip.so")
SOURCES = ("api.hip", "binconv.hip", "direct.hip", "pack.hip", "estimate.hip", "training.hip", "probe.hip")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-fno-gpu-rdc", "-ffp-contract=off",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    # per-kernel register / LDS report, parsed below
    "-Rpass-analysis=kernel-resource-usage",
]


def kernel_resources(log: str) -> dict:
    """{kernel name: {"VGPRs": .., "AGPRs": .., "ScratchSize [bytes/lane]": .., ...}} from hipcc's remarks."""
    out, cur = {}, None
    for line in log.splitlines():
        if "remark:" not in line:
            continue
        text = line.split("remark:", 1)[1].split("[-Rpass-analysis", 1)[0].strip()
        if text.startswith("Function Name:"):
            cur = out.setdefault(text.split(":", 1)[1].strip(), {})
        elif cur is not None and ":" in text:
            key, val = text.rsplit(":", 1)
            try:
                cur[key.strip()] = int(val)
            except ValueError:
                pass
    return out


def check_resources(res: dict) -> None:
    """Refuse a build with a kernel whose register allocation is exactly 64 VGPRs (granule 8, no AGPRs),
    or with any kernel that spills to scratch memory.

    Measured on MI355X with the estimation kernel: such an allocation gave wrong results whenever two
    workgroups shared a compute unit, the same instructions with a 72-register allocation did not."""
    for name, r in res.items():
        v, a = r.get("VGPRs", 0), r.get("AGPRs", 0)
        if a == 0 and 56 < v <= 64:
            raise RuntimeError(f"kernel {name} is allocated exactly 64 VGPRs; reserve one more register in it")
        if r.get("ScratchSize [bytes/lane]", 0) != 0:
            raise RuntimeError(f"kernel {name} spills to scratch memory ({r['ScratchSize [bytes/lane]']} bytes per lane)")


def _without_remarks(text: str) -> str:
    """Compiler output minus the resource remarks (and their source excerpts) and a known harmless warning."""
    keep, skipping = [], False
    for line in text.splitlines():
        if "-Rpass-analysis=kernel-resource-usage" in line or "is not a recognized feature for this target" in line:
            skipping = True
            continue
        if skipping and (line.lstrip().startswith("|") or line.split("|", 1)[0].strip().isdigit()):
            continue
        skipping = False
        keep.append(line)
    return "\n".join(keep)


def build(verbose: bool = False) -> str:
    """Compile every HIP translation unit and link libdab_hip.so; returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log = _without_remarks(proc.stdout)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log, flush=True)
    res = kernel_resources(proc.stdout)
    if not res:
        raise RuntimeError("hipcc printed no kernel resource report")
    check_resources(res)
    if verbose:
        for name, r in sorted(res.items()):
            print(f"  {name}: VGPRs {r.get('VGPRs')} AGPRs {r.get('AGPRs')} SGPRs {r.get('TotalSGPRs')} "
                  f"LDS {r.get('LDS Size [bytes/block]')} scratch {r.get('ScratchSize [bytes/lane]')} "
                  f"waves/SIMD {r.get('Occupancy [waves/SIMD]')}", flush=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-q" not in sys.argv))
