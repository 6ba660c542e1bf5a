"""Builds ``libpat.so`` (planner + HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libpat.so")
PROBE_LIB = os.path.join(HERE, "libpat_probe.so")       # measurement kernels (bench, calibration)

SOURCES = ["pat_plan.cpp", "pat_cache.cpp", "pat_api.hip", "pat_forward.hip", "pat_merge.hip"]

HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # packed-fp32 VALU forms are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False, jobs: int = 4) -> str:
    """Compile every source for gfx950 and link the shared library. Always recompiles."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src + ".o")
        objs.append(obj)
        cmd = [hipcc(), *HIP_FLAGS, "-I", INCLUDE, "-I", CSRC, "-c", os.path.join(CSRC, src),
               "-o", obj]
        if src.endswith(".cpp"):
            cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-Wall", "-I", INCLUDE, "-I", CSRC,
                   "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        if len(procs) >= jobs:
            _drain(procs, verbose)
    _drain(procs, verbose)
    check_forward_isa(objdir, verbose)
    link = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.check_call(link)
    probe = [hipcc(), *HIP_FLAGS, "-shared", "-o", PROBE_LIB, os.path.join(CSRC, "pat_probe.hip")]
    if verbose:
        print(" ".join(probe), flush=True)
    out = subprocess.run(probe, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    if out.returncode != 0:
        raise RuntimeError("hipcc failed on pat_probe.hip:\n" + out.stdout.decode(errors="replace"))
    return LIB


RING_FIRST_VGPR = 224      # pat_tile_packed.hip.h: v224..v255 hold loads in flight


def check_forward_isa(objdir: str, verbose: bool = False) -> None:
    """The packed tile keeps its K/V loads in flight in v224..v255, named in inline asm only.
    That is safe only if the compiler never allocates those registers itself and the kernel's
    register count still covers them; both depend on how this compiler version reads the
    kernel's VGPR-limit attribute, so the generated ISA is checked on every build."""
    asm = os.path.join(objdir, "pat_forward.s")
    cmd = [hipcc(), *HIP_FLAGS, "-I", INCLUDE, "-I", CSRC, "-S", "--cuda-device-only",
           os.path.join(CSRC, "pat_forward.hip"), "-o", asm]
    out = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    if out.returncode != 0:
        raise RuntimeError("hipcc -S failed on pat_forward.hip:\n" + out.stdout.decode(errors="replace"))
    in_asm = False
    counts = {}
    kernel = None
    for n, line in enumerate(open(asm), 1):
        m = re.match(r"(_ZN3pat\w+):", line)
        if m:
            kernel = m.group(1)
        if "ASMSTART" in line:
            in_asm = True
        elif "ASMEND" in line:
            in_asm = False
        elif line.lstrip().startswith("; NumVgprs:"):
            counts[kernel] = int(line.split(":")[1])
        elif not in_asm and not line.lstrip().startswith((";", ".")):
            for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", line.split(";")[0]):
                top = int(m.group(2) or m.group(3))
                if top >= RING_FIRST_VGPR:
                    raise RuntimeError(f"{asm}:{n}: the compiler allocated a ring register: {line.strip()}")
    # every kernel that holds the packed tile must declare the whole register file (the 16-row
    # kernel of two-kernel launches does not hold it and must stay within half of it)
    ring = {k: c for k, c in counts.items() if "forward_stream_kernel" not in k}
    if not ring or any(c != 256 for c in ring.values()):
        raise RuntimeError(f"{asm}: kernels with the packed tile must declare 256 VGPRs, found {counts}")
    if any(c > 256 for c in counts.values()):
        raise RuntimeError(f"{asm}: more than 256 VGPRs: {counts}")
    if verbose:
        print(f"forward ISA check passed ({counts})")


def _drain(procs, verbose):
    for src, p in procs:
        out = p.communicate()[0].decode(errors="replace")
        # hipcc's host pass warns that it does not know the packed-fp32 feature: harmless
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    procs.clear()


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
