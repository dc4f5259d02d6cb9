"""Builds libmoe_hip.so (gfx950) in-tree with hipcc.  `python -m paper_2502_02581_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

from . import asm_check

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmoe_hip.so")
SOURCES = ["common.hip", "route.hip", "dispatch.hip", "combine.hip", "expert.hip", "planner.hip"]
# sources with device code: their gfx950 assembly is kept and checked (asm_check.py)
CHECKED = ["common.hip", "route.hip", "dispatch.hip", "combine.hip", "expert.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def device_asm(src: str) -> str:
    """Where the compile step of `src` leaves its gfx950 assembly."""
    return os.path.join(HERE, "_build", src.replace(".hip", "") + "-hip-amdgcn-amd-amdhsa-gfx950.s")


def build(verbose: bool = True) -> str:
    """Compiles every HIP source and links the shared library; always recompiles."""
    objs = []
    procs = []
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        cmd = [hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if src in CHECKED:
            cmd.insert(1, "-save-temps=obj")
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        lines = [ln for ln in out.splitlines() if "packed-fp32-ops" not in ln and "is not a recognized feature" not in ln]
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n" + "\n".join(lines))
        if verbose and any("warning" in ln or "error" in ln for ln in lines):
            print("\n".join(lines), file=sys.stderr)
    for src in CHECKED:
        findings = asm_check.check(device_asm(src))
        if findings:
            raise RuntimeError(f"device assembly of {src} fails its checks:\n" + "\n".join(findings))
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
