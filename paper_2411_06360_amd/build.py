"""Build step: compile the HIP library (csrc/) for gfx950 into ``librsr.so`` next to this file.

``python -m paper_2411_06360_amd.build`` or ``build()`` always compiles; the binding only loads
what is already built.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librsr.so")
SOURCES = ["rsr_lib.hip", "rsr_dense.hip", "rsr_prep.hip", "rsr_pack.cpp", "rsr_qbit.cpp"]
ARCH = "gfx950"

# -packed-fp32-ops off: the compiler must not form packed fp32 instructions from the float adds.
FLAGS = [
    "-O3", "-std=c++17", f"--offload-arch={ARCH}", "-fPIC", "-shared", "-fno-strict-aliasing",
    "-fno-gpu-rdc", "-Wall", "-Wno-unused-command-line-argument",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build(extra_flags=(), output: str = LIB, verbose: bool = False) -> str:
    tmp = output + f".tmp{os.getpid()}"
    cmd = [hipcc(), *FLAGS, *extra_flags, "-o", tmp, *[os.path.join(CSRC, s) for s in SOURCES], "-lpthread"]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the device-only target feature and says so; that is harmless
    log = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError(f"hipcc failed ({proc.returncode}):\n{log}")
    if verbose and log.strip():
        print(log)
    os.replace(tmp, output)
    return output


if __name__ == "__main__":
    print(build(extra_flags=sys.argv[1:], verbose=True))
