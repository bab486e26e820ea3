"""Builds libkvq.so (hand-written HIP for gfx950 + the host bookkeeping) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvq.so")
SOURCES = ["kvq_host.cpp", "kvq_quant.hip", "kvq_attention.hip", "kvq_attention_batch.hip", "kvq_attention_i16_append.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fhip-fp32-correctly-rounded-divide-sqrt", "-ffp-contract=on",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes"]


STAMPS_LIB = os.path.join(HERE, "libkvq_stamps.so")
NOARITH_LIB = os.path.join(HERE, "libkvq_noarith.so")


def build(verbose: bool = False, phase_stamps: bool = False, no_arithmetic: bool = False) -> str:
    """phase_stamps: build the measurement variant libkvq_stamps.so (attention kernels that record when a workgroup
    passes each phase, see csrc/kvq_phase_stamps.h) instead of the library.  no_arithmetic: build libkvq_noarith.so,
    whose attention kernels load every tile but compute on none (the floor of the launch; results meaningless).
    Nothing loads either of them but phase_table.py."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    flags = FLAGS + (["-DKVQ_PHASE_STAMPS"] if phase_stamps else []) + (["-DKVQ_NO_ARITHMETIC"] if no_arithmetic else [])
    lib = STAMPS_LIB if phase_stamps else NOARITH_LIB if no_arithmetic else LIB
    suffix = ".stamps.o" if phase_stamps else ".noarith.o" if no_arithmetic else ".o"
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + suffix)
        cmd = [hipcc, *flags, "-I", os.path.join(HERE, "..", "include"), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return lib


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, phase_stamps="--phase-stamps" in sys.argv, no_arithmetic="--no-arithmetic" in sys.argv))
