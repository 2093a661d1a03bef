"""Build step: compile the HIP sources for gfx950 into ``librf.so`` (in-tree).

Usage: ``python -m paper_2603_10026_amd.build``  (hipcc cross-compiles without
a GPU).  The library is written next to this file so that it travels with the
source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librf.so")

SOURCES = [
    "api.hip",
    "softmax.hip",
    "variance.hip",
    "moe_routing.hip",
    "fp8_quant_gemm.hip",
    "attention_f32.hip",
    "attention_bf16.hip",
    "attention_bf16_wide.hip",
    "attention_splitk.hip",
    "merge_states.hip",
    "rmsnorm_gemm.hip",
    "diag.hip",
]

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-fvisibility=hidden",
    "-DRF_BUILDING=1",
    # packed fp32 VALU ops are switched off for device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unknown-attributes",
    # the direct-to-LDS loads are raw instructions that write M0 and say so in their clobber
    # lists; clang remarks that M0 is a reserved register
    "-Wno-inline-asm",
]


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose=True, jobs=8):
    """Compile every source to an object file (in parallel) and link librf.so."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    cc = hipcc()
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [cc, *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _drain(procs)
    _drain(procs)
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    check_waits(verbose)
    return LIB


def check_waits(verbose=True):
    """Kernels that load registers from inline assembly and count their own waits are
    checked against a model of the vector-memory counter (see check_isa); a register touched
    while its load is in flight fails the build."""
    from . import check_isa
    cc = hipcc()
    for src in SOURCES:
        path = os.path.join(CSRC, src)
        counters = check_isa.hand_counted(path)
        if not counters:
            continue
        n, hazards = check_isa.check_source(path, cc, HIPCC_FLAGS, counters)
        if verbose:
            print(f"check_isa {src} ({'+'.join(counters)}): {n} kernels, {len(hazards)} hazards", flush=True)
        if hazards:
            raise RuntimeError(f"{src}: registers touched while their loads are in flight:\n  "
                               + "\n  ".join(hazards[:20]))


def _drain(procs):
    while procs:
        src, p = procs.pop(0)
        out, _ = p.communicate()
        lines = [ln for ln in out.splitlines() if "packed-fp32-ops" not in ln and ln.strip()]
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n" + out)
        if lines:
            print(f"[{src}]\n" + "\n".join(lines), flush=True)


if __name__ == "__main__":
    build_library()
    print("built", LIB)
