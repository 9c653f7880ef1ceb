"""Build the HIP library in-tree: hipcc cross-compiles for gfx950 without a GPU.

Every source is compiled to an object of its own (in parallel) and the objects are linked into one shared library.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(LIB_DIR, "libdreamddp.so")
# (source, object name, extra flags); the table-driven fused kernel has the most instantiations and is built in two halves
SOURCES = [("ddp_kernels_fused.hip", "ddp_kernels_fused_adamw", ["-DDDP_FUSED_ADAM=1"]),
           ("ddp_kernels_fused.hip", "ddp_kernels_fused_sgdm", ["-DDDP_FUSED_ADAM=0"]),
           ("ddp_kernels_fused_dense.hip", "ddp_kernels_fused_dense", []), ("ddp_kernels_mean.hip", "ddp_kernels_mean", []),
           ("ddp_kernels_update.hip", "ddp_kernels_update", []), ("ddp_kernels_copy.hip", "ddp_kernels_copy", []),
           ("ddp_context.hip", "ddp_context", []), ("ddp_noalloc.hip", "ddp_noalloc", []), ("ddp_probe.hip", "ddp_probe", []),
           ("ddp_stream.hip", "ddp_stream", []), ("ddp_schedule.cpp", "ddp_schedule", [])]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                                            # products and sums stay separate operations
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed fp32 instructions (a device feature)
    "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-unused-function",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]

# hipcc hands -target-feature to its host pass as well, where an x86 compiler answers with this line for a feature it
# cannot know; the device pass, which the flag is for, accepts it.  The line is dropped from the echoed diagnostics.
_HOST_PASS_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"


def _diagnostics(text: str) -> str:
    return "\n".join(ln for ln in text.splitlines() if ln.strip() and ln.strip() != _HOST_PASS_NOTE)


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    diag = _diagnostics(r.stdout + r.stderr)
    if r.returncode != 0:
        sys.stderr.write(diag + "\n")
        raise RuntimeError("hipcc failed: " + " ".join(cmd[-3:]))
    if verbose and diag:
        print(diag, flush=True)


def build(verbose: bool = False, jobs: int = 0) -> str:
    os.makedirs(LIB_DIR, exist_ok=True)
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = jobs or min(len(SOURCES), max(1, len(os.sched_getaffinity(0))))
    objs = [os.path.join(OBJ_DIR, name + ".o") for _, name, _ in SOURCES]
    cmds = [[hipcc] + FLAGS + extra + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", o] for (src, _, extra), o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(lambda c: _run(c, verbose), cmds))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
