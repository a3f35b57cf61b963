"""Build libssg.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc; and libssg_probe.so, the
matrix-core ceiling probe that only the benchmark loads."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libssg.so")
SOURCES = ["ssg_api.hip", "ssg_quant.hip", "ssg_gemm.hip", "ssg_gemm_bwd.hip", "ssg_adam.hip"]
PROBE_LIB = os.path.join(HERE, "libssg_probe.so")
PROBE_SOURCES = ["ssg_probe.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                                   # no FMA contraction: every fp32 step rounds once
    "-fhip-fp32-correctly-rounded-divide-sqrt",            # scales use correctly rounded divisions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-Wno-inline-asm",                                     # m0 in the clobber list of the LDS-DMA asm is "reserved": intended
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature; harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        sys.stderr.write(res.stderr)
        raise RuntimeError("hipcc failed: " + " ".join(cmd))
    if verbose and err.strip():
        sys.stderr.write(err + "\n")


def build(verbose: bool = True, extra_flags=()) -> str:
    """Compile every source to an object (in parallel: the files are independent) and link the two libraries."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    with tempfile.TemporaryDirectory(prefix="ssg_build_") as tmp:
        obj = {s: os.path.join(tmp, os.path.splitext(s)[0] + ".o") for s in SOURCES + PROBE_SOURCES}
        cmds = [[hipcc] + FLAGS + list(extra_flags) + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in obj.items()]
        with ThreadPoolExecutor(max_workers=min(len(cmds), 8)) as pool:
            list(pool.map(lambda c: _run(c, verbose), cmds))
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"]
        _run(link + [obj[s] for s in SOURCES] + ["-o", LIB], verbose)
        _run(link + [obj[s] for s in PROBE_SOURCES] + ["-o", PROBE_LIB], verbose)
    return LIB


if __name__ == "__main__":
    build()
