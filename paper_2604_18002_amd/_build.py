"""Build the HIP libraries in-tree for gfx950: ``paper_2604_18002_amd/libngc.so`` (the method) and
``paper_2604_18002_amd/libngc_probe.so`` (streaming probes for the measurement harness)."""
from __future__ import annotations

import os
import shutil
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_PKG, "csrc")
LIB_PATH = os.path.join(_PKG, "libngc.so")
PROBE_LIB_PATH = os.path.join(_PKG, "libngc_probe.so")   # measurement probes, not part of the method

_COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
           # packed fp32 instructions stay off on the test machines
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]

# (source, extra flags).  The eviction units hold the exactly specified noise
# arithmetic: no contraction there.
_UNITS = (
    ("ngc_evict.hip", ["-ffp-contract=off"]),
    ("ngc_paged.hip", ["-ffp-contract=off"]),
    ("ngc_attn.hip", []),
    ("ngc_score.hip", []),
    ("ngc_replay.hip", []),
)
_PROBE_UNITS = (("ngc_probe.hip", []),)


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the HIP library cannot be built")
    return exe


def build(verbose: bool = False) -> str:
    """Compile every translation unit and link the shared library.  Always
    recompiles (this is the 'does it build' check)."""
    hipcc = _hipcc()
    bdir = os.path.join(_PKG, "_build")
    os.makedirs(bdir, exist_ok=True)
    for units, lib in ((_UNITS, LIB_PATH), (_PROBE_UNITS, PROBE_LIB_PATH)):
        objs = []
        for src, extra in units:
            obj = os.path.join(bdir, src.replace(".hip", ".o"))
            cmd = [hipcc, *_COMMON, *extra, "-c", os.path.join(_CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            r = subprocess.run(cmd, capture_output=True, text=True)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
            objs.append(obj)
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stderr}")
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
