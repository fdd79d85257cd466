"""Build libcalidrop.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2507_19906_amd.build`."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libcalidrop.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # matrix-core results go straight to ordinary vector registers (saves the accumulator-register
    # copies in the kernels whose vector ALU is the busy unit)
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the CaliDrop kernels need the ROCm toolchain")


PROBES_PATH = os.path.join(PKG_DIR, "libcalidrop_probes.so")


def _compile(src: str, out: str, verbose: bool, extra_flags=()) -> str:
    tmp = out + ".tmp"
    cmd = [hipcc_path(), *HIPCC_FLAGS, *extra_flags, src, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    os.replace(tmp, out)
    return out


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile csrc/calidrop.hip into libcalidrop.so next to this file (and the machine probes the
    benchmark uses into libcalidrop_probes.so); returns the library's path."""
    _compile(os.path.join(CSRC, "probes.hip"), PROBES_PATH, verbose)
    return _compile(os.path.join(CSRC, "calidrop.hip"), LIB_PATH, verbose, extra_flags)


if __name__ == "__main__":
    print(build(verbose=True))
