"""Compile the HIP sources of this package into libmeda.so (gfx950) next to this file."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
LIB_PATH = os.path.join(PKG_DIR, "libmeda.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions out of ordinary float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # matrix products accumulate in ordinary vector registers: the scoring kernels read every accumulator
    # element with vector instructions, which would cost one extra move per element out of the accumulator file
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wno-unused-command-line-argument",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass reports that it does not know the device-only target feature: harmless
    err = "\n".join(line for line in res.stderr.splitlines() if "packed-fp32-ops" not in line)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build_library(verbose: bool = False, lib_path: str = LIB_PATH, extra_flags=()) -> str:
    """Every translation unit is compiled to an object file (in parallel), then linked."""
    from concurrent.futures import ThreadPoolExecutor
    sources = sorted(glob.glob(os.path.join(PKG_DIR, "csrc", "*.hip")))
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    obj_dir = os.path.join(PKG_DIR, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    tag = os.path.splitext(os.path.basename(lib_path))[0]
    objs = [os.path.join(obj_dir, f"{tag}.{os.path.splitext(os.path.basename(s))[0]}.o") for s in sources]
    common = [hipcc, *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include")]
    with ThreadPoolExecutor(max_workers=min(8, len(sources))) as pool:
        list(pool.map(lambda so: _run([*common, "-c", so[0], "-o", so[1]], verbose), zip(sources, objs)))
    _run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", lib_path, *objs], verbose)
    return lib_path


if __name__ == "__main__":
    print(build_library(verbose=True))
