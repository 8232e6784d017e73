"""Builds libfb4.so (the C-ABI library with its gfx950 kernels) in-tree with hipcc."""

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfb4.so")
OBJ_DIR = os.path.join(HERE, "_build")
# one translation unit per group of entry points, compiled side by side
SOURCES = [os.path.join(CSRC, f) for f in ("fb4_api.hip", "fb4_producers.hip", "fb4_attention.hip")]
DEPS = SOURCES + [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".hpp")] + [
    os.path.join(os.path.dirname(HERE), "include", "fb4.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 instructions stay off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the dispatcher fills up to 16 leading kernel-argument registers before a wavefront starts
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-Wall", "-Wno-unused-function",
]
# the host pass does not know the device-only feature flag and says so
NOISE = "is not a recognized feature for this target"


def up_to_date():
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    return all(os.path.getmtime(d) <= t for d in DEPS)


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if NOISE not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    return err


def build(force=True, verbose=False):
    """Compile the library.  force=False skips the compile when the library is newer than its sources."""
    if not force and up_to_date():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, os.path.basename(s)[:-4] + ".o") for s in SOURCES]
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
        errs = list(pool.map(lambda so: _run([hipcc] + HIPCC_FLAGS + ["-c", so[0], "-o", so[1]]), zip(SOURCES, objs)))
    errs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs))
    if verbose and any(e.strip() for e in errs):
        print("\n".join(e for e in errs if e.strip()), file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
