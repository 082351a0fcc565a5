"""Build libgf.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgf.so")
OBJ = os.path.join(HERE, "_build")
PROBE_SRC = os.path.join(HERE, "csrc_probe", "gf_probe.hip")
PROBE_LIB = os.path.join(HERE, "libgf_probe.so")

# -packed-fp32-ops off: hand the compiler no packed-FP32 forms (they are not trusted on this target)
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False) -> str:
    """Compile every translation unit (in parallel) and link libgf.so. Always rebuilds."""
    os.makedirs(OBJ, exist_ok=True)
    cc = _hipcc()

    def one(src):
        obj = os.path.join(OBJ, os.path.basename(src) + ".o")
        cmd = [cc, *HIPCC_FLAGS, "-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(one, sources()))
    r = subprocess.run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    # the measurement probes of bench.py --ceilings: a library of their own, never loaded by the product path
    r = subprocess.run([cc, *HIPCC_FLAGS, "-shared", PROBE_SRC, "-o", PROBE_LIB], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for the probes:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
