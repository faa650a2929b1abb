"""Compile the HIP library (csrc/*.hip and the .hpp parts they include -> libpqtopk.so, in-tree) for gfx950.

The translation units are compiled side by side (the scan kernels are large: tens of seconds each) and linked
into one shared library."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
OBJ = os.path.join(_HERE, "_build")                              # object files (not tracked)
SOURCES = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h")) + \
    sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp"))
LIB = os.path.join(_HERE, "libpqtopk.so")

# -packed-fp32-ops switches the packed FP32 instructions (v_pk_add_f32 and friends) off in the DEVICE code.  hipcc hands
# -Xclang options to its host pass as well, where the x86 back end answers with one line per function saying that it does
# not know the feature; those lines (and only those) are dropped from what the compiler prints.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                                       # the kernels spell out every fused multiply-add
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]
_HOST_PASS_NOISE = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(line for line in r.stdout.splitlines() if _HOST_PASS_NOISE not in line)
    if out.strip():
        print(out, file=sys.stderr, flush=True)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)


def build(force: bool = True, verbose: bool = False, jobs: int = 0) -> str:
    """Run hipcc.  Cross-compiles on a host without a GPU."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = [os.path.join(OBJ, os.path.basename(s)[:-4] + ".o") for s in SOURCES]
    newest_header = max(os.path.getmtime(h) for h in HEADERS)

    def compile_one(pair):
        src, obj = pair
        if not force and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            return
        _run([hipcc, *HIPCC_FLAGS, *inc, "-c", src, "-o", obj], verbose)

    jobs = jobs or min(len(SOURCES), max(1, min(int(os.environ.get("MAX_JOBS", "8")), os.cpu_count() or 1)))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(compile_one, zip(SOURCES, objs)))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], verbose)
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))
