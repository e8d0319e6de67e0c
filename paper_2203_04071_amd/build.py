"""Build the HIP library (gfx950 only) in-tree with hipcc: one object per translation unit, compiled side by side."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libadapt_mi355.so")
SOURCES = [os.path.join(CSRC, f) for f in ("api_core.hip", "api_layers.hip", "api_i16.hip", "api_backward.hip")]
# ceiling probes for bench.py: a library of their own, not part of the product
PROBES_LIB = os.path.join(HERE, "libadapt_probes.so")
PROBES_SOURCE = os.path.join(CSRC, "probes.hip")
# translation units whose kernels issue loads from inline assembly (what isa_check.py scans)
HAND_SCHEDULED = [os.path.join(CSRC, "api_layers.hip")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                      # every fp32 step rounds where the code says it does
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources_newer_than_lib() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "adapt_mi355.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + r.stdout + r.stderr)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile csrc/*.hip into libadapt_mi355.so next to this file."""
    if not force and not sources_newer_than_lib():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, os.path.basename(s)[:-4] + ".o") for s in SOURCES]
    extra = os.environ.get("ADAPT_EXTRA_HIPCC_FLAGS", "").split()      # e.g. -DADAPT_TUNING_KNOBS for tuning experiments
    jobs = [[hipcc] + HIPCC_FLAGS + extra + ["-c", src, "-o", obj] for src, obj in zip(SOURCES, objs)]
    jobs.append([hipcc] + HIPCC_FLAGS + ["-shared", "-o", PROBES_LIB, PROBES_SOURCE])
    with ThreadPoolExecutor(max_workers=len(jobs)) as pool:
        list(pool.map(lambda cmd: _run(cmd, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
