"""Builds libvista.so in-tree with hipcc for gfx950 (cross-compiles without a GPU).

    python -m paper_2510_22049_amd.build

Every translation unit under csrc/ is compiled to an object (in parallel) and
linked into paper_2510_22049_amd/libvista.so, the one library the binding loads;
calibrate.hip (the benchmark's calibration kernels, not on the product path)
becomes libvista_calibrate.so, a library of its own.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libvista.so")
CAL_LIB = os.path.join(HERE, "libvista_calibrate.so")
CAL_SRC = "calibrate.hip"
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# Packed-fp32 instructions are switched off for all device code on the test machines.
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-ignored-attributes",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src[:-4] + ".o")
    extra = os.environ.get("VISTA_EXTRA_HIPCC_FLAGS", "").split()   # developer knob (-D... for experiments)
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as ex:
        objs = list(ex.map(_compile, sources()))
    srcs = sources()
    for lib, group in ((LIB, [o for o, f in zip(objs, srcs) if f != CAL_SRC]),
                       (CAL_LIB, [o for o, f in zip(objs, srcs) if f == CAL_SRC])):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *group, "-o", lib]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
        if verbose:
            print(f"built {lib} from {len(group)} sources")
    return LIB


if __name__ == "__main__":
    build()
