"""Builds ``libpatdnn.so`` (the C-ABI library) for gfx950 with hipcc, in-tree.

Steps: generate the pattern-specialised FMA bodies for every sparse variant listed in
``csrc/variants.def`` (``csrc/gen_dispatch.py``), compile each translation unit, link.
hipcc cross-compiles without a GPU.  Packed-FP32 code generation is switched off.
"""

from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libpatdnn.so")
PROBES_LIB = os.path.join(HERE, "libpatdnn_probes.so")     # bench-side measurement probes
SOURCES = ["patdnn_api.hip", "kernel_fkw.hip", "kernel_dw.hip", "kernel_compare.hip", "kernel_tiled.hip", "selftest.hip", "encoder.cpp", "projection.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sparse_geometries():
    """(G, PR, PC, S, TGX, MODE) of every non-dense X(...) line of variants.def."""
    geos = set()
    with open(os.path.join(CSRC, "variants.def")) as f:
        for line in f:
            if line.lstrip().startswith("//"):
                continue
            m = re.search(r"X\(\s*\w+\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(true|false)"
                          r"\s*,\s*\d+\s*,\s*(\d+)", line)
            if m and m.group(6) == "false":
                g = [int(m.group(i)) for i in (1, 2, 3, 4, 5, 7)]
                g[5] &= 15          # MODE bit 4 belongs to the kernel; the interpreter is shared
                geos.add(tuple(g))
    return sorted(geos)


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + FLAGS + (["-x", "hip"] if src.endswith(".cpp") else []) + \
          ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    sys.path.insert(0, CSRC)
    try:
        import gen_dispatch
        gen_dispatch.main(["gen_dispatch", os.path.join(CSRC, "gen")] +
                          [",".join(str(v) for v in g) for g in sparse_geometries()])
    finally:
        sys.path.pop(0)
    sources = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    with ThreadPoolExecutor(max_workers=min(8, len(sources))) as ex:
        objs = list(ex.map(_compile, sources))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    # the measurement probes bench.py times beside the kernels: a library of their own
    probe_obj = _compile("bench_probes.hip")
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PROBES_LIB, probe_obj],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    if verbose:
        print(f"built {LIB} and {PROBES_LIB}")
    return LIB


if __name__ == "__main__":
    build(verbose=True)
