"""Build libpfc.so and libpfc_probe.so (hand-written HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2203_15565_amd.build        # compiles every source, links the library
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpfc.so")
SOURCES = ["pfc_api.hip", "pfc_sample.hip", "pfc_fwd_bwd.hip", "pfc_update.hip"]
# calibration probes of the benchmark: a library of their own, not part of the product ABI
PROBE_LIB = os.path.join(HERE, "libpfc_probe.so")
PROBE_SOURCES = ["pfc_probe.hip"]

# -packed-fp32-ops off: the compiler must not form v_pk_*_f32 from ordinary float code.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in proc.stdout.splitlines()
             if "is not a recognized feature for this target" not in l]
    if proc.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), "\n".join(lines)))
    return "\n".join(lines)


def build(verbose: bool = False) -> str:
    """Compile all sources (always, even if a library exists) and link libpfc.so."""
    hipcc = _hipcc()
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]
    probe_objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in PROBE_SOURCES]

    def compile_one(pair):
        src, obj = pair
        out = _run([hipcc, *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
        if verbose and out.strip():
            print(out)

    with ThreadPoolExecutor(max_workers=4) as ex:
        list(ex.map(compile_one, zip(SOURCES + PROBE_SOURCES, objs + probe_objs)))
    for lib, lobjs in ((LIB, objs), (PROBE_LIB, probe_objs)):
        out = _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *lobjs])
        if verbose and out.strip():
            print(out)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
