"""Builds liboctopus.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build" + os.environ.get("OCTOPUS_VARIANT", ""))
LIB = os.environ.get("OCTOPUS_LIB_OUT", os.path.join(HERE, "liboctopus.so"))

# one translation unit per head dimension and kernel family; a pool of workers compiles them in this order,
# the slowest (d = 256, then the matrix-core decode kernels) first
SOURCES = []
for _d in ("256", "128", "64"):
    SOURCES += [_family + _d + ".hip" for _family in ("octopus_d", "octopus_paged_d", "octopus_paged_qjl_d", "octopus_scores_d", "octopus_vq_d",
                                                      "octopus_valu_d", "octopus_qjl_d", "octopus_enc_d", "octopus_round_d")]
    SOURCES += ["octopus_vqm_d" + _d + "_b" + _b + ".hip" for _b in ("4", "3", "2")]
SOURCES += ["octopus_sweep_dec_d128.hip", "octopus_sweep_enc_d128.hip", "octopus_common.hip", "octopus_values.hip",
            "octopus_host.cpp"]
# -packed-fp32-ops is switched off on purpose: hipcc must not form packed fp32 instructions here.
FLAGS = (["-D" + d for d in os.environ.get("OCTOPUS_DEFS", "").split(",") if d]) + ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src):
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc()] + FLAGS + (["-x", "hip"] if src.endswith(".cpp") else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    return obj


def build(verbose=True, only=None):
    """Compile every source (or, for quick experiments, only those named in `only` / the environment
    variable OCTOPUS_ONLY, reusing the other objects of the last full build) and link liboctopus.so."""
    os.makedirs(OBJ, exist_ok=True)
    only = only or [s for s in os.environ.get("OCTOPUS_ONLY", "").split(",") if s]
    todo = [s for s in SOURCES if not only or s in only or
            not os.path.exists(os.path.join(OBJ, os.path.splitext(s)[0] + ".o"))]
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        list(pool.map(_compile, todo))
    objs = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    tmp = LIB + f".tmp{os.getpid()}"
    res = subprocess.run([_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs,
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    os.replace(tmp, LIB)
    if verbose:
        print(f"built {LIB}", file=sys.stderr)
    return LIB


if __name__ == "__main__":
    build()
