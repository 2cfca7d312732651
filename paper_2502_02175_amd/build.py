"""Builds libvlac.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libvlac.so")
SOURCES = ["api.hip", "select.hip", "embed.hip", "rows.hip", "gemm.hip", "gemm_tall.hip", "attn.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-I" + os.path.join(ROOT, "include"), "-I" + SRC,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), err))
    return err


# The sources that place waits for compiler-invisible copies by hand; libvlac_safe.so is the
# same library with those sources compiled with -DVLAC_SAFE_WAITS (every such wait is for all
# outstanding loads): a checking aid that a GPU test compares with libvlac.so bit for bit.
HAND_WAITS = ["gemm_tall.hip", "attn.hip"]
LIB_SAFE = os.path.join(HERE, "libvlac_safe.so")


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    jobs = [(s, os.path.join(OBJ, s.replace(".hip", ".o")), []) for s in SOURCES]
    jobs += [(s, os.path.join(OBJ, s.replace(".hip", ".safe.o")), ["-DVLAC_SAFE_WAITS"]) for s in HAND_WAITS]
    with ThreadPoolExecutor(max_workers=8) as ex:
        list(ex.map(lambda j: _run([hipcc, *FLAGS, *j[2], "-c", os.path.join(SRC, j[0]), "-o", j[1]]), jobs))
    objs = [j[1] for j in jobs if not j[2]]
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    safe = [o.replace(".o", ".safe.o") if os.path.basename(o).replace(".o", ".hip") in HAND_WAITS else o for o in objs]
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_SAFE, *safe])
    if verbose:
        print("built", LIB, "and", LIB_SAFE)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
