"""Build the HIP library in-tree: `python -m paper_2506_22668_amd.build`."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdistshap_hip.so")
OBJ = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "sampler.hip", "extract.hip", "eval.hip", "eval_zt.hip", "gat_eval.hip", "bitmat.hip", "tiles.hip",
           "gram_chol.hip", "cgls.hip", "fidelity.hip", "plan.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# The one flag list of the shipped code objects (tests that inspect the generated code import it).
COMPILE_FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-ffp-contract=off",
                 "-Wno-unused-value", "-Wno-unused-result",
                 # packed-fp32 VALU forms are kept out of the generated code on purpose
                 "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
_NOISE = "is not a recognized feature for this target"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if _NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)


def build_library(verbose=True, only=None):
    """Compile every source (or the ones named in `only`, reusing the other objects) and link."""
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, s + ".o") for s in SOURCES]
    todo = [(s, o) for s, o in zip(SOURCES, objs) if only is None or s in only or not os.path.exists(o)]
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        list(pool.map(lambda so: _run([HIPCC] + COMPILE_FLAGS + ["-c", os.path.join(CSRC, so[0]), "-o", so[1]],
                                      verbose), todo))
    _run([HIPCC, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", LIB] + objs, verbose)
    return LIB


if __name__ == "__main__":
    build_library(only=sys.argv[1:] or None)
    sys.exit(0)
