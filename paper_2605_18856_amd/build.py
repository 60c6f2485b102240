"""Build libbsse.so (gfx950 only) in-tree with hipcc.

    python -m paper_2605_18856_amd.build [--force]

Each .hip file is compiled to an object, then linked into
``paper_2605_18856_amd/libbsse.so``.  hipcc cross-compiles without a GPU present.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbsse.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

SOURCES = ["bsse_api.hip", "gen_kernels.hip", "sweep_valu.hip", "sweep_mfma.hip", "sweep_small.hip", "reduce.hip", "prior_batch.hip", "profile_lp.hip", "topk.hip", "ceilings.hip"]
HEADERS = [os.path.join(CSRC, "bsse_internal.h"), os.path.join(CSRC, "mfma_device.h"),
           os.path.join(os.path.dirname(HERE), "include", "bsse.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
         "-Wno-unused-parameter",
         # correctly rounded fp32 division (the lattice points are defined by it)
         "-fhip-fp32-correctly-rounded-divide-sqrt",
         # no packed-fp32 VALU forms
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    jobs = []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, src.replace(".hip", ".o"))
        if force or _stale(o, [s] + HEADERS):
            jobs.append([HIPCC] + FLAGS + ["-c", s, "-o", o])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)

    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        list(ex.map(run, jobs))
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    if force or jobs or _stale(LIB, objs):
        run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
