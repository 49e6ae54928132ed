"""Build liblpk.so and the benchmark's yardstick library libmembw.so (gfx950 only) in-tree with hipcc.

    python -m paper_1810_05486_amd.build [--force]

Each source of liblpk is compiled to an object under csrc/_build/ and linked into
paper_1810_05486_amd/liblpk.so; csrc/membw.hip (memory-system yardsticks, used by
bench.py only, not part of the C ABI) becomes paper_1810_05486_amd/libmembw.so.
Nothing is built at import time: the bindings load the libraries that are there
and fail loudly when they are missing.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "liblpk.so")
MEMBW_SRC = os.path.join(CSRC, "membw.hip")
MEMBW_LIB = os.path.join(HERE, "libmembw.so")
SOURCES = ["lpk_host.hip", "kahan_step.hip", "momentum_step.hip", "adam_step.hip", "select_fraclen.hip", "quantize.hip",
           "noalloc_step.hip"]
HEADERS = [os.path.join(CSRC, "lpk_device.hpp"), os.path.join(CSRC, "step_common.hpp"), os.path.join(CSRC, "host_common.hpp"),
           os.path.join(HERE, "..", "include", "lpk.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Wall", "-Wno-unused-function",
         # packed fp32 VALU forms stay off: the compiler must not form v_pk_{add,mul,fma}_f32
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force=False, verbose=True):
    os.makedirs(OBJ, exist_ok=True)
    objs, jobs = [], []
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(OBJ, s.replace(".hip", ".o"))
        objs.append(obj)
        if force or _stale(obj, [src] + HEADERS):
            jobs.append([HIPCC] + FLAGS + ["-c", src, "-o", obj])
    if force or _stale(MEMBW_LIB, [MEMBW_SRC]):
        jobs.append([HIPCC] + FLAGS + ["-shared", MEMBW_SRC, "-o", MEMBW_LIB])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)

    with ThreadPoolExecutor(max_workers=4) as ex:
        list(ex.map(run, jobs))
    if force or _stale(LIB, objs):
        run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    build(force="--force" in sys.argv)
    print(LIB)
