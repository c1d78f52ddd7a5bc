"""Compile the HIP sources of the library into paper_2504_12329_amd/libst.so (gfx950 only)."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libst.so")
SOURCES = ["api.hip", "decode.hip", "prefill.hip", "trigger.hip", "persist.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    subprocess.run(["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=5) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    if verbose:
        print("built", LIB)
    return LIB


def build_stage_profiling():
    """The library with stage timestamps compiled into the persistent decode kernel (-DST_PERSIST_PROF), as
    _build/libst_prof.so; for persist_stages.py.  The other objects are those of the last build()."""
    os.makedirs(OBJ, exist_ok=True)
    obj = os.path.join(OBJ, "persist_prof.o")
    subprocess.run(["hipcc", *FLAGS, "-DST_PERSIST_PROF", "-DST_PERSIST_PROF_IN", "-c", os.path.join(CSRC, "persist.hip"),
                    "-o", obj], check=True)
    others = [os.path.join(OBJ, src.replace(".hip", ".o")) for src in SOURCES if src != "persist.hip"]
    lib = os.path.join(OBJ, "libst_prof.so")
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *others, obj], check=True)
    return lib


if __name__ == "__main__":
    build(verbose=True)
