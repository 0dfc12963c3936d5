"""Build libmpk.so (host compiler + HIP runtime) for gfx950, in-tree.

The kernels come in specialised sets (head_dim, query heads per KV head, batch class, mixture of
experts); csrc/variants.hip is compiled once per set, in parallel, and the objects are linked with
the host side.  Objects go to _build/ next to this file (not committed)."""
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_OBJ = os.path.join(_HERE, "_build")
LIB = os.path.join(_HERE, "libmpk.so")
SOURCES = [os.path.join(_CSRC, f) for f in ("compiler.cpp", "runtime.hip", "variants.hip")]
HEADERS = [os.path.join(_CSRC, "mpk_internal.h"), os.path.join(_CSRC, "kernels.h"),
           os.path.join(os.path.dirname(_HERE), "include", "mpk.h")]
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
         "-I" + os.path.join(os.path.dirname(_HERE), "include"),
         # packed fp32 instructions are not to be generated on this machine pool
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _n_variants() -> int:
    with open(os.path.join(_CSRC, "kernels.h")) as f:
        return int(re.search(r"kNumVariants\s*=\s*(\d+)", f.read()).group(1))


def _compile(job):
    src, obj, extra = job
    subprocess.check_call(["hipcc", *FLAGS, *extra, "-c", src, "-o", obj],
                          stderr=subprocess.DEVNULL if os.environ.get("MPK_BUILD_QUIET") else None)
    return obj


def build(force: bool = True, jobs: int = 8) -> str:
    """Compile the library.  force=False rebuilds only when a source is newer than the library."""
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(p) for p in SOURCES + HEADERS)
        if os.path.getmtime(LIB) >= newest:
            return LIB
    os.makedirs(_OBJ, exist_ok=True)
    work = [(SOURCES[0], os.path.join(_OBJ, "compiler.o"), []),
            (SOURCES[1], os.path.join(_OBJ, "runtime.o"), [])]
    work += [(SOURCES[2], os.path.join(_OBJ, f"variant{i}.o"), [f"-DMPK_VARIANT_INDEX={i}"])
             for i in range(_n_variants())]
    # the generic fallbacks take longest: start them first
    work.sort(key=lambda j: 0 if j[1].endswith(("variant6.o", "variant7.o")) else 1)
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(work)))) as pool:
        objs = list(pool.map(_compile, work))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB])
    return LIB


if __name__ == "__main__":
    print(build())
