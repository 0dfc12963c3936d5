"""Build libmpk.so (host compiler + HIP runtime) for gfx950, in-tree."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(_HERE, "libmpk.so")
SOURCES = [os.path.join(_HERE, "csrc", f) for f in ("compiler.cpp", "runtime.hip")]
HEADERS = [os.path.join(_HERE, "csrc", "mpk_internal.h"),
           os.path.join(os.path.dirname(_HERE), "include", "mpk.h")]


def build(force: bool = True) -> str:
    """Compile the library.  force=False rebuilds only when a source is newer than the library."""
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(p) for p in SOURCES + HEADERS)
        if os.path.getmtime(LIB) >= newest:
            return LIB
    cmd = ["hipcc", "-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC",
           "-I" + os.path.join(os.path.dirname(_HERE), "include"),
           # packed fp32 instructions are not to be generated on this machine pool
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           *SOURCES, "-o", LIB]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
