"""Build libmom.so (planner + gfx950 kernels) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmom.so")
SOURCES = [os.path.join(CSRC, "eval.hip"), os.path.join(CSRC, "plan.cpp")]


def _newest_source_mtime() -> float:
    paths = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    paths.append(os.path.join(os.path.dirname(HERE), "include", "mom.h"))
    return max(os.path.getmtime(p) for p in paths)


def is_built() -> bool:
    return os.path.exists(LIB)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile for gfx950.  With force=False an up-to-date library is kept."""
    if not force and is_built() and os.path.getmtime(LIB) >= _newest_source_mtime():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument",
           "-o", tmp] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
