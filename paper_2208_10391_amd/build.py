"""Build libmom.so (planner + gfx950 kernels) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmom.so")
SOURCES = [os.path.join(CSRC, f) for f in ("eval.hip", "plan.cpp", "product_nn.hip", "product_tn.hip",
                                            "product_nt.hip", "product_tt.hip")]


# Per-source additions to the compile line.  eval.hip holds the kernels whose accumulators are read
# out by other instructions than MFMAs (LDS writes of the skinny-pair kernel, the batched kernels'
# stores): there the accumulators stay in the vector registers proper, which those instructions can
# take as they are; from the accumulation registers every value would cost a vector move first.
EXTRA_FLAGS = {"eval.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _newest_source_mtime() -> float:
    paths = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    paths.append(os.path.join(os.path.dirname(HERE), "include", "mom.h"))
    return max(os.path.getmtime(p) for p in paths)


def is_built() -> bool:
    return os.path.exists(LIB)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile for gfx950: one object per source, side by side, then one shared library.
    With force=False an up-to-date library is kept."""
    if not force and is_built() and os.path.getmtime(LIB) >= _newest_source_mtime():
        return LIB
    import concurrent.futures
    import shutil
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-command-line-argument"]
    work = tempfile.mkdtemp(prefix="mom_build_")
    try:
        def compile_one(src):
            obj = os.path.join(work, os.path.basename(src) + ".o")
            cmd = [hipcc] + flags + EXTRA_FLAGS.get(os.path.basename(src), []) + ["-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 4, 8)) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        tmp = LIB + ".tmp.%d" % os.getpid()
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(work, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
