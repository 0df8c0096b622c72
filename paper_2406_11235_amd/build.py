"""Build libqtip.so for gfx950 with hipcc (cross-compiles without a GPU)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqtip.so")
SOURCES = ["qtip_api.hip", "qtip_decode.hip", "qtip_lut14.hip", "qtip_rht.hip", "qtip_viterbi.hip", "qtip_ldlq.hip", "qtip_quantize.cpp"]
HEADERS = ["qtip_device.h", "qtip_rht_device.h", "qtip_internal.h", os.path.join("..", "..", "include", "qtip.h")]

# Packed-FP32 VALU forms are switched off for every device compile.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.abspath(__file__)]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force=True, extra_flags=(), verbose=False, out=None, jobs=None):
    """Compile every source into paper_2406_11235_amd/libqtip.so (or `out`): one hipcc
    process per source file, a few at a time, then one link."""
    if out is None and not force and not is_stale():
        return LIB
    import concurrent.futures
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    compile_flags = [f for f in FLAGS if f != "-shared"] + list(extra_flags)
    jobs = jobs or min(len(SOURCES), max(1, (os.cpu_count() or 2) - 1))
    scratch = os.path.join(HERE, "_build")  # object files only; removed again below
    os.makedirs(scratch, exist_ok=True)
    with tempfile.TemporaryDirectory(prefix="obj_", dir=scratch) as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, os.path.splitext(src)[0] + ".o")
            cmd = [hipcc] + compile_flags + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), file=sys.stderr)
            subprocess.run(cmd, check=True)
            return obj
        with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread"] + objs + ["-o", out or LIB]
        if verbose:
            print(" ".join(link), file=sys.stderr)
        subprocess.run(link, check=True)
    return out or LIB


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
