"""Compile the HIP sources into librtoss.so for gfx950 with hipcc (cross-compiles without a GPU)."""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librtoss.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # never emit packed-fp32 VALU ops
    "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-unknown-warning-option", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _compile_one(args):
    hipcc, src, obj = args
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    cmd = [hipcc] + flags + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj]
    subprocess.check_call(cmd)
    return obj


def build_library(verbose=True):
    """Compiles every source to an object (in parallel: the files are independent) and links them."""
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp%d" % os.getpid()
    srcs = sources()
    jobs = max(1, min(len(srcs), int(os.environ.get("MAX_JOBS", "0")) or (os.cpu_count() or 4), 8))
    with tempfile.TemporaryDirectory(prefix="rtoss_build_") as objdir:
        work = [(hipcc, s, os.path.join(objdir, os.path.basename(s) + ".o")) for s in srcs]
        if verbose:
            print("hipcc %s -c {%s}  (%d jobs)" % (" ".join(f for f in HIPCC_FLAGS if f != "-shared"),
                                                 ", ".join(os.path.basename(s) for s in srcs), jobs), flush=True)
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            objs = list(pool.map(_compile_one, work))
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
        if verbose:
            print(" ".join(link[:6]) + " <%d objects>" % len(objs), flush=True)
        subprocess.check_call(link)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
