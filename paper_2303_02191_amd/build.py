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


def check_matrix_hazards(asm_path):
    """Scans the device assembly the compiler generated for one source file.

    The kernels issue their matrix instructions as asm statements, which the compiler's hazard handling does
    not see.  One hazard slips through that way, and it was observed to corrupt results: a v_accvgpr_read (or
    v_accvgpr_mov) -- the instruction with which the register allocator brings back a value it had parked in the
    accumulation registers -- writing a vector register that an asm matrix instruction reads right afterwards.
    Those moves run through the matrix pipeline, and nothing interlocks the matrix instruction's operand read
    against them.  (Ordinary vector-ALU results, e.g. a v_perm_b32 directly in front of the matrix instruction
    that consumes it, are interlocked: kernels with that pattern match the oracle bit for bit.)  Returns the
    offending (writer, matrix instruction) pairs.  Two instructions in between were seen to be enough; the scan
    flags anything closer than five instructions apart.
    """
    import re

    def regs(tok):
        tok = tok.strip().split()[0] if tok.strip() else ""
        m = re.match(r"v\[(\d+):(\d+)\]$", tok)
        if m:
            return set(range(int(m.group(1)), int(m.group(2)) + 1))
        m = re.match(r"v(\d+)$", tok)
        return {int(m.group(1))} if m else set()

    found, window, in_asm = [], [], False
    for raw in open(asm_path, errors="replace"):
        line = raw.strip()
        if line.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if line.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not line or line[0] in ";." or line.endswith(":"):
            continue
        op = line.split()[0]
        if in_asm and (op.startswith("v_mfma") or op.startswith("v_smfmac")):
            operands = line.split(None, 1)[1].split(",")
            sources = set()
            for tok in operands[1:]:
                sources |= regs(tok)
            for prev in window:
                pop = prev.split()[0]
                if pop.startswith("v_accvgpr_read") or pop.startswith("v_accvgpr_mov"):
                    if regs(prev.split(None, 1)[1].split(",")[0]) & sources:
                        found.append((prev, line))
            window = []  # (a matrix instruction in between is far more than two wait states)
            continue
        if op == "s_nop":  # s_nop N idles N + 1 cycles
            n = int(line.split()[1]) if len(line.split()) > 1 and line.split()[1].isdigit() else 0
            window += ["s_nop"] * (n + 1)
        else:
            window.append(line)
        window = window[-4:]
    return found


def _compile_one(args):
    hipcc, src, obj = args
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    # -save-temps leaves the device assembly next to the object: input of the hazard scan
    cmd = [hipcc] + flags + ["-save-temps", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj]
    subprocess.check_call(cmd, cwd=os.path.dirname(obj), stderr=subprocess.DEVNULL if os.environ.get("RTOSS_QUIET_BUILD") else None)
    stem = os.path.splitext(os.path.basename(src))[0]
    for f in os.listdir(os.path.dirname(obj)):
        if f.startswith(stem + "-hip-amdgcn") and f.endswith(".s"):
            bad = check_matrix_hazards(os.path.join(os.path.dirname(obj), f))
            if bad:
                raise RuntimeError("%s: %d matrix instruction(s) read a vector-ALU result too early, e.g. `%s` -> `%s`; "
                                   "lower the register pressure of the kernel or define RTOSS_MFMA_SETTLE for this file"
                                   % (os.path.basename(src), len(bad), bad[0][0], bad[0][1]))
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
