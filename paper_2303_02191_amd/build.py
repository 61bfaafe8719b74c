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
    not see.  Two hazards slip through that way, and both were observed to corrupt results:
    (1) a v_accvgpr_read (or v_accvgpr_mov) -- the instruction with which the register allocator brings back a
        value it had parked in the accumulation registers -- writing a vector register that an asm matrix
        instruction reads right afterwards.  Those moves run through the matrix pipeline, and nothing interlocks
        the matrix instruction's operand read against them.  (Ordinary vector-ALU results, e.g. a v_perm_b32
        directly in front of the matrix instruction that consumes it, are interlocked: kernels with that pattern
        match the oracle bit for bit.)  Two instructions in between were seen to be enough; the scan flags anything
        closer than five instructions apart.
    (2) an accumulator move (v_accvgpr_read / _mov / _write, or a spill reload into accumulation registers) that
        touches the destination of an asm matrix instruction issued fewer than 20 cycles before: the compiler
        shuffles accumulators where control-flow paths with different register assignments join, and it does not
        know that the asm statement in front is still writing them.  (The kernels' own reads of the accumulators
        come behind two s_nop 15.)
    Returns the offending (first, second) instruction pairs.
    """
    import re

    def regs(tok, cls="v"):
        tok = tok.strip().split()[0] if tok.strip() else ""
        m = re.match(cls + r"\[(\d+):(\d+)\]$", tok)
        if m:
            return set(range(int(m.group(1)), int(m.group(2)) + 1))
        m = re.match(cls + r"(\d+)$", tok)
        return {int(m.group(1))} if m else set()

    found, window, in_asm = [], [], False
    recent_dest = []  # [cycles since issue, accumulator registers written, text] of asm matrix instructions
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
        cost = 1
        if op == "s_nop":  # s_nop N idles N + 1 cycles
            cost = (int(line.split()[1]) if len(line.split()) > 1 and line.split()[1].isdigit() else 0) + 1
        is_asm_matrix = in_asm and (op.startswith("v_mfma") or op.startswith("v_smfmac"))
        # ---- (2) accumulator moves behind an asm matrix instruction ----
        touched = set()
        if op.startswith("v_accvgpr") or (op.startswith("scratch_load") or op.startswith("global_load") or op.startswith("ds_read")):
            for tok in line.split(None, 1)[1].split(",") if len(line.split(None, 1)) > 1 else []:
                touched |= regs(tok, "a")
        if touched and not is_asm_matrix:
            for age, dest, text in recent_dest:
                if age < 20 and (dest & touched):
                    found.append((text, line))
                    break
        for entry in recent_dest:
            entry[0] += cost
        recent_dest = [e for e in recent_dest if e[0] < 20]
        if is_asm_matrix:
            operands = line.split(None, 1)[1].split(",")
            recent_dest.append([0, regs(operands[0], "a"), line])
            # ---- (1) parked values restored in front of the instruction ----
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
        if op == "s_nop":
            window += ["s_nop"] * cost
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
                raise RuntimeError("%s: %d register hazard(s) around asm matrix instructions, e.g. `%s` -> `%s`; "
                                   "lower the register pressure of the kernel, keep accumulators out of control-flow joins, "
                                   "or define RTOSS_MFMA_SETTLE for this file"
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
