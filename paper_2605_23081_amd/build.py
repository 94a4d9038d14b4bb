"""Build the HIP library in-tree: hipcc for gfx950, one shared object next to this file."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libthrift_hip.so")
SOURCES = ["thrift_api.hip", "thrift_prepass.hip", "thrift_prefill.hip", "thrift_decode.hip", "thrift_cache.hip", "thrift_probe.hip"]
DMA_SOURCES = ["thrift_prefill.hip", "thrift_decode.hip"]      # kernels whose inline assembly sets M0 and keeps DMA in flight
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # NaN inputs are outside the contract (include/thrift.h); without this every maximum of matrix-unit results
         # is preceded by instructions that only quiet signalling NaNs
         "-fno-honor-nans",
         # packed-FP32 VALU forms are kept out of the generated code on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", INCLUDE, "-I", CSRC]


def scratch_in_loops(asm_text: str):
    """Kernel names whose generated code touches scratch memory (register spills) inside a loop.

    The fused kernel keeps LDS DMA in flight across key blocks; a spill reload inside the walk would sit in the
    same in-order memory queue and wait for those transfers at every block.  A spill that is stored before the
    walk and reloaded after it costs nothing.  The compiler's listing marks every basic block that belongs to a
    loop in the comment of its label line."""
    bad, kernel, depth = set(), None, 0
    kernels, blocks, loop_blocks = 0, 0, 0
    for line in asm_text.splitlines():
        t = line.strip()
        if t.startswith("_Z") and t.split(":")[0].isidentifier() and ":" in t:
            kernel, depth = t.split(":")[0], 0
            kernels += 1
        elif t.startswith(".LBB") or t.startswith("; %bb."):
            depths = [int(d) for d in re.findall(r"Depth=(\d+)", t)]
            depth = max(depths) if depths else 0
            blocks += 1
            loop_blocks += depth > 0
        elif t.startswith(";") and "Loop" in t and "Depth=" in t:
            # continuation lines of a label's comment: a nested loop's header names its parent first, itself below
            depth = max([depth] + [int(d) for d in re.findall(r"Depth=(\d+)", t)])
        elif t.startswith("scratch_") and kernel and depth >= (2 if "persistent" in kernel else 1):
            # in a persistent kernel the outermost loop is the loop over work items: a reload at an item's start or end
            # is outside the walk over the key blocks, like a reload before or after the walk of the other kernels
            bad.add(kernel)
    # The labels are the compiler's listing format, not a stable interface: a listing in which no kernel, no basic
    # block or no loop annotation is recognised cannot be checked and must not pass for clean.
    if kernels == 0 or blocks == 0 or loop_blocks == 0:
        raise RuntimeError("the prefill kernel's listing has no recognisable kernel labels / basic blocks / loop annotations: "
                           "the spill check cannot read this compiler's output")
    return sorted(bad)


def m0_outside_inline_asm(asm_text: str) -> int:
    """Number of compiler-generated instructions that touch M0.

    The LDS DMA instruction takes its LDS base from M0, which the inline assembly sets without the compiler knowing.
    That is sound only while the compiler itself never keeps a value in M0 across those statements: the fused
    kernel's listing must mention M0 nowhere but between the ASMSTART / ASMEND markers."""
    inside, count, statements, seen_inside = False, 0, 0, 0
    for line in asm_text.splitlines():
        t = line.strip()
        if t.startswith(";;#ASMSTART"):
            inside = True
            statements += 1
        elif t.startswith(";;#ASMEND"):
            inside = False
        elif not t.startswith(";") and "m0" in t.replace(",", " ").split():
            if inside:
                seen_inside += 1
            else:
                count += 1
    # the kernel does set M0 in its DMA statements: a listing in which that cannot be seen is in a format this check cannot read
    if statements == 0 or seen_inside == 0:
        raise RuntimeError("the prefill kernel's listing shows no inline-assembly markers around its M0 writes: "
                           "the M0 check cannot read this compiler's output")
    return count


def build(verbose: bool = False, extra=()):
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    # the device listings of the kernels that stage by LDS DMA, for the spill and M0 checks (run beside the object builds)
    listings = []
    for src in DMA_SOURCES:
        listing = os.path.join(CSRC, src.replace(".hip", ".gfx950.s"))
        lcmd = ["hipcc", *FLAGS, *extra, "-S", "--cuda-device-only", os.path.join(CSRC, src), "-o", listing]
        listings.append((src, listing, lcmd, subprocess.Popen(lcmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "not a recognized feature for this target" not in l)
        if p.returncode != 0:
            sys.stderr.write(out + "\n")
            raise RuntimeError("hipcc failed: " + " ".join(cmd))
        if verbose and out.strip():
            print(out)
    for src, listing, lcmd, lproc in listings:
        lout, _ = lproc.communicate()
        if lproc.returncode != 0:
            sys.stderr.write(lout + "\n")
            raise RuntimeError("hipcc failed: " + " ".join(lcmd))
        with open(listing) as f:
            text = f.read()
        os.remove(listing)
        spilling = scratch_in_loops(text)
        if spilling:
            raise RuntimeError(f"{src}: spilled registers are reloaded inside a loop: " + ", ".join(spilling))
        if m0_outside_inline_asm(text):
            raise RuntimeError(f"{src}: the compiler uses M0: the LDS DMA statements would clobber it")
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=tuple(sys.argv[1:])))
