#!/usr/bin/env python3
"""Build-time check of the hand-scheduled loads in pointwise_ring_kernel.

The kernel issues its residual and bias loads through inline assembly so that the compiler
does not count them (it would otherwise drain the LDS ring before their first use), waits for
them by hand and only then "redefines" the destination registers with an empty asm statement.
Between the load and that wait the compiler believes the registers already hold the data.
Nothing stops it, in principle, from copying or reusing them there; this script compiles the
kernels to assembly and fails if any instruction between the first such load and the wait that
covers them reads or writes one of the destination registers, or if one of the loads takes its
address from such a register.

Usage: check_async_loads.py [kernels.s]   (without an argument it compiles kernels.hip itself)
"""
import os
import re
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
KERNELS = ("pointwise_ring_kernelILi1E", "pointwise_ring_kernelILi2E")
HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-S", "--cuda-device-only"]


def compile_to_asm(out_path):
    cmd = ["hipcc", *HIPCC_FLAGS, "-I", os.path.join(HERE, "..", "..", "include"), "-o", out_path,
           os.path.join(HERE, "kernels.hip")]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)


def vregs(text):
    """Vector registers named in an operand string."""
    out = set()
    for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", text):
        out |= set(range(int(a), int(b) + 1))
    out |= {int(a) for a in re.findall(r"\bv(\d+)\b", text)}
    return out


LOAD = re.compile(r"\s*global_load_dwordx[24]\s+(v\[\d+:\d+\]),\s*(v\[\d+:\d+\])")


def check_kernel(asm, name):
    m = re.search(r"^_ZN4npas\d+%s.*?:\n(.*?)s_endpgm" % name, asm, re.S | re.M)
    if not m:
        return ["kernel %s not found in the assembly" % name]
    lines = m.group(1).split("\n")
    loads = [i for i, l in enumerate(lines) if LOAD.match(l)]
    if not loads:
        return ["%s: no asm loads found (has the kernel changed? update this check)" % name]
    dest = set()
    for i in loads:
        dest |= vregs(LOAD.match(lines[i]).group(1))
    end = next((i for i in range(loads[-1], len(lines)) if "s_waitcnt vmcnt(" in lines[i]), None)
    if end is None:
        return ["%s: no wait after the asm loads" % name]
    problems = []
    seen = set()
    for i in range(loads[0], end):
        l = lines[i].split(";")[0]
        if not l.strip() or l.strip().startswith("."):
            continue
        lm = LOAD.match(l)
        if lm:
            if vregs(lm.group(2)) & (dest - vregs(lm.group(1))) & seen:
                problems.append("%s: load address in a register still being loaded: %s" % (name, l.strip()))
            seen |= vregs(lm.group(1))
            continue
        if vregs(l) & seen:
            problems.append("%s: register touched before its load is awaited: %s" % (name, l.strip()))
    return problems


def main(argv):
    if len(argv) > 1:
        asm = open(argv[1]).read()
    else:
        with tempfile.TemporaryDirectory() as d:
            path = os.path.join(d, "kernels.s")
            compile_to_asm(path)
            asm = open(path).read()
    problems = []
    for k in KERNELS:
        problems += check_kernel(asm, k)
    for p in problems:
        print(p)
    print("async-load check: %s" % ("FAILED" if problems else "ok"))
    return 1 if problems else 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
