"""Developer check for the streaming kernels: transfer and unpack must overlap inside a wave.

The chunk transfers are issued from inline assembly and waited for explicitly (csrc/unpack.h).
A compiler-inserted `s_waitcnt vmcnt(..)` that lands between a transfer and the next explicit
wait makes the wave wait for the chunk it has just requested, which silently serializes the two
(the kernels stay correct, only slower).  This script compiles the kernel sources to assembly
with the library's flags and lists such waits per kernel; an empty list is the expected result.

    python -m paper_2512_24449_amd.check_waits
"""
import os
import re
import subprocess
import sys
import tempfile

from . import build

FILES = ("k_matvec.hip", "v_matvec.hip", "attn_decode.hip")


def stray_waits(asm_text):
    """-> {kernel: [(line number, instruction)]} of compiler waits that follow a transfer.
    Linear in layout order, so a listed wait still needs a look at its control flow; waits that
    an explicit wait follows within a few instructions and blocks outside the loops are skipped."""
    lines = asm_text.split("\n")
    found, kernel, pending, in_asm = {}, None, False, False
    for n, line in enumerate(lines, 1):
        m = re.match(r"^(_ZN6packkv\w*):", line)
        if m:
            kernel, pending = m.group(1), False
            found[kernel] = []
        if kernel is None:
            continue
        if re.match(r"^\.LBB\d+_\d+:", line) and "Loop" not in line:
            pending = False              # a block outside the loops: not reached from the transfer above
        if "#ASMSTART" in line:
            in_asm = True
        elif "#ASMEND" in line:
            in_asm = False
        elif "global_load_lds" in line:
            pending = True
        elif "s_waitcnt" in line and "vmcnt" in line:
            if in_asm:
                pending = False          # an explicit, counted wait
            elif pending:
                ahead = [l for l in lines[n:n + 40] if l.strip() and not l.strip().startswith(";") or "ASMSTART" in l]
                explicit_next = any("ASMSTART" in a and "s_waitcnt" in b for a, b in zip(ahead[:12], ahead[1:13]))
                if not explicit_next:
                    found[kernel].append((n, line.strip()))
        elif "s_endpgm" in line:
            kernel = None
    return found


def main():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    bad = 0
    with tempfile.TemporaryDirectory() as tmp:
        for name in FILES:
            out = os.path.join(tmp, name + ".s")
            subprocess.check_call([hipcc] + flags + ["-I", os.path.join(build.ROOT, "include"), "-I", build.CSRC,
                                                     "-S", "--cuda-device-only", os.path.join(build.CSRC, name), "-o", out],
                                  stderr=subprocess.DEVNULL)
            for kernel, waits in stray_waits(open(out).read()).items():
                short = re.sub(r"^_ZN6packkv\d+", "", kernel)
                print("%-14s %-44s %s" % (name, short[:44], waits if waits else "ok"))
                bad += len(waits)
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main())
