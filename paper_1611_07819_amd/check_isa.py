"""Checks the compiler's output for this library's fp16 kernels against one hazard that the
compiler cannot see: the 16x16x32 matrix instructions of the fp16 pipeline are written as inline
assembly (their accumulators tied in place), so the compiler does not know that their results
take several cycles to land, and the hardware does not interlock a vector instruction that reads
an accumulator register against a matrix instruction still writing it.  Where the compiler
renames accumulators between differently scheduled parts of a k-loop it may therefore place a
copy (v_accvgpr_mov / v_accvgpr_read, or a store straight from an accumulator register) right
behind the matrix instruction that produces the value, and the copy reads the old contents.  The
pipeline drains the matrix cores (two s_nop 15) wherever it hands the accumulators to other code;
this check finds the copies that end up in front of such a drain.  The other direction: a matrix
instruction must not read an accumulator register in the cycle after a vector instruction wrote it;
the assembly statement carries a wait state (s_nop 0) for that except in the steady state of the
k-loop, where the compiler is expected to put no copy in front of it -- the check reports any
v_accvgpr_write / v_accvgpr_mov into a register that the very next instruction, a matrix
instruction, accumulates into.

    python -m paper_1611_07819_amd.check_isa            # compiles gemm_f16.hip and conv_mfma.hip

For every kernel that contains the inline-assembly instruction it walks the assembly in program
order (and once more across every backward branch, with the state at the branch) and reports any
instruction other than a matrix instruction that names an accumulator register written fewer
than WINDOW instructions earlier with no drain in between.  A 16x16x32 instruction occupies the
matrix core for 16 cycles and a wavefront issues at most one instruction per cycle (a vector or
matrix instruction every four), so WINDOW = 16 instructions is a safe distance.

Compiling the two sources to assembly takes about five minutes, so the test that runs this check
(tests/test_isa_hazards.py) only does so when DMATH_CHECK_ISA=1 is set; assembly files made
before can be given as arguments instead."""
import os
import re
import subprocess
import sys
import tempfile

from . import build as _build

WINDOW = 16
MFMA = "v_mfma_f32_16x16x32_f16"


def compile_to_asm(src: str, out_dir: str) -> str:
    """hipcc -S (device side only) with the library's own flags."""
    out = os.path.join(out_dir, os.path.basename(src) + ".s")
    cmd = (["hipcc"] + _build.HIP_FLAGS + ["-x", "hip", "--cuda-device-only", "-S", os.path.join(_build.CSRC, src),
                                           "-o", out])
    subprocess.run(cmd, check=True, stderr=subprocess.DEVNULL)
    return out


def _regs(text: str):
    """Accumulator registers an operand string names: a5, a[4:7]."""
    out = []
    for lo, hi in re.findall(r"\ba\[(\d+):(\d+)\]", text):
        out.extend(range(int(lo), int(hi) + 1))
    out.extend(int(r) for r in re.findall(r"\ba(\d+)\b", text))
    return out


def scan_function(lines):
    """lines: the instructions and labels of one kernel.  Returns [(line index, text, distance)]."""
    label_at = {l[:-1]: i for i, l in enumerate(lines) if l.endswith(":")}
    found = []

    def walk(start, stop, written, drained_at, base):
        # written: register -> position of the matrix instruction that wrote it (same scale as base + i)
        snapshots = []
        prev = ""
        for i in range(start, stop):
            l, pos = lines[i], base + (i - start)
            if l.endswith(":"):
                continue
            if l.startswith("s_nop 15"):
                drained_at = pos
                prev = l
                continue
            if l.startswith(MFMA):
                dst = re.match(MFMA + r"\s+(a\[\d+:\d+\])", l)
                acc = _regs(dst.group(1))
                if re.match(r"v_accvgpr_(write|mov)_b32\s+a(\d+)", prev) and int(re.match(r"\S+\s+a(\d+)", prev).group(1)) in acc:
                    found.append((i, prev + "  ->  " + l, 1))
                for r in acc:
                    written[r] = pos
                prev = l
                continue
            prev = l
            if l.startswith("v_mfma"):
                continue
            ops = l.split(None, 1)[1] if " " in l else ""
            for r in _regs(ops):
                w = written.get(r)
                if w is not None and pos - w < WINDOW and drained_at < w:
                    found.append((i, l, pos - w))
                    break
            m = re.match(r"s_c?branch\S*\s+(\S+)", l)
            if m and m.group(1) in label_at and label_at[m.group(1)] <= i:
                snapshots.append((label_at[m.group(1)], dict(written), drained_at, pos + 1))
        return snapshots

    for target, written, drained_at, pos in walk(0, len(lines), {}, -10 ** 9, 0):
        # once more from the top of each loop, as the instructions that follow the backward branch
        walk(target, min(len(lines), target + WINDOW + 8), written, drained_at, pos)
    return sorted(set(found))


def scan_file(path: str):
    """Returns {kernel name: [(index, instruction, distance)]} for the kernels with findings and
    the number of kernels looked at."""
    text = open(path).read()
    report, looked = {}, 0
    for name, body in re.findall(r"^(_Z\S+):[^\n]*\n(.*?)s_endpgm", text, re.S | re.M):
        if MFMA not in body:
            continue
        looked += 1
        lines = [l.split(";")[0].strip() for l in body.split("\n")]
        lines = [l for l in lines if l and (not l.startswith(".") or re.match(r"\.LBB\w+:", l))]
        bad = scan_function(lines)
        if bad:
            report[name] = bad
    return report, looked


def check(sources=("gemm_f16.hip", "conv_mfma.hip")):
    total, looked = {}, 0
    with tempfile.TemporaryDirectory() as tmp:
        for src in sources:
            rep, n = scan_file(compile_to_asm(src, tmp))
            total.update(rep)
            looked += n
    return total, looked


if __name__ == "__main__":
    if len(sys.argv) > 1:
        rep, looked = {}, 0
        for path in sys.argv[1:]:
            r, n = scan_file(path)
            rep.update(r)
            looked += n
    else:
        rep, looked = check()
    for name, bad in rep.items():
        print(name)
        for i, l, d in bad[:8]:
            print(f"    line {i}: {l}   ({d} instructions after the matrix instruction that writes it)")
    print(f"{looked} kernels with inline-assembly matrix instructions checked, {len(rep)} with early accumulator reads")
    sys.exit(1 if rep else 0)
