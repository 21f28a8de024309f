"""Checks the compiler's output for this library's pipelined fp16 and fp64 kernels against a
hazard that the compiler cannot see: their matrix instructions (v_mfma_f32_16x16x32_f16,
v_mfma_f64_16x16x4_f64) are written as inline assembly with the accumulators tied in place, so
the compiler does not know that their results take 16 / 64 cycles to land, and the hardware does
not interlock a vector instruction that reads an accumulator register against a matrix
instruction still writing it.  Where the compiler renames accumulators between differently
scheduled parts of a k-loop it may therefore place a copy (v_accvgpr_mov / v_accvgpr_read, or a
store straight from an accumulator register) right behind the matrix instruction that produces
the value, and the copy reads the old contents.  The pipelines drain the matrix cores (a run of
s_nop 15) wherever they hand the accumulators to other code; this check finds the copies that
end up in front of such a drain.  The other direction: a matrix instruction must not read an
accumulator register in the cycle after a vector instruction wrote it; the assembly statement
carries a wait state (s_nop 0) for that except in the steady state of the fp16 k-loop, where the
compiler is expected to put no copy in front of it -- the check reports any v_accvgpr_write /
v_accvgpr_mov into a register that the very next instruction, a matrix instruction, accumulates
into.  The fp64 pipelines, and the fp16 weight gradient of the convolution, go further and keep
their accumulators in fixed registers that the compiler knows nothing about (mfma.hpp): in a
kernel with fp64 matrix instructions, or with the comment that acc_fixed_marker() leaves, every
instruction that names an accumulation register must be one of the three forms the pipeline
writes itself (the matrix instruction, v_accvgpr_write_b32 aN, 0 and v_accvgpr_read_b32 vM, aN).

    python -m paper_1611_07819_amd.check_isa     # compiles gemm_f16.hip, gemm_f64.hip, conv_mfma.hip

For every kernel that contains such an instruction it walks the assembly in program order (and
once more across every backward branch, with the state at the branch), counting one cycle per
instruction -- a wavefront issues no faster -- and N+1 for s_nop N, and reports any instruction
other than a matrix instruction that names an accumulator register fewer than NEED cycles (the
instruction's occupancy of the matrix core plus four) after the matrix instruction that wrote it.

Compiling the sources to assembly takes several minutes, so the test that runs this check
(tests/test_isa_hazards.py) only does so when DMATH_CHECK_ISA=1 is set; assembly files made
before can be given as arguments instead."""
import os
import re
import subprocess
import sys
import tempfile

from . import build as _build

NEED = {"v_mfma_f32_16x16x32_f16": 20, "v_mfma_f64_16x16x4_f64": 68}
LOOKAHEAD = 96  # instructions re-walked from the top of a loop with the state at its backward branch


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


FIXED_MARKER = "dmath: fixed accumulation registers"  # comment left by acc_fixed_marker() (mfma.hpp)


def scan_function(lines, fixed=False):
    """lines: the instructions and labels of one kernel.  fixed: the kernel keeps its accumulators
    in fixed registers (every fp64 kernel does).  Returns [(line index, text, cycles)]."""
    label_at = {l[:-1]: i for i, l in enumerate(lines) if l.endswith(":")}
    found = []
    if fixed or any(l.startswith("v_mfma_f64_16x16x4_f64") for l in lines):
        own = re.compile(r"v_mfma_f64_16x16x4_f64 |v_mfma_f32_16x16x32_f16 a\[\d+:\d+\], v\[\d+:\d+\], v\[\d+:\d+\], a\[\d+:\d+\]$|"
                         r"v_accvgpr_write_b32 a\d+, 0$|v_accvgpr_read_b32 v\d+, a\d+$")
        for i, l in enumerate(lines):
            ops = l.split(None, 1)[1] if " " in l and not l.endswith(":") else ""
            if _regs(ops) and not own.match(l):
                found.append((i, l + "   (accumulation register used by the compiler)", 0))

    def walk(start, stop, written, clock):
        # written: register -> (cycle at which the matrix instruction that wrote it issued, cycles it needs)
        snapshots = []
        prev = ""
        for i in range(start, stop):
            l = lines[i]
            if l.endswith(":"):
                continue
            nop = re.match(r"s_nop\s+(\d+)", l)
            clock += int(nop.group(1)) + 1 if nop else 1
            name = l.split()[0]
            if name in NEED:
                acc = _regs(re.match(r"\S+\s+(a\[\d+:\d+\])", l).group(1))
                if re.match(r"v_accvgpr_(write|mov)_b32\s+a(\d+)", prev) and int(re.match(r"\S+\s+a(\d+)", prev).group(1)) in acc:
                    found.append((i, prev + "  ->  " + l, 1))
                for r in acc:
                    written[r] = (clock, NEED[name])
                prev = l
                continue
            prev = l
            if name.startswith("v_mfma"):
                continue
            ops = l.split(None, 1)[1] if " " in l else ""
            for r in _regs(ops):
                w = written.get(r)
                if w is not None and clock - w[0] < w[1]:
                    found.append((i, l, clock - w[0]))
                    break
            m = re.match(r"s_c?branch\S*\s+(\S+)", l)
            if m and m.group(1) in label_at and label_at[m.group(1)] <= i:
                snapshots.append((label_at[m.group(1)], dict(written), clock))
        return snapshots

    for target, written, clock in walk(0, len(lines), {}, 0):
        # once more from the top of each loop, as the instructions that follow the backward branch
        walk(target, min(len(lines), target + LOOKAHEAD), written, clock)
    return sorted(set(found))


def scan_file(path: str):
    """Returns {kernel name: [(index, instruction, distance)]} for the kernels with findings and
    the number of kernels looked at."""
    text = open(path).read()
    report, looked = {}, 0
    for name, body in re.findall(r"^(_Z\S+):[^\n]*\n(.*?)s_endpgm", text, re.S | re.M):
        if not any(name in body for name in NEED):
            continue
        looked += 1
        lines = [l.split(";")[0].strip() for l in body.split("\n")]
        lines = [l for l in lines if l and (not l.startswith(".") or re.match(r"\.LBB\w+:", l))]
        bad = scan_function(lines, fixed=FIXED_MARKER in body)
        if bad:
            report[name] = bad
    return report, looked


def check(sources=("gemm_f16.hip", "gemm_f64.hip", "conv_mfma.hip")):
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
            print(f"    line {i}: {l}   ({d} cycles at most after the matrix instruction that writes it)")
    print(f"{looked} kernels with inline-assembly matrix instructions checked, {len(rep)} with early accumulator reads")
    sys.exit(1 if rep else 0)
