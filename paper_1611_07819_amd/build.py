"""Builds libdmath.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdmath.so")
# measurement build: the fp16 GEMM kernel counts its own cycles (dmath_cycle_probe_read)
OBJ_PROBE = os.path.join(HERE, "_build_probe")
LIB_PROBE = os.path.join(HERE, "libdmath_probe.so")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")

# -packed-fp32-ops off: packed fp32 instructions are not to be generated on the test machines.
HIP_FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Xclang", "-target-feature",
             "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
             "-Wno-unknown-warning-option", "-I", INCLUDE]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith((".cpp", ".hip")))


def _newest_header():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")]
    hs += [os.path.join(INCLUDE, h) for h in os.listdir(INCLUDE) if h.endswith(".h")]
    return max(os.path.getmtime(h) for h in hs)


def _compile(src, force, probe=False):
    obj = os.path.join(OBJ_PROBE if probe else OBJ, src + ".o")
    path = os.path.join(CSRC, src)
    if (not force and os.path.exists(obj) and os.path.getmtime(obj) >= os.path.getmtime(path)
            and os.path.getmtime(obj) >= _newest_header()):
        return obj, False
    cmd = (["hipcc"] + HIP_FLAGS + (["-DDMATH_CYCLE_PROBE"] if probe else []) +
           (["-x", "hip"] if src.endswith(".hip") else []) + ["-c", path, "-o", obj])
    subprocess.run(cmd, check=True)
    return obj, True


def build(force: bool = False, verbose: bool = False, probe: bool = False) -> str:
    lib = LIB_PROBE if probe else LIB
    os.makedirs(OBJ_PROBE if probe else OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        res = list(ex.map(lambda s: _compile(s, force, probe), sources()))
    if force or any(changed for _, changed in res) or not os.path.exists(lib):
        cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib] + [o for o, _ in res]
        subprocess.run(cmd, check=True)
        if verbose:
            print("linked", lib)
    return lib


if __name__ == "__main__":
    import sys
    build(force="--force" in sys.argv, verbose=True, probe="--probe" in sys.argv)
