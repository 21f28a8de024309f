"""ctypes front end of the CPU oracle (``dmath_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the benchmark's
``cpu_baseline`` leg.  Nothing on the product path may import this module, and this module
imports nothing from the GPU package.

The oracle is the textbook definition of the operations that the paper names in its abstract
(matrix multiplication, convolution) on matrices cut into non-overlapping blocks (section 2.1),
in the storage precisions of section 1 (d) (double, float, half), with all arithmetic in fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dmath_oracle.c")
_LIB = os.path.join(_HERE, "libdmath_oracle.so")

_DTYPE_CODE = {np.dtype(np.float64): 0, np.dtype(np.float32): 1, np.dtype(np.float16): 2}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (portable x86-64 code: the library is built on one machine
    and may run on another, so no -march=native)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _OMat(ctypes.Structure):
    _fields_ = [
        ("rows", ctypes.c_int64),
        ("cols", ctypes.c_int64),
        ("grid_r", ctypes.c_int32),
        ("grid_c", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("pad_", ctypes.c_int32),
        ("blocks", ctypes.POINTER(ctypes.c_void_p)),
    ]


class _OConv(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n", "c", "h", "w", "k", "r", "s", "pad_h", "pad_w", "stride_h", "stride_w")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        i64, dbl, p = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        pm = ctypes.POINTER(_OMat)
        _lib.oracle_gemm.restype = ctypes.c_int
        _lib.oracle_gemm.argtypes = [ctypes.c_int, ctypes.c_int, dbl, pm, pm, dbl, pm,
                                     i64, i64, i64, i64, p, p]
        for name in ("oracle_conv_fwd", "oracle_conv_bwd_filter", "oracle_conv_bwd_data"):
            fn = getattr(_lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [ctypes.POINTER(_OConv), dbl, pm, pm, dbl, pm, i64, p, p]
        _lib.oracle_half_to_double.restype = dbl
        _lib.oracle_half_to_double.argtypes = [ctypes.c_uint16]
        _lib.oracle_num_threads.restype = ctypes.c_int
        _lib.oracle_part_valid.restype = ctypes.c_int
        _lib.oracle_part_valid.argtypes = [i64, ctypes.c_int32]
        _lib.oracle_conv_out_dims.restype = ctypes.c_int
        _lib.oracle_conv_out_dims.argtypes = [ctypes.POINTER(_OConv), ctypes.POINTER(i64),
                                              ctypes.POINTER(i64)]
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def half_to_double(bits: int) -> float:
    return float(lib().oracle_half_to_double(bits))


def split_bounds(n: int, g: int):
    """Part p of g along a dimension of length n covers [p*ceil(n/g), min(n,(p+1)*ceil(n/g)))."""
    step = -(-n // g)
    return [(p * step, min(n, (p + 1) * step)) for p in range(g)]


class BlockMatrix:
    """A dense 2-D array cut into a grid of separately stored, contiguous row-major blocks
    (section 2.1).  Holds the block arrays alive for the C side."""

    def __init__(self, dense: np.ndarray, grid=(1, 1)):
        dense = np.asarray(dense)
        if dense.ndim != 2 or dense.dtype not in _DTYPE_CODE:
            raise ValueError("BlockMatrix wants a 2-D float64/float32/float16 array")
        self.rows, self.cols = dense.shape
        self.grid = (int(grid[0]), int(grid[1]))
        self.dtype = dense.dtype
        if not lib().oracle_part_valid(self.rows, self.grid[0]) or \
                not lib().oracle_part_valid(self.cols, self.grid[1]):
            raise ValueError("grid leaves an empty trailing block")
        self.blocks = []
        for (r0, r1) in split_bounds(self.rows, self.grid[0]):
            for (c0, c1) in split_bounds(self.cols, self.grid[1]):
                self.blocks.append(np.ascontiguousarray(dense[r0:r1, c0:c1]))
        self._ptrs = (ctypes.c_void_p * len(self.blocks))(*[b.ctypes.data for b in self.blocks])
        self.c = _OMat(self.rows, self.cols, self.grid[0], self.grid[1],
                       _DTYPE_CODE[self.dtype], 0, self._ptrs)


def _as_block(m, grid=(1, 1)):
    if m is None or isinstance(m, BlockMatrix):
        return m
    return BlockMatrix(m, grid)


def _sel(sel, n):
    if sel is None:
        return n, None, None
    arr = np.ascontiguousarray(np.asarray(sel, dtype=np.int64))
    return int(arr.size), arr, arr.ctypes.data


def gemm(transA: bool, transB: bool, alpha: float, A, B, beta: float, C=None, rows=None):
    """alpha*op(A)*op(B) + beta*C in fp64; ``rows`` restricts the result to those rows of it.
    A, B, C: BlockMatrix or plain 2-D arrays (taken as a 1x1 grid)."""
    A, B, C = _as_block(A), _as_block(B), _as_block(C)
    M = A.cols if transA else A.rows
    K = A.rows if transA else A.cols
    N = B.rows if transB else B.cols
    nsel, keep, selp = _sel(rows, M)
    out = np.empty((nsel, N), dtype=np.float64)
    rc = lib().oracle_gemm(int(bool(transA)), int(bool(transB)), float(alpha),
                           ctypes.byref(A.c), ctypes.byref(B.c), float(beta),
                           ctypes.byref(C.c) if C is not None else None,
                           M, N, K, nsel, selp, out.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle_gemm: error {rc}")
    return out


@dataclass
class ConvDesc:
    n: int
    c: int
    h: int
    w: int
    k: int
    r: int
    s: int
    pad_h: int = 0
    pad_w: int = 0
    stride_h: int = 1
    stride_w: int = 1

    def c_struct(self):
        return _OConv(self.n, self.c, self.h, self.w, self.k, self.r, self.s,
                      self.pad_h, self.pad_w, self.stride_h, self.stride_w)

    def out_hw(self):
        oh, ow = ctypes.c_int64(), ctypes.c_int64()
        cs = self.c_struct()
        if lib().oracle_conv_out_dims(ctypes.byref(cs), ctypes.byref(oh), ctypes.byref(ow)):
            raise ValueError("bad convolution geometry")
        return int(oh.value), int(ow.value)


def _conv_call(name, d, alpha, P, Q, beta, R, sel, nfull, width):
    P, Q, R = _as_block(P), _as_block(Q), _as_block(R)
    nsel, keep, selp = _sel(sel, nfull)
    out = np.empty((nsel, width), dtype=np.float64)
    cs = d.c_struct()
    rc = getattr(lib(), name)(ctypes.byref(cs), float(alpha), ctypes.byref(P.c),
                              ctypes.byref(Q.c), float(beta),
                              ctypes.byref(R.c) if R is not None else None,
                              nsel, selp, out.ctypes.data)
    if rc != 0:
        raise ValueError(f"{name}: error {rc}")
    return out


def conv_fwd(d: ConvDesc, alpha, X, F, beta=0.0, Y=None, images=None):
    """[N x K*OH*OW] fp64 (rows restricted to ``images``)."""
    oh, ow = d.out_hw()
    return _conv_call("oracle_conv_fwd", d, alpha, X, F, beta, Y, images, d.n, d.k * oh * ow)


def conv_bwd_filter(d: ConvDesc, alpha, X, dY, beta=0.0, dF=None, filters=None):
    """[K x C*R*S] fp64 (rows restricted to ``filters``)."""
    return _conv_call("oracle_conv_bwd_filter", d, alpha, X, dY, beta, dF, filters, d.k,
                      d.c * d.r * d.s)


def conv_bwd_data(d: ConvDesc, alpha, dY, F, beta=0.0, dX=None, images=None):
    """[N x C*H*W] fp64 (rows restricted to ``images``)."""
    return _conv_call("oracle_conv_bwd_data", d, alpha, dY, F, beta, dX, images, d.n,
                      d.c * d.h * d.w)


def convert(dense, dtype):
    """Re-layout with precision change (section 3.3, "change precision during reshape"): the
    values are unchanged when widening and rounded once, to nearest even, when narrowing.  The
    block grid does not enter: a matrix is the same matrix however it is cut (section 3.2)."""
    return np.asarray(dense).astype(dtype)


def rel_frobenius(got, ref) -> float:
    """||got - ref||_F / ||ref||_F in fp64; if ref is all zero, returns ||got||_F."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = float(np.linalg.norm(ref.ravel()))
    num = float(np.linalg.norm((got - ref).ravel()))
    return num if den == 0.0 else num / den
