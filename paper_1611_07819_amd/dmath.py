"""ctypes binding of ``include/dmath.h``: argument marshalling only.  Every step of the
computation runs in the HIP library; if the library is missing this module raises."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# DMATH_LIBRARY may point at another build of the same library (debug variants)
_LIB_PATH = os.environ.get("DMATH_LIBRARY") or os.path.join(_HERE, "libdmath.so")

F64, F32, F16 = 0, 1, 2
OP_N, OP_T = 0, 1
_NP = {F64: np.float64, F32: np.float32, F16: np.float16}
_CODE = {np.dtype(np.float64): F64, np.dtype(np.float32): F32, np.dtype(np.float16): F16}


class DmathError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {status_string(code)}")


class _TuneResult(ctypes.Structure):
    _fields_ = [("candidates", ctypes.c_int32), ("skipped", ctypes.c_int32), ("kernel", ctypes.c_int32),
                ("tile_m", ctypes.c_int32), ("tile_n", ctypes.c_int32), ("split_k", ctypes.c_int32),
                ("workspace_bytes", ctypes.c_uint64), ("chosen_us", ctypes.c_double),
                ("default_us", ctypes.c_double)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class _PlanInfo(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int64), ("n", ctypes.c_int64), ("k", ctypes.c_int64),
                ("m_segments", ctypes.c_int32), ("n_segments", ctypes.c_int32),
                ("k_segments", ctypes.c_int32), ("tile_m", ctypes.c_int32),
                ("tile_n", ctypes.c_int32), ("tile_k", ctypes.c_int32), ("tiles", ctypes.c_int32),
                ("split_k", ctypes.c_int32), ("kernel", ctypes.c_int32), ("cached", ctypes.c_int32),
                ("split_tiles", ctypes.c_int32), ("workspace_bytes", ctypes.c_uint64)]


class _ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n", "c", "h", "w", "k", "r", "s", "pad_h", "pad_w", "stride_h", "stride_w")]


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

    def _c(self):
        return _ConvDesc(self.n, self.c, self.h, self.w, self.k, self.r, self.s, self.pad_h,
                         self.pad_w, self.stride_h, self.stride_w)


_lib = None


def load_library(build_if_missing: bool = True):
    """Loads libdmath.so (building it with hipcc only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(_LIB_PATH)
        from .build import build
        build()
    L = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, dbl, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_double, ctypes.c_size_t
    P = ctypes.POINTER
    sig = {
        "dmath_init": [P(vp), vp, sz, vp],
        "dmath_finalize": [vp],
        "dmath_matrix_create": [vp, i64, i64, i32, i32, ctypes.c_int, P(vp)],
        "dmath_matrix_destroy": [vp],
        "dmath_matrix_set": [vp, vp, i64],
        "dmath_matrix_get": [vp, vp, i64],
        "dmath_matrix_info": [vp, P(i64), P(i64), P(i32), P(i32), P(ctypes.c_int)],
        "dmath_matrix_block": [vp, i32, i32, P(vp), P(i64), P(i64), P(i64)],
        "dmath_matrix_reblock": [vp, vp, vp],
        "dmath_gemm": [vp, ctypes.c_int, ctypes.c_int, dbl, vp, vp, dbl, vp],
        "dmath_gemm_noalloc": [vp, ctypes.c_int, ctypes.c_int, dbl, vp, vp, dbl, vp],
        "dmath_gemm_plan_info": [vp, ctypes.c_int, ctypes.c_int, vp, vp, vp, P(_PlanInfo)],
        "dmath_conv_fwd": [vp, P(_ConvDesc), dbl, vp, vp, dbl, vp],
        "dmath_conv_bwd_filter": [vp, P(_ConvDesc), dbl, vp, vp, dbl, vp],
        "dmath_conv_bwd_data": [vp, P(_ConvDesc), dbl, vp, vp, dbl, vp],
        "dmath_set_kernel_policy": [vp, i32],
        "dmath_gemm_tune": [vp, ctypes.c_int, ctypes.c_int, vp, vp, vp, sz, i32, P(_TuneResult)],
        "dmath_conv_tune": [vp, i32, P(_ConvDesc), vp, vp, vp, sz, i32, P(_TuneResult)],
        "dmath_tune_reset": [vp],
        "dmath_set_relayout_reuse": [vp, i32],
        "dmath_relayout_stats": [vp, P(ctypes.c_uint64), P(ctypes.c_uint64), P(sz)],
        "dmath_matrix_touch": [vp],
        "dmath_pipeline_begin": [vp],
        "dmath_pipeline_end": [vp, P(i32)],
        "dmath_pipeline_replay": [vp, i32],
        "dmath_pipeline_destroy": [vp, i32],
        "dmath_synchronize": [vp],
        "dmath_cycle_probe_read": [vp, P(ctypes.c_uint64)],
        "dmath_mfma_peak_probe": [vp, ctypes.c_int, i32, P(dbl)],
        "dmath_mfma_peak_probe_f16_32x32x16": [vp, i32, P(dbl)],
        "dmath_pool_stats": [vp, P(sz), P(sz), P(sz)],
    }
    for name, args in sig.items():
        fn = getattr(L, name)
        fn.argtypes = args
        fn.restype = ctypes.c_int
    L.dmath_status_string.argtypes = [ctypes.c_int]
    L.dmath_status_string.restype = ctypes.c_char_p
    _lib = L
    return L


def status_string(code: int) -> str:
    return load_library().dmath_status_string(int(code)).decode()


def _check(code, where):
    if code != 0:
        raise DmathError(code, where)


class Context:
    """A pool over caller-owned device memory plus a HIP stream.

    ``slab``: a torch uint8 CUDA tensor (kept alive here), or an integer device address with
    ``slab_bytes``.  ``stream``: a raw hipStream_t value (0 = default stream)."""

    def __init__(self, slab, slab_bytes: int | None = None, stream: int = 0):
        self._lib = load_library()
        self._slab = slab
        if hasattr(slab, "data_ptr"):
            ptr, nbytes = slab.data_ptr(), slab.numel() * slab.element_size()
        else:
            ptr, nbytes = int(slab), int(slab_bytes)
        self._h = ctypes.c_void_p()
        _check(self._lib.dmath_init(ctypes.byref(self._h), ptr, nbytes, stream), "dmath_init")

    def matrix(self, rows, cols, grid=(1, 1), dtype=F32) -> "Matrix":
        return Matrix(self, rows, cols, grid, dtype)

    def from_host(self, array: np.ndarray, grid=(1, 1)) -> "Matrix":
        array = np.ascontiguousarray(array)
        m = Matrix(self, array.shape[0], array.shape[1], grid, _CODE[array.dtype])
        m.set(array)
        return m

    def set_kernel_policy(self, policy: int):
        _check(self._lib.dmath_set_kernel_policy(self._h, policy), "dmath_set_kernel_policy")

    def tune_reset(self):
        _check(self._lib.dmath_tune_reset(self._h), "dmath_tune_reset")

    def set_relayout_reuse(self, enable: bool):
        _check(self._lib.dmath_set_relayout_reuse(self._h, 1 if enable else 0), "dmath_set_relayout_reuse")

    def relayout_stats(self):
        a, b, c = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_size_t()
        _check(self._lib.dmath_relayout_stats(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)),
               "dmath_relayout_stats")
        return {"reused": a.value, "written": b.value, "bytes_held": c.value}

    def mfma_peak_probe(self, dtype: int, iters: int, wide_f16: bool = False) -> float:
        """Enqueues the MFMA-only micro-kernel; returns the flops it performs (wide_f16: fp16
        on the 32x32x16 instruction instead of 16x16x32)."""
        f = ctypes.c_double()
        if wide_f16:
            _check(self._lib.dmath_mfma_peak_probe_f16_32x32x16(self._h, iters, ctypes.byref(f)),
                   "dmath_mfma_peak_probe_f16_32x32x16")
        else:
            _check(self._lib.dmath_mfma_peak_probe(self._h, dtype, iters, ctypes.byref(f)),
                   "dmath_mfma_peak_probe")
        return f.value

    def pipeline_begin(self):
        _check(self._lib.dmath_pipeline_begin(self._h), "dmath_pipeline_begin")

    def pipeline_end(self) -> int:
        pid = ctypes.c_int32()
        _check(self._lib.dmath_pipeline_end(self._h, ctypes.byref(pid)), "dmath_pipeline_end")
        return pid.value

    def pipeline_replay(self, pid: int):
        _check(self._lib.dmath_pipeline_replay(self._h, pid), "dmath_pipeline_replay")

    def pipeline_destroy(self, pid: int):
        _check(self._lib.dmath_pipeline_destroy(self._h, pid), "dmath_pipeline_destroy")

    def cycle_probe_read(self):
        """Cycle counts of the last specialised fp16 GEMM (probe builds of the library only)."""
        out = (ctypes.c_uint64 * 6)()
        _check(self._lib.dmath_cycle_probe_read(self._h, out), "dmath_cycle_probe_read")
        keys = ("prologue", "loop", "epilogue", "barrier_wait", "ticks_100mhz", "ktiles")
        return dict(zip(keys, [int(v) for v in out]))

    def synchronize(self):
        _check(self._lib.dmath_synchronize(self._h), "dmath_synchronize")

    def pool_stats(self):
        a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
        _check(self._lib.dmath_pool_stats(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)),
               "dmath_pool_stats")
        return {"in_use": a.value, "high_water": b.value, "capacity": c.value}

    def close(self):
        if self._h:
            _check(self._lib.dmath_finalize(self._h), "dmath_finalize")
            self._h = ctypes.c_void_p()

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


class Matrix:
    def __init__(self, ctx: Context, rows, cols, grid=(1, 1), dtype=F32):
        self.ctx = ctx
        self.rows, self.cols, self.grid, self.dtype = int(rows), int(cols), tuple(grid), int(dtype)
        self._h = ctypes.c_void_p()
        _check(ctx._lib.dmath_matrix_create(ctx._h, self.rows, self.cols, int(grid[0]), int(grid[1]),
                                            self.dtype, ctypes.byref(self._h)), "dmath_matrix_create")

    def set(self, array: np.ndarray):
        a = np.ascontiguousarray(array, dtype=_NP[self.dtype])
        if a.shape != (self.rows, self.cols):
            raise ValueError("shape mismatch")
        _check(self.ctx._lib.dmath_matrix_set(self._h, a.ctypes.data, self.cols), "dmath_matrix_set")

    def get(self) -> np.ndarray:
        out = np.empty((self.rows, self.cols), dtype=_NP[self.dtype])
        _check(self.ctx._lib.dmath_matrix_get(self._h, out.ctypes.data, self.cols), "dmath_matrix_get")
        return out

    def block(self, bi, bj):
        p, r, c, ld = ctypes.c_void_p(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        _check(self.ctx._lib.dmath_matrix_block(self._h, bi, bj, ctypes.byref(p), ctypes.byref(r),
                                                ctypes.byref(c), ctypes.byref(ld)), "dmath_matrix_block")
        return {"ptr": p.value, "rows": r.value, "cols": c.value, "ld": ld.value}

    def touch(self):
        _check(self.ctx._lib.dmath_matrix_touch(self._h), "dmath_matrix_touch")

    def info(self):
        r, c, gr, gc, dt = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int()
        _check(self.ctx._lib.dmath_matrix_info(self._h, ctypes.byref(r), ctypes.byref(c),
                                               ctypes.byref(gr), ctypes.byref(gc), ctypes.byref(dt)),
               "dmath_matrix_info")
        return {"rows": r.value, "cols": c.value, "grid": (gr.value, gc.value), "dtype": dt.value}

    def destroy(self):
        if self._h:
            _check(self.ctx._lib.dmath_matrix_destroy(self._h), "dmath_matrix_destroy")
            self._h = ctypes.c_void_p()


def reblock(ctx: Context, src: Matrix, dst: Matrix):
    """dst <- src across block grids and precisions."""
    _check(ctx._lib.dmath_matrix_reblock(ctx._h, src._h, dst._h), "dmath_matrix_reblock")


def gemm(ctx: Context, transA, transB, alpha, A: Matrix, B: Matrix, beta, C: Matrix):
    _check(ctx._lib.dmath_gemm(ctx._h, int(transA), int(transB), float(alpha), A._h, B._h,
                               float(beta), C._h), "dmath_gemm")


def gemm_noalloc(ctx: Context, transA, transB, alpha, A: Matrix, B: Matrix, beta, C: Matrix):
    """dmath_gemm that takes nothing from the pool: its scratch is the library's static device array."""
    _check(ctx._lib.dmath_gemm_noalloc(ctx._h, int(transA), int(transB), float(alpha), A._h, B._h,
                                       float(beta), C._h), "dmath_gemm_noalloc")


def gemm_plan_info(ctx: Context, transA, transB, A: Matrix, B: Matrix, C: Matrix) -> dict:
    info = _PlanInfo()
    _check(ctx._lib.dmath_gemm_plan_info(ctx._h, int(transA), int(transB), A._h, B._h, C._h,
                                         ctypes.byref(info)), "dmath_gemm_plan_info")
    return {f: getattr(info, f) for f, _ in _PlanInfo._fields_}


def conv_fwd(ctx: Context, desc: ConvDesc, alpha, X: Matrix, F: Matrix, beta, Y: Matrix):
    d = desc._c()
    _check(ctx._lib.dmath_conv_fwd(ctx._h, ctypes.byref(d), float(alpha), X._h, F._h, float(beta),
                                   Y._h), "dmath_conv_fwd")


def conv_bwd_filter(ctx: Context, desc: ConvDesc, alpha, X: Matrix, dY: Matrix, beta, dF: Matrix):
    d = desc._c()
    _check(ctx._lib.dmath_conv_bwd_filter(ctx._h, ctypes.byref(d), float(alpha), X._h, dY._h,
                                          float(beta), dF._h), "dmath_conv_bwd_filter")


def conv_bwd_data(ctx: Context, desc: ConvDesc, alpha, dY: Matrix, F: Matrix, beta, dX: Matrix):
    d = desc._c()
    _check(ctx._lib.dmath_conv_bwd_data(ctx._h, ctypes.byref(d), float(alpha), dY._h, F._h,
                                        float(beta), dX._h), "dmath_conv_bwd_data")


def gemm_tune(ctx: Context, transA, transB, A: Matrix, B: Matrix, C: Matrix, workspace_limit: int,
              trials: int = 5) -> dict:
    r = _TuneResult()
    _check(ctx._lib.dmath_gemm_tune(ctx._h, int(transA), int(transB), A._h, B._h, C._h,
                                    int(workspace_limit), int(trials), ctypes.byref(r)), "dmath_gemm_tune")
    return r.as_dict()


def conv_tune(ctx: Context, mode: int, desc: ConvDesc, X: Matrix, F: Matrix, Y: Matrix,
              workspace_limit: int, trials: int = 5) -> dict:
    r = _TuneResult()
    d = desc._c()
    _check(ctx._lib.dmath_conv_tune(ctx._h, int(mode), ctypes.byref(d), X._h, F._h, Y._h,
                                    int(workspace_limit), int(trials), ctypes.byref(r)), "dmath_conv_tune")
    return r.as_dict()
