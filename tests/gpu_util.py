"""Helpers of the GPU parity tests: a context over a torch-owned slab, upload/download, and the
tolerances of the three precisions (relative Frobenius error against the fp64 oracle)."""
import numpy as np

import paper_1611_07819_amd as dm

TOL = {dm.F64: 1e-12, dm.F32: 1e-5, dm.F16: 2e-3}   # by INPUT precision
CODE = {np.dtype(np.float64): dm.F64, np.dtype(np.float32): dm.F32, np.dtype(np.float16): dm.F16}


def make_context(gib: float = 6.0):
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    slab = torch.empty(int(gib * (1 << 30)), dtype=torch.uint8, device="cuda:0")
    return dm.Context(slab, stream=torch.cuda.current_stream().cuda_stream)


def rel_fro(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((got - ref).ravel())
    return num if den == 0 else num / den
