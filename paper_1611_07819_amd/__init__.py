"""MI355X (gfx950) implementation of dMath's per-worker block GEMM and implicit-GEMM
convolution: a C-ABI HIP library (``libdmath.so``) and this thin ctypes binding."""
from .dmath import (Context, Matrix, ConvDesc, DmathError, F64, F32, F16, OP_N, OP_T,  # noqa: F401
                    gemm, gemm_noalloc, gemm_plan_info, gemm_tune, conv_tune, reblock, conv_fwd, conv_bwd_filter,
                    conv_bwd_data, load_library)
