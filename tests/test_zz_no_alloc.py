"""dmath_gemm_noalloc (the GEMM call for callers that cannot allocate) against dmath_gemm, through
the C ABI: same kernels on the same plan choice, so the results must agree bit for bit; the pool
must be untouched; two calls in a row share the static scratch array, the second one smaller."""
import numpy as np
import pytest

import paper_1611_07819_amd as dm
from paper_1611_07819_amd import dmath as binding
from gpu_util import TOL, make_context, rel_fro

pytestmark = pytest.mark.gpu
NP = {dm.F64: np.float64, dm.F32: np.float32, dm.F16: np.float16}


def _both(ctx, oracle, dt, out, ta, tb, M, N, K, grids, seed, alpha=1.5, beta=-0.5):
    r = np.random.default_rng(seed)
    A = r.uniform(-1, 1, (K, M) if ta else (M, K)).astype(NP[dt])
    B = r.uniform(-1, 1, (N, K) if tb else (K, N)).astype(NP[dt])
    C0 = r.uniform(-1, 1, (M, N)).astype(NP[out])
    dA, dB = ctx.from_host(A, grids[0]), ctx.from_host(B, grids[1])
    dC1, dC2 = ctx.from_host(C0, grids[2]), ctx.from_host(C0, grids[2])
    info = dm.gemm_plan_info(ctx, ta, tb, dA, dB, dC1)
    dm.gemm(ctx, ta, tb, alpha, dA, dB, beta, dC1)
    want = dC1.get()
    ctx.synchronize()
    before = ctx.pool_stats()
    for _ in range(2):                                    # the second call finds its plan in place
        dC2.set(C0)
        dm.gemm_noalloc(ctx, ta, tb, alpha, dA, dB, beta, dC2)
        got = dC2.get()
        assert np.array_equal(got, want), (dt, out, ta, tb, (M, N, K), info)
    after = ctx.pool_stats()
    assert after["in_use"] == before["in_use"] and after["high_water"] == before["high_water"]
    ref = oracle.gemm(bool(ta), bool(tb), alpha, oracle.BlockMatrix(A, grids[0]), oracle.BlockMatrix(B, grids[1]),
                      beta, oracle.BlockMatrix(C0, grids[2]))
    assert rel_fro(got, ref) <= TOL[dt]
    for m in (dA, dB, dC1, dC2):
        m.destroy()
    return info


def test_noalloc_matches_gemm_on_two_calls_in_a_row():
    from oracle import cpu_oracle as oracle
    oracle.build()
    ctx = make_context(1.0)
    try:
        # deep K, few tiles: split k-loop, partial sums in the static array; block grids that do not line up
        info = _both(ctx, oracle, dm.F32, dm.F32, 0, 0, 96, 80, 8192, ((1, 3), (2, 1), (1, 1)), 5001)
        assert info["split_k"] > 1 and info["workspace_bytes"] > 0, info
        # smaller input right after it, fp16 with a k-tail (K = 1000: zero-padded panels in the array)
        info = _both(ctx, oracle, dm.F16, dm.F32, 0, 1, 72, 64, 1000, ((1, 1), (1, 1), (1, 1)), 5002)
        assert info["kernel"] > 0 and info["workspace_bytes"] > 0, info
        # larger again, every precision and op pair once, fp16 output, the generic kernel
        _both(ctx, oracle, dm.F64, dm.F64, 1, 0, 200, 136, 512, ((2, 2), (2, 1), (1, 2)), 5003)
        _both(ctx, oracle, dm.F16, dm.F16, 1, 1, 320, 256, 2048, ((2, 2), (2, 2), (2, 2)), 5004)
        _both(ctx, oracle, dm.F32, dm.F32, 0, 1, 33, 17, 45, ((1, 1), (1, 1), (1, 1)), 5005)
    finally:
        ctx.close()


def test_noalloc_argument_errors_and_two_contexts_sharing_the_array():
    from oracle import cpu_oracle as oracle
    oracle.build()
    c1, c2 = make_context(0.25), make_context(0.25)
    try:
        r = np.random.default_rng(5100)
        A = r.uniform(-1, 1, (128, 256)).astype(np.float32)
        B = r.uniform(-1, 1, (256, 64)).astype(np.float32)
        ref = oracle.gemm(False, False, 1.0, A, B, 0.0)
        dev = []
        for c in (c1, c2):
            dev.append((c.from_host(A), c.from_host(B), c.matrix(128, 64, (1, 1), dm.F32)))
        # the contexts take turns: each call finds the array rewritten by the other and restores its plan
        for rep in range(2):
            for c, (dA, dB, dC) in zip((c1, c2), dev):
                dC.set(np.full((128, 64), np.nan, np.float32))
                dm.gemm_noalloc(c, 0, 0, 1.0, dA, dB, 0.0, dC)
                assert rel_fro(dC.get(), ref) <= TOL[dm.F32]
        dA, dB, dC = dev[0]
        with pytest.raises(binding.DmathError) as e:
            dm.gemm_noalloc(c1, 0, 0, 1.0, dA, dB, 0.0, dA)
        assert e.value.code == 5                                   # alias
        with pytest.raises(binding.DmathError) as e:
            dm.gemm_noalloc(c1, 1, 0, 1.0, dA, dB, 0.0, dC)
        assert e.value.code == 2                                   # shape
        with pytest.raises(binding.DmathError) as e:
            dm.gemm_noalloc(c1, 0, 0, 1.0, dA, dev[1][1], 0.0, dC)
        assert e.value.code == 1                                   # a handle of another context
    finally:
        c1.close()
        c2.close()


def test_noalloc_refuses_plans_beyond_the_scratch_array():
    # a million 2x2 blocks of C: the tile table alone (32 bytes per tile) exceeds the 32 MiB array
    ctx = make_context(1.0)
    try:
        dA = ctx.matrix(2048, 2, (1024, 1), dm.F32)
        dB = ctx.matrix(2, 2048, (1, 1024), dm.F32)
        dC = ctx.matrix(2048, 2048, (1024, 1024), dm.F32)
        before = ctx.pool_stats()["in_use"]
        with pytest.raises(binding.DmathError) as e:
            dm.gemm_noalloc(ctx, 0, 0, 1.0, dA, dB, 0.0, dC)
        assert e.value.code == 9 and "SCRATCH_LIMIT" in str(e.value)
        assert ctx.pool_stats()["in_use"] == before
    finally:
        ctx.close()
