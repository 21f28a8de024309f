"""Selection of kernel, tile shape and split-K count from timing samples under a memory limit
(paper section 4.1: the convolution algorithm is picked at start-up from timing samples within
the system's constraints).  Whatever is chosen, results must stay within the oracle's bar; the
limit must be honoured; the choice must carry over to other matrices laid out the same way."""
import numpy as np
import pytest

import paper_1611_07819_amd as dm
from gpu_util import TOL, rel_fro

pytestmark = pytest.mark.gpu
NP = {dm.F64: np.float64, dm.F32: np.float32, dm.F16: np.float16}


@pytest.fixture()
def ctx():
    import torch
    stream = torch.cuda.Stream()
    slab = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    c = dm.Context(slab, stream=stream.cuda_stream)
    yield c
    c.close()


@pytest.mark.parametrize("dt,out,shape", [(dm.F32, dm.F32, (256, 384, 8192)),
                                          (dm.F16, dm.F32, (512, 1024, 4096)),
                                          (dm.F64, dm.F64, (256, 256, 2048))])
def test_gemm_tune_honours_the_limit_and_keeps_parity(ctx, oracle, dt, out, shape):
    M, N, K = shape
    r = np.random.default_rng(1100)
    A = r.uniform(-1, 1, (M, K)).astype(NP[dt])
    B = r.uniform(-1, 1, (K, N)).astype(NP[dt])
    ref = oracle.gemm(False, False, 1.0, A, B, 0.0)
    dA, dB, dC = ctx.from_host(A, (1, 2)), ctx.from_host(B, (2, 1)), ctx.matrix(M, N, (1, 1), out)
    model = dm.gemm_plan_info(ctx, 0, 0, dA, dB, dC)

    def check(info_expected):
        dC.set(np.full((M, N), np.nan, NP[out]))
        dm.gemm(ctx, 0, 0, 1.0, dA, dB, 0.0, dC)
        assert rel_fro(dC.get(), ref) <= TOL[dt]
        info = dm.gemm_plan_info(ctx, 0, 0, dA, dB, dC)
        for k in ("kernel", "tile_m", "tile_n", "split_k"):
            assert info[k] == info_expected[k], k

    # no memory beyond the operands: nothing split may be chosen, split candidates are left out
    t0 = dm.gemm_tune(ctx, 0, 0, dA, dB, dC, 0, trials=3)
    assert t0["candidates"] >= 2 and t0["skipped"] >= 1
    assert t0["split_k"] == 1 and t0["workspace_bytes"] == 0 and t0["chosen_us"] > 0
    check(t0)
    # generous limit: more candidates, the chosen one is at least as fast as the cost model's
    t1 = dm.gemm_tune(ctx, 0, 0, dA, dB, dC, 1 << 28, trials=3)
    assert t1["candidates"] > t0["candidates"] and t1["skipped"] == 0
    assert t1["default_us"] > 0 and t1["chosen_us"] <= t1["default_us"]
    assert t1["workspace_bytes"] <= 1 << 28
    check(t1)
    # the choice belongs to the layout, not to the handles
    eA, eB, eC = ctx.from_host(A, (1, 2)), ctx.from_host(B, (2, 1)), ctx.matrix(M, N, (1, 1), out)
    info = dm.gemm_plan_info(ctx, 0, 0, eA, eB, eC)
    for k in ("kernel", "tile_m", "tile_n", "split_k"):
        assert info[k] == t1[k], k
    dm.gemm(ctx, 0, 0, 1.0, eA, eB, 0.0, eC)
    assert rel_fro(eC.get(), ref) <= TOL[dt]
    # another grid is another layout: cost model
    fA = ctx.from_host(A, (1, 1))
    other = dm.gemm_plan_info(ctx, 0, 0, fA, dB, dC)
    assert other["kernel"] == model["kernel"]
    ctx.tune_reset()
    check(model)


def test_gemm_tune_counts_the_scratch_panels_of_k_tails(ctx, oracle):
    """K = 1000 is not a multiple of the fp32 kernels' k-step: the specialised kernels read the
    end of K from scratch panels in the pool, which count against the memory limit."""
    M, N, K = 256, 384, 1000
    r = np.random.default_rng(1103)
    A = r.uniform(-1, 1, (M, K)).astype(np.float32)
    B = r.uniform(-1, 1, (K, N)).astype(np.float32)
    ref = oracle.gemm(False, False, 1.0, A, B, 0.0)
    dA, dB, dC = ctx.from_host(A), ctx.from_host(B), ctx.matrix(M, N, (1, 1), dm.F32)
    t0 = dm.gemm_tune(ctx, 0, 0, dA, dB, dC, 0, trials=2)
    assert t0["kernel"] == 0 and t0["workspace_bytes"] == 0 and t0["skipped"] >= 2
    dm.gemm(ctx, 0, 0, 1.0, dA, dB, 0.0, dC)
    assert rel_fro(dC.get(), ref) <= TOL[dm.F32]
    t1 = dm.gemm_tune(ctx, 0, 0, dA, dB, dC, 1 << 26, trials=2)
    assert t1["kernel"] != 0 and t1["workspace_bytes"] >= (M + N) * 32 * 4
    info = dm.gemm_plan_info(ctx, 0, 0, dA, dB, dC)
    assert info["kernel"] == t1["kernel"] and info["workspace_bytes"] == t1["workspace_bytes"]
    dm.gemm(ctx, 0, 0, 1.0, dA, dB, 0.0, dC)
    assert rel_fro(dC.get(), ref) <= TOL[dm.F32]
    ctx.tune_reset()


GEO = dict(n=4, c=128, h=16, w=16, k=256, r=3, s=3, pad_h=1, pad_w=1)


@pytest.mark.parametrize("dt", [dm.F16, dm.F32, dm.F64])
def test_conv_tune_all_modes(ctx, oracle, dt):
    d, od = dm.ConvDesc(**GEO), oracle.ConvDesc(**GEO)
    r = np.random.default_rng(1101)
    hx = r.uniform(0, 1, (4, 128 * 256)).astype(NP[dt])
    hf = r.normal(0, 0.05, (256, 128 * 9)).astype(NP[dt])
    hy = r.normal(0, 0.1, (4, 256 * 256)).astype(NP[dt])
    X, F, dY = ctx.from_host(hx), ctx.from_host(hf), ctx.from_host(hy)
    out = dm.F64 if dt == dm.F64 else dm.F32
    Y = ctx.matrix(4, 256 * 256, (1, 1), out)
    dF = ctx.matrix(256, 128 * 9, (1, 1), out)
    dX = ctx.matrix(4, 128 * 256, (1, 1), out)
    refs = {0: oracle.conv_fwd(od, 1.0, hx, hf), 1: oracle.conv_bwd_filter(od, 1.0, hx, hy),
            2: oracle.conv_bwd_data(od, 1.0, hy, hf)}

    def run(mode):
        if mode == 0:
            dm.conv_fwd(ctx, d, 1.0, X, F, 0.0, Y)
            return Y.get()
        if mode == 1:
            dm.conv_bwd_filter(ctx, d, 1.0, X, dY, 0.0, dF)
            return dF.get()
        dm.conv_bwd_data(ctx, d, 1.0, dY, F, 0.0, dX)
        return dX.get()

    operands = {0: (X, F, Y), 1: (X, dF, dY), 2: (dX, F, dY)}
    # no memory beyond the tensors: only the generic kernel without split-K qualifies, and the
    # copies that the rejected candidates would need are not held afterwards
    for mode in (0, 1, 2):
        t = dm.conv_tune(ctx, mode, d, *operands[mode], 0, trials=2)
        assert t["kernel"] == 0 and t["split_k"] == 1 and t["workspace_bytes"] == 0
        assert t["skipped"] >= 1 and t["candidates"] == 1
        assert rel_fro(run(mode), refs[mode]) <= TOL[dt], mode
    assert ctx.relayout_stats()["bytes_held"] == 0
    # generous limit: the specialised kernels are candidates too; the chosen configuration is
    # never slower than the cost model's (which of them wins on so small a layer is not fixed)
    for mode in (0, 1, 2):
        t = dm.conv_tune(ctx, mode, d, *operands[mode], 1 << 28, trials=3)
        assert t["skipped"] == 0 and t["candidates"] >= (2 if mode == 2 else 3)
        assert t["workspace_bytes"] <= 1 << 28 and (t["kernel"] == 0 or t["workspace_bytes"] > 0)
        assert t["default_us"] > 0 and t["chosen_us"] <= t["default_us"]
        assert rel_fro(run(mode), refs[mode]) <= TOL[dt], mode
        assert rel_fro(run(mode), refs[mode]) <= TOL[dt], mode      # second call: copies reused
    ctx.tune_reset()
    for mode in (0, 1, 2):
        assert rel_fro(run(mode), refs[mode]) <= TOL[dt], mode


def test_conv_tune_of_a_1x1_layer_counts_what_its_block_gemm_takes(ctx, oracle):
    """A 1x1 stride-1 layer can run as a block GEMM without re-layout copies; its weight gradient
    is a deep split-K GEMM whose partial sums (and padded k-tails) come from the pool and count
    against the limit."""
    geo = dict(n=8, c=128, h=24, w=24, k=128, r=1, s=1)
    d, od = dm.ConvDesc(**geo), oracle.ConvDesc(**geo)
    r = np.random.default_rng(1104)
    hx = r.uniform(0, 1, (8, 128 * 576)).astype(np.float16)
    hf = r.normal(0, 0.05, (128, 128)).astype(np.float16)
    hy = r.normal(0, 0.1, (8, 128 * 576)).astype(np.float16)
    X, F, dY = ctx.from_host(hx), ctx.from_host(hf), ctx.from_host(hy)
    Y = ctx.matrix(8, 128 * 576, (1, 1), dm.F32)
    dF = ctx.matrix(128, 128, (1, 1), dm.F32)
    # forward: the block GEMM needs nothing from the pool and is a candidate even with no memory
    t = dm.conv_tune(ctx, 0, d, X, F, Y, 0, trials=2)
    assert t["candidates"] >= 2 and t["workspace_bytes"] == 0
    dm.conv_fwd(ctx, d, 1.0, X, F, 0.0, Y)
    assert rel_fro(Y.get(), oracle.conv_fwd(od, 1.0, hx, hf)) <= TOL[dm.F16]
    # weight gradient: with no memory only configurations without partial sums remain
    t0 = dm.conv_tune(ctx, 1, d, X, dF, dY, 0, trials=2)
    assert t0["workspace_bytes"] == 0 and t0["skipped"] >= 1
    dm.conv_bwd_filter(ctx, d, 1.0, X, dY, 0.0, dF)
    assert rel_fro(dF.get(), oracle.conv_bwd_filter(od, 1.0, hx, hy)) <= TOL[dm.F16]
    t1 = dm.conv_tune(ctx, 1, d, X, dF, dY, 1 << 28, trials=2)
    assert t1["candidates"] > t0["candidates"] and t1["chosen_us"] <= t0["chosen_us"] * 1.05
    dm.conv_bwd_filter(ctx, d, 1.0, X, dY, 0.0, dF)
    assert rel_fro(dF.get(), oracle.conv_bwd_filter(od, 1.0, hx, hy)) <= TOL[dm.F16]
    ctx.tune_reset()


@pytest.mark.parametrize("dt", [dm.F16, dm.F32])
def test_conv_tune_of_a_small_batch_splits_the_k_loop(ctx, oracle, dt):
    """One image of a deep layer: eight output tiles against a k-loop of 2304.  The cost model and
    the tuner cut the loop of the forward pass and the data gradient into parts (the unsplit
    configuration is several times slower), and the partial sums count as workspace."""
    geo = dict(n=1, c=256, h=14, w=14, k=256, r=3, s=3, pad_h=1, pad_w=1)
    d, od = dm.ConvDesc(**geo), oracle.ConvDesc(**geo)
    r = np.random.default_rng(1105)
    hx = r.uniform(0, 1, (1, 256 * 196)).astype(NP[dt])
    hf = r.normal(0, 0.05, (256, 256 * 9)).astype(NP[dt])
    hy = r.normal(0, 0.1, (1, 256 * 196)).astype(NP[dt])
    X, F, dY = ctx.from_host(hx), ctx.from_host(hf), ctx.from_host(hy)
    Y = ctx.matrix(1, 256 * 196, (1, 1), dm.F32)
    dX = ctx.matrix(1, 256 * 196, (1, 1), dm.F32)
    for mode, operands in ((0, (X, F, Y)), (2, (dX, F, dY))):
        t = dm.conv_tune(ctx, mode, d, *operands, 1 << 28, trials=5)
        assert t["kernel"] == 1 and t["split_k"] > 1, t
        assert t["default_us"] > 0 and t["chosen_us"] >= 0.6 * t["default_us"], t    # the model's own choice is split too
        tile_rows = 256 if dt == dm.F16 else 128
        assert t["workspace_bytes"] >= t["split_k"] * tile_rows * 256 * 4
    dm.conv_fwd(ctx, d, 1.0, X, F, 0.0, Y)
    assert rel_fro(Y.get(), oracle.conv_fwd(od, 1.0, hx, hf)) <= TOL[dt]
    dm.conv_bwd_data(ctx, d, 1.0, dY, F, 0.0, dX)
    assert rel_fro(dX.get(), oracle.conv_bwd_data(od, 1.0, hy, hf)) <= TOL[dt]
    ctx.tune_reset()
    for m in (X, F, dY, Y, dX):
        m.destroy()


def test_tune_argument_errors(ctx):
    A, B = ctx.matrix(128, 128, (1, 1), dm.F32), ctx.matrix(128, 128, (1, 1), dm.F32)
    C = ctx.matrix(128, 128, (1, 1), dm.F32)
    with pytest.raises(dm.DmathError) as e:
        dm.gemm_tune(ctx, 0, 0, A, B, C, 0, trials=0)
    assert e.value.code == 1
    with pytest.raises(dm.DmathError) as e:
        dm.gemm_tune(ctx, 0, 0, A, B, A, 0, trials=1)
    assert e.value.code == 5                                  # alias
    ctx.set_kernel_policy(1)
    with pytest.raises(dm.DmathError) as e:
        dm.gemm_tune(ctx, 0, 0, A, B, C, 0, trials=1)
    assert e.value.code == 7
    ctx.set_kernel_policy(0)
    dm.gemm(ctx, 0, 0, 1.0, A, B, 0.0, C)
    ctx.pipeline_begin()
    with pytest.raises(dm.DmathError) as e:
        dm.gemm_tune(ctx, 0, 0, A, B, C, 0, trials=1)
    assert e.value.code == 7
    ctx.pipeline_destroy(ctx.pipeline_end())


def test_full_pool_falls_back_to_configurations_without_workspace(oracle):
    """Section 4.1's other half: where memory is the constraint a slower configuration is taken.
    A pool that cannot hold the split-K partial sums, or the convolution's re-layout copies, must
    still give the result (unsplit kernel, generic convolution kernel)."""
    import torch
    stream = torch.cuda.Stream()
    slab = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    ctx = dm.Context(slab, stream=stream.cuda_stream)
    r = np.random.default_rng(1102)

    def fill_pool(leave):
        st = ctx.pool_stats()
        n = (st["capacity"] - st["in_use"] - leave) // 256 * 256
        return ctx.matrix(1, n // 4, (1, 1), dm.F32)

    # GEMM: 4 tiles, K = 16384: the cost model wants 32 splits = 8 MB of partial sums
    M, N, K = 256, 256, 16384
    A = r.uniform(-1, 1, (M, K)).astype(np.float32)
    B = r.uniform(-1, 1, (K, N)).astype(np.float32)
    dA, dB, dC = ctx.from_host(A), ctx.from_host(B), ctx.matrix(M, N, (1, 1), dm.F32)
    assert dm.gemm_plan_info(ctx, 0, 0, dA, dB, dC)["split_k"] > 1
    filler = fill_pool(1 << 20)
    dm.gemm(ctx, 0, 0, 1.0, dA, dB, 0.0, dC)
    info = dm.gemm_plan_info(ctx, 0, 0, dA, dB, dC)
    assert info["split_k"] == 1 and info["workspace_bytes"] == 0 and info["kernel"] != 0
    assert rel_fro(dC.get(), oracle.gemm(False, False, 1.0, A, B, 0.0)) <= TOL[dm.F32]
    for m in (filler, dA, dB, dC):
        m.destroy()

    # convolution: the specialised kernels need ~0.9 MB of copies; 256 KiB are left
    d, od = dm.ConvDesc(**GEO), oracle.ConvDesc(**GEO)
    hx = r.uniform(0, 1, (4, 128 * 256)).astype(np.float16)
    hf = r.normal(0, 0.05, (256, 128 * 9)).astype(np.float16)
    hy = r.normal(0, 0.1, (4, 256 * 256)).astype(np.float16)
    X, F, dY = ctx.from_host(hx), ctx.from_host(hf), ctx.from_host(hy)
    Y = ctx.matrix(4, 256 * 256, (1, 1), dm.F32)
    dF = ctx.matrix(256, 128 * 9, (1, 1), dm.F32)
    filler = fill_pool(256 << 10)
    dm.conv_fwd(ctx, d, 1.0, X, F, 0.0, Y)
    dm.conv_bwd_filter(ctx, d, 1.0, X, dY, 0.0, dF)
    assert ctx.relayout_stats()["bytes_held"] == 0
    assert rel_fro(Y.get(), oracle.conv_fwd(od, 1.0, hx, hf)) <= TOL[dm.F16]
    assert rel_fro(dF.get(), oracle.conv_bwd_filter(od, 1.0, hx, hy)) <= TOL[dm.F16]
    # with room again (and fresh plans) the specialised path comes back
    filler.destroy()
    ctx.tune_reset()
    dm.conv_fwd(ctx, d, 1.0, X, F, 0.0, Y)
    assert ctx.relayout_stats()["bytes_held"] > 0
    assert rel_fro(Y.get(), oracle.conv_fwd(od, 1.0, hx, hf)) <= TOL[dm.F16]
    # room for the copies (0.9 MB) but not for the partial sums of a forward pass whose k-loop is
    # split (4 tiles: the cost model wants at least 2 parts of 1 MB each): same kernel, unsplit
    ctx.tune_reset()
    assert ctx.relayout_stats()["bytes_held"] == 0
    filler = fill_pool((1 << 20) + (600 << 10))
    dm.conv_fwd(ctx, d, 1.0, X, F, 0.0, Y)
    assert ctx.relayout_stats()["bytes_held"] > 0            # the specialised kernel's copies
    assert ctx.pool_stats()["capacity"] - ctx.pool_stats()["in_use"] < 1 << 20
    assert rel_fro(Y.get(), oracle.conv_fwd(od, 1.0, hx, hf)) <= TOL[dm.F16]
    filler.destroy()
    ctx.close()
