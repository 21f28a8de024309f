"""Pool accounting after tear-down (paper section 1: GPU memory is pooled and reused, so whatever
an operation takes from the pool beyond its operands must come back when its matrices go):
plans with padded k-tail panels, split-K partial sums, the copies and partial sums of the three
convolution modes, a recorded pipeline and timing samples all return their memory."""
import numpy as np
import pytest

import paper_1611_07819_amd as dm
from gpu_util import TOL, rel_fro

pytestmark = pytest.mark.gpu


@pytest.fixture()
def ctx():
    import torch
    stream = torch.cuda.Stream()          # recording needs a non-default stream (default priority)
    slab = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    c = dm.Context(slab, stream=stream.cuda_stream)
    yield c
    c.close()


def _round_trip(ctx, oracle, base):
    r = np.random.default_rng(4100)
    made = []

    def up(a, grid=(1, 1)):
        m = ctx.from_host(a, grid)
        made.append(m)
        return m

    def new(rows, cols, grid=(1, 1), dt=dm.F32):
        m = ctx.matrix(rows, cols, grid, dt)
        made.append(m)
        return m

    # K = 1000: the last 40 elements of the k-loop go through zero-padded scratch panels
    A = r.uniform(-1, 1, (512, 1000)).astype(np.float16)
    B = r.uniform(-1, 1, (1000, 256)).astype(np.float16)
    dA, dB, dC = up(A), up(B), new(512, 256)
    info = dm.gemm_plan_info(ctx, 0, 0, dA, dB, dC)
    assert info["kernel"] > 0 and info["workspace_bytes"] > 0, info     # specialised kernel + scratch panels
    dm.gemm(ctx, 0, 0, 1.0, dA, dB, 0.0, dC)
    assert rel_fro(dC.get(), oracle.gemm(False, False, 1.0, A, B, 0.0)) <= TOL[dm.F16]
    # deep K, few tiles: split-K partial sums
    A2 = r.uniform(-1, 1, (96, 8192)).astype(np.float32)
    B2 = r.uniform(-1, 1, (8192, 80)).astype(np.float32)
    dA2, dB2, dC2 = up(A2, (1, 2)), up(B2, (2, 1)), new(96, 80)
    info = dm.gemm_plan_info(ctx, 0, 0, dA2, dB2, dC2)
    assert info["split_k"] > 1 and info["workspace_bytes"] > 0, info
    dm.gemm(ctx, 0, 0, 1.0, dA2, dB2, 0.0, dC2)
    assert rel_fro(dC2.get(), oracle.gemm(False, False, 1.0, A2, B2, 0.0)) <= TOL[dm.F32]
    # the three convolution modes (channels-last copies, permuted filters, partial sums)
    g = dict(n=4, c=64, h=14, w=14, k=64, r=3, s=3, pad_h=1, pad_w=1)
    d = dm.ConvDesc(**g)
    x = r.uniform(0, 1, (4, 64 * 196)).astype(np.float16)
    f = r.normal(0, 0.05, (64, 64 * 9)).astype(np.float16)
    dy = r.normal(0, 0.1, (4, 64 * 196)).astype(np.float16)
    dx_, df_, ddy = up(x), up(f), up(dy)
    y, gf, gx = new(4, 64 * 196), new(64, 64 * 9), new(4, 64 * 196)
    dm.conv_fwd(ctx, d, 1.0, dx_, df_, 0.0, y)
    dm.conv_bwd_filter(ctx, d, 1.0, dx_, ddy, 0.0, gf)
    dm.conv_bwd_data(ctx, d, 1.0, ddy, df_, 0.0, gx)
    od = oracle.ConvDesc(**g)
    assert rel_fro(y.get(), oracle.conv_fwd(od, 1.0, x, f)) <= TOL[dm.F16]
    assert rel_fro(gf.get(), oracle.conv_bwd_filter(od, 1.0, x, dy)) <= TOL[dm.F16]
    assert rel_fro(gx.get(), oracle.conv_bwd_data(od, 1.0, dy, f)) <= TOL[dm.F16]
    assert ctx.relayout_stats()["bytes_held"] > 0
    # a recorded pipeline over the plans made above
    ctx.pipeline_begin()
    dm.gemm(ctx, 0, 0, 1.0, dA, dB, 0.0, dC)
    dm.gemm(ctx, 0, 0, 1.0, dA2, dB2, 0.0, dC2)
    dm.conv_fwd(ctx, d, 1.0, dx_, df_, 0.0, y)
    pid = ctx.pipeline_end()
    ctx.pipeline_replay(pid)
    assert rel_fro(dC.get(), oracle.gemm(False, False, 1.0, A, B, 0.0)) <= TOL[dm.F16]
    # timing samples of a GEMM and of a convolution
    assert dm.gemm_tune(ctx, 0, 0, dA2, dB2, dC2, 1 << 28, trials=2)["candidates"] >= 1
    assert dm.conv_tune(ctx, 1, d, dx_, gf, ddy, 1 << 28, trials=2)["candidates"] >= 1
    dm.gemm(ctx, 0, 0, 1.0, dA2, dB2, 0.0, dC2)           # plans on the tuner's choices
    dm.conv_bwd_filter(ctx, d, 1.0, dx_, ddy, 0.0, gf)
    ctx.synchronize()
    assert ctx.pool_stats()["in_use"] > base
    for m in made:
        m.destroy()
    ctx.synchronize()


def test_pool_returns_to_its_baseline_after_teardown(ctx, oracle):
    keep = ctx.from_host(np.ones((32, 32), np.float32))    # something that stays allocated
    base = ctx.pool_stats()["in_use"]
    for _ in range(2):                                      # the second pass reuses the first one's holes
        _round_trip(ctx, oracle, base)
        assert ctx.pool_stats()["in_use"] == base
        assert ctx.relayout_stats()["bytes_held"] == 0
    high = ctx.pool_stats()["high_water"]
    _round_trip(ctx, oracle, base)
    assert ctx.pool_stats()["high_water"] == high           # no growth from pass to pass: nothing leaks
    ctx.tune_reset()
    assert ctx.pool_stats()["in_use"] == base
    keep.destroy()
    assert ctx.pool_stats()["in_use"] == 0
