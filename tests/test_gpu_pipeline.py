"""Pipeline record / replay (paper section 3.3: a fixed forward+backward sequence is remembered
and re-issued through one identifier): every replay must equal the eager result for the
contents the matrices hold at replay time."""
import numpy as np
import pytest

import paper_1611_07819_amd as dm
from gpu_util import TOL, rel_fro

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import torch
    stream = torch.cuda.Stream()          # capture needs a non-default stream (default priority)
    slab = torch.empty(2 << 30, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    c = dm.Context(slab, stream=stream.cuda_stream)
    yield c
    c.close()


def test_replay_equals_eager_on_current_contents(ctx, oracle):
    r = np.random.default_rng(800)
    b, i, o = 512, 1024, 768
    X = r.uniform(0, 1, (b, i)).astype(np.float16)
    W = r.normal(0, 1 / 32, (i, o)).astype(np.float16)
    dY = r.normal(0, 0.1, (b, o)).astype(np.float16)
    g = (2, 2)
    dX_, dW_, ddY = ctx.from_host(X, g), ctx.from_host(W, g), ctx.from_host(dY, g)
    Y, gW, gX = ctx.matrix(b, o, g, dm.F32), ctx.matrix(i, o, g, dm.F32), ctx.matrix(b, i, g, dm.F32)
    # a small convolution rides along in the same pipeline
    geo = dict(n=4, c=128, h=16, w=16, k=256, r=3, s=3, pad_h=1, pad_w=1)
    cd = dm.ConvDesc(**geo)
    cx = r.uniform(0, 1, (4, 128 * 256)).astype(np.float16)
    cf = r.normal(0, 0.05, (256, 128 * 9)).astype(np.float16)
    dcx, dcf = ctx.from_host(cx), ctx.from_host(cf)
    dcy = ctx.matrix(4, 256 * 256, (1, 1), dm.F32)

    def step():
        dm.gemm(ctx, 0, 0, 1.0, dX_, dW_, 0.0, Y)
        dm.gemm(ctx, 1, 0, 1.0, dX_, ddY, 0.0, gW)
        dm.gemm(ctx, 0, 1, 1.0, ddY, dW_, 0.0, gX)
        dm.conv_fwd(ctx, cd, 1.0, dcx, dcf, 0.0, dcy)

    def outputs():
        return [m.get() for m in (Y, gW, gX, dcy)]

    step()                                   # eager: builds the plans
    eager0 = outputs()
    ctx.pipeline_begin()
    with pytest.raises(dm.DmathError) as e:  # not allowed while recording
        dX_.set(X)
    assert e.value.code == 7
    step()
    pid = ctx.pipeline_end()
    for rep in range(3):
        # new contents each time, eager work and synchronisation between the replays
        X2 = r.uniform(0, 1, (b, i)).astype(np.float16)
        cx2 = r.uniform(0, 1, cx.shape).astype(np.float16)
        dX_.set(X2)
        dcx.set(cx2)
        for m in (Y, gW, gX, dcy):
            m.set(np.full((m.rows, m.cols), np.nan, np.float32))
        ctx.pipeline_replay(pid)
        replayed = outputs()
        step()
        eager = outputs()
        for a, bb in zip(replayed, eager):
            assert np.array_equal(a, bb)     # same kernels, same order: bitwise
        assert rel_fro(replayed[0], oracle.gemm(False, False, 1.0, X2, W, 0.0)) <= TOL[dm.F16]
        assert rel_fro(replayed[3], oracle.conv_fwd(oracle.ConvDesc(**geo), 1.0, cx2, cf)) <= TOL[dm.F16]
    assert not np.array_equal(eager0[0], replayed[0])
    ctx.pipeline_destroy(pid)
    with pytest.raises(dm.DmathError):
        ctx.pipeline_replay(pid)


def test_recording_an_operation_without_a_plan_is_refused(ctx):
    A = ctx.from_host(np.ones((128, 128), np.float32))
    B = ctx.from_host(np.ones((128, 128), np.float32))
    C = ctx.matrix(128, 128, (1, 1), dm.F32)
    ctx.pipeline_begin()
    with pytest.raises(dm.DmathError) as e:
        dm.gemm(ctx, 0, 0, 1.0, A, B, 0.0, C)    # never run eagerly: no plan
    assert e.value.code == 7
    pid = ctx.pipeline_end()                       # an empty pipeline is fine
    ctx.pipeline_replay(pid)
    ctx.pipeline_destroy(pid)
    dm.gemm(ctx, 0, 0, 1.0, A, B, 0.0, C)
    assert np.array_equal(C.get(), np.full((128, 128), 128, np.float32))


def test_replay_with_workspaces_split_k_and_weight_gradient(ctx, oracle):
    """Operations that go through pool workspaces (split-K partial sums and their reduction
    kernel, the weight gradient's partial sums, accumulation with beta = 1) replayed three times
    on changing inputs: every replay must equal the eager run bit for bit and the oracle."""
    r = np.random.default_rng(801)
    M, N, K = 64, 512, 4096                       # few tiles, deep K: split-K + reduction kernel
    A = r.integers(-2, 3, (M, K)).astype(np.float16)
    B = r.integers(-2, 3, (K, N)).astype(np.float16)
    dA, dB, dC = ctx.from_host(A), ctx.from_host(B), ctx.matrix(M, N, (1, 1), dm.F32)
    assert dm.gemm_plan_info(ctx, 0, 0, dA, dB, dC)["split_k"] > 1
    geo = dict(n=4, c=128, h=16, w=16, k=256, r=3, s=3, pad_h=1, pad_w=1)
    cd, od = dm.ConvDesc(**geo), oracle.ConvDesc(**geo)
    hx = r.integers(-1, 2, (4, 128 * 256)).astype(np.float16)
    hy = r.integers(-1, 2, (4, 256 * 256)).astype(np.float16)
    dX, dY = ctx.from_host(hx), ctx.from_host(hy)
    dF = ctx.matrix(256, 128 * 9, (1, 1), dm.F32)

    def step():
        dm.gemm(ctx, 0, 0, 1.0, dA, dB, 1.0, dC)                 # accumulates into C
        dm.conv_bwd_filter(ctx, cd, 1.0, dX, dY, 0.0, dF)

    dC.set(np.zeros((M, N), np.float32))
    step()
    ctx.pipeline_begin()
    step()
    pid = ctx.pipeline_end()
    for rep in range(3):
        A2 = r.integers(-2, 3, (M, K)).astype(np.float16)
        x2 = r.integers(-1, 2, hx.shape).astype(np.float16)
        c0 = r.integers(-3, 4, (M, N)).astype(np.float32)
        dA.set(A2); dX.set(x2); dC.set(c0)
        ctx.pipeline_replay(pid)
        got_c, got_f = dC.get(), dF.get()
        assert np.array_equal(got_c.astype(np.float64), oracle.gemm(False, False, 1.0, A2, B, 1.0, c0))
        assert np.array_equal(got_f.astype(np.float64), oracle.conv_bwd_filter(od, 1.0, x2, hy))
        dC.set(c0)
        step()
        assert np.array_equal(dC.get(), got_c) and np.array_equal(dF.get(), got_f)
    ctx.pipeline_destroy(pid)


def test_replay_refreshes_the_padded_k_tails(ctx, oracle):
    """A GEMM whose K is not a multiple of the kernel's k-step reads the end of K from scratch
    panels that a copy kernel refreshes before the GEMM kernel; that copy is part of the
    recorded sequence, so a replay on new operands must see their last columns (integer data,
    bit for bit; fp32 forward and the fp32 convolution path beside it)."""
    r = np.random.default_rng(802)
    M, N, K = 256, 384, 1000
    A = r.integers(-2, 3, (M, K)).astype(np.float32)
    B = r.integers(-2, 3, (K, N)).astype(np.float32)
    dA, dB, dC = ctx.from_host(A), ctx.from_host(B), ctx.matrix(M, N, (1, 1), dm.F32)
    assert dm.gemm_plan_info(ctx, 0, 0, dA, dB, dC)["kernel"] != 0
    geo = dict(n=4, c=64, h=12, w=12, k=64, r=3, s=3, pad_h=1, pad_w=1)
    cd, od = dm.ConvDesc(**geo), oracle.ConvDesc(**geo)
    hx = r.integers(-1, 2, (4, 64 * 144)).astype(np.float32)
    hf = r.integers(-1, 2, (64, 64 * 9)).astype(np.float32)
    dX, dF, dY = ctx.from_host(hx), ctx.from_host(hf), ctx.matrix(4, 64 * 144, (1, 1), dm.F32)

    def step():
        dm.gemm(ctx, 0, 0, 1.0, dA, dB, 0.0, dC)
        dm.conv_fwd(ctx, cd, 1.0, dX, dF, 0.0, dY)

    step()
    ctx.pipeline_begin()
    step()
    pid = ctx.pipeline_end()
    for rep in range(3):
        A2 = A.copy()
        A2[:, K - 8:] = r.integers(-2, 3, (M, 8))          # only the tail of K changes
        B2 = B.copy()
        B2[K - 8:, :] = r.integers(-2, 3, (8, N))
        x2 = r.integers(-1, 2, hx.shape).astype(np.float32)
        dA.set(A2); dB.set(B2); dX.set(x2)
        dC.set(np.full((M, N), np.nan, np.float32))
        ctx.pipeline_replay(pid)
        assert np.array_equal(dC.get().astype(np.float64), oracle.gemm(False, False, 1.0, A2, B2, 0.0))
        assert np.array_equal(dY.get().astype(np.float64), oracle.conv_fwd(od, 1.0, x2, hf))
    ctx.pipeline_destroy(pid)


def test_replay_with_split_last_rounds(ctx, oracle, monkeypatch):
    """A GEMM whose tiles after the last full round of workgroups are split (two launches over
    views of one tile table and a reduction over those tiles) and a convolution forward pass
    whose (r, s, c) loop is split, recorded and replayed three times on changing inputs: every
    replay equals the eager run bit for bit and the oracle on sampled rows."""
    monkeypatch.setenv("DMATH_TILE", "128x64")
    monkeypatch.setenv("DMATH_GEMM_SPLIT", "4t")
    monkeypatch.setenv("DMATH_CONV_SPLIT", "3")
    r = np.random.default_rng(803)
    M, N, K = 1300, 4128, 256                     # 715 tiles of 128x64 on 512 workgroup slots
    A = r.integers(-2, 3, (M, K)).astype(np.float32)
    B = r.integers(-2, 3, (K, N)).astype(np.float32)
    dA, dB, dC = ctx.from_host(A), ctx.from_host(B), ctx.matrix(M, N, (1, 1), dm.F32)
    info = dm.gemm_plan_info(ctx, 0, 0, dA, dB, dC)
    assert info["split_k"] == 4 and 0 < info["split_tiles"] < info["tiles"], info
    geo = dict(n=3, c=128, h=14, w=14, k=256, r=3, s=3, pad_h=1, pad_w=1)
    cd, od = dm.ConvDesc(**geo), oracle.ConvDesc(**geo)
    hx = r.integers(-1, 2, (3, 128 * 196)).astype(np.float16)
    hf = r.integers(-1, 2, (256, 128 * 9)).astype(np.float16)
    dX, dF = ctx.from_host(hx), ctx.from_host(hf)
    dY = ctx.matrix(3, 256 * 196, (1, 1), dm.F32)
    rows = list(range(0, M, 97)) + [M - 1]

    def step():
        dm.gemm(ctx, 0, 0, 1.0, dA, dB, 1.0, dC)                 # accumulates into C
        dm.conv_fwd(ctx, cd, 1.0, dX, dF, 0.0, dY)

    dC.set(np.zeros((M, N), np.float32))
    step()
    ctx.pipeline_begin()
    step()
    pid = ctx.pipeline_end()
    for rep in range(3):
        A2 = r.integers(-2, 3, (M, K)).astype(np.float32)
        x2 = r.integers(-1, 2, hx.shape).astype(np.float16)
        c0 = r.integers(-3, 4, (M, N)).astype(np.float32)
        dA.set(A2); dX.set(x2); dC.set(c0)
        ctx.pipeline_replay(pid)
        got_c, got_y = dC.get(), dY.get()
        assert np.array_equal(got_c[rows].astype(np.float64), oracle.gemm(False, False, 1.0, A2, B, 1.0, c0, rows=rows))
        assert np.array_equal(got_y.astype(np.float64), oracle.conv_fwd(od, 1.0, x2, hf))
        dC.set(c0)
        step()
        assert np.array_equal(dC.get(), got_c) and np.array_equal(dY.get(), got_y)
    ctx.pipeline_destroy(pid)
    ctx.tune_reset()                              # drop the plans made under the overrides
    for m in (dA, dB, dC, dX, dF, dY):
        m.destroy()
