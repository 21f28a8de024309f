"""GPU parity of dmath_gemm against the CPU oracle, through the C ABI (needs an MI355X).

Bars (relative Frobenius error over the whole result, by input precision): 1e-12 fp64,
1e-5 fp32, 2e-3 fp16 inputs with fp32 accumulation (either output type); bitwise equality on
small-integer inputs, where every summation order gives the same bits."""
import itertools

import numpy as np
import pytest

import paper_1611_07819_amd as dm
from paper_1611_07819_amd import synth
from gpu_util import TOL, CODE, make_context, rel_fro

pytestmark = pytest.mark.gpu

NP = {dm.F64: np.float64, dm.F32: np.float32, dm.F16: np.float16}
OPS = list(itertools.product([0, 1], repeat=2))


@pytest.fixture(scope="module")
def ctx():
    c = make_context(6.0)
    yield c
    c.close()


def stored(op_mat, trans):
    return np.ascontiguousarray(op_mat.T if trans else op_mat)


def run_gemm(ctx, oracle, ta, tb, alpha, opA, opB, beta, C0, grids, out_dtype=None, rows=None,
             policy=0):
    """op(A) = opA, op(B) = opB are given logically; they are stored transposed when ta/tb."""
    A, B = stored(opA, ta), stored(opB, tb)
    ga, gb, gc = grids
    ctx.set_kernel_policy(policy)
    dA, dB = ctx.from_host(A, ga), ctx.from_host(B, gb)
    C0 = C0 if out_dtype is None else C0.astype(NP[out_dtype])
    dC = ctx.from_host(C0, gc)
    dm.gemm(ctx, ta, tb, alpha, dA, dB, beta, dC)
    got = dC.get()
    ref = oracle.gemm(bool(ta), bool(tb), alpha, oracle.BlockMatrix(A, ga), oracle.BlockMatrix(B, gb),
                      beta, oracle.BlockMatrix(C0, gc), rows=rows)
    for m in (dA, dB, dC):
        m.destroy()
    return got if rows is None else got[rows], ref


@pytest.mark.parametrize("policy", [0, 1])
@pytest.mark.parametrize("dt", [dm.F64, dm.F32, dm.F16])
@pytest.mark.parametrize("ta,tb", OPS)
def test_ragged_multi_tile_all_ops(ctx, oracle, dt, ta, tb, policy):
    # several tiles in every direction, ragged tails, grids that do not line up
    r = np.random.default_rng(100 + dt)
    M, N, K = 150, 203, 117
    opA = r.uniform(-1, 1, (M, K)).astype(NP[dt])
    opB = r.uniform(-1, 1, (K, N)).astype(NP[dt])
    C0 = r.uniform(-1, 1, (M, N)).astype(NP[dt])
    for grids in [((1, 1), (1, 1), (1, 1)), ((2, 3), (2, 2), (3, 2))]:
        got, ref = run_gemm(ctx, oracle, ta, tb, 1.5, opA, opB, -0.5, C0, grids, policy=policy)
        assert rel_fro(got, ref) <= TOL[dt]
        assert np.abs(got.astype(np.float64) - ref).max() <= 50 * TOL[dt] * np.abs(ref).max()


@pytest.mark.parametrize("policy", [0, 1])
@pytest.mark.parametrize("dt,out", [(dm.F64, dm.F64), (dm.F32, dm.F32), (dm.F16, dm.F32), (dm.F16, dm.F16)])
@pytest.mark.parametrize("ta,tb", OPS)
def test_small_integers_are_bitwise_exact(ctx, oracle, dt, out, ta, tb, policy):
    # entries in {-3..3}: all partial sums are exactly representable, so any summation order,
    # tiling or split-K must reproduce the oracle bit for bit.  |result| <= 2048 for fp16 out.
    r = np.random.default_rng(200)
    M, N, K = 192, 130, 96
    opA = r.integers(-3, 4, (M, K)).astype(NP[dt])
    opB = r.integers(-3, 4, (K, N)).astype(NP[dt])
    C0 = r.integers(-3, 4, (M, N)).astype(NP[out])
    for grids in [((1, 1), (1, 1), (1, 1)), ((3, 2), (2, 2), (2, 2)), ((4, 3), (3, 5), (5, 4))]:
        got, ref = run_gemm(ctx, oracle, ta, tb, 2.0, opA, opB, 1.0, C0, grids, out_dtype=out,
                            policy=policy)
        assert np.array_equal(got.astype(np.float64), ref)


@pytest.mark.parametrize("dt", [dm.F64, dm.F32, dm.F16])
def test_deep_k_uses_split_k_and_stays_exact(ctx, oracle, dt):
    r = np.random.default_rng(201)
    M, N, K = 96, 80, 8192
    opA = r.integers(-1, 2, (M, K)).astype(NP[dt])
    opB = r.integers(-1, 2, (K, N)).astype(NP[dt])
    C0 = r.integers(-3, 4, (M, N)).astype(NP[dt])
    dA, dB, dC = ctx.from_host(opA, (1, 3)), ctx.from_host(opB, (2, 1)), ctx.from_host(C0, (1, 1))
    info = dm.gemm_plan_info(ctx, 0, 0, dA, dB, dC)
    assert info["split_k"] > 1 and info["workspace_bytes"] > 0
    dm.gemm(ctx, 0, 0, 1.0, dA, dB, 1.0, dC)
    got = dC.get()
    ref = oracle.gemm(False, False, 1.0, opA, opB, 1.0, C0)
    assert np.array_equal(got.astype(np.float64), ref)
    for m in (dA, dB, dC):
        m.destroy()


@pytest.mark.parametrize("dt", [dm.F64, dm.F32, dm.F16])
def test_identity_and_alpha_beta_rules(ctx, oracle, dt):
    r = np.random.default_rng(202)
    n = 100
    A = r.uniform(-1, 1, (n, n)).astype(NP[dt])
    I = np.eye(n, dtype=NP[dt])
    C0 = r.uniform(-1, 1, (n, n)).astype(NP[dt])
    got, _ = run_gemm(ctx, oracle, 0, 0, 1.0, A, I, 0.0, C0, ((2, 2), (2, 2), (2, 2)))
    assert np.array_equal(got, A)
    got, _ = run_gemm(ctx, oracle, 1, 0, 1.0, A, I, 0.0, C0, ((2, 2), (2, 2), (2, 2)))
    assert np.array_equal(got, A)                      # op(A) was given logically
    nan = np.full((n, n), np.nan, NP[dt])
    got, ref = run_gemm(ctx, oracle, 0, 0, 1.0, A, I, 0.0, nan, ((1, 1),) * 3)
    assert np.array_equal(got, A)                      # beta == 0: old C not read
    got, ref = run_gemm(ctx, oracle, 0, 0, 0.0, nan, I, 2.0, C0, ((1, 1),) * 3)
    assert np.array_equal(got.astype(np.float64), ref) # alpha == 0: A not read; C = 2*C0 exactly
    got, ref = run_gemm(ctx, oracle, 0, 0, 0.0, nan, nan, 0.0, nan, ((1, 1),) * 3)
    assert np.array_equal(got, np.zeros((n, n), NP[dt]))
    for (al, be) in [(1.0, 1.0), (1.5, -0.5)]:
        got, ref = run_gemm(ctx, oracle, 0, 0, al, A, A, be, C0, ((2, 1), (1, 2), (2, 2)))
        assert rel_fro(got, ref) <= TOL[dt]


def test_run_to_run_bitwise_reproducible(ctx):
    r = np.random.default_rng(203)
    A = r.uniform(-1, 1, (96, 4096)).astype(np.float32)
    B = r.uniform(-1, 1, (4096, 64)).astype(np.float32)
    dA, dB = ctx.from_host(A), ctx.from_host(B)
    outs = []
    for _ in range(3):
        dC = ctx.matrix(96, 64, (1, 1), dm.F32)
        dm.gemm(ctx, 0, 0, 1.0, dA, dB, 0.0, dC)
        outs.append(dC.get())
        dC.destroy()
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


def test_config1_full(ctx, oracle):
    w = synth.config1()
    m = w.mats
    got, ref = run_gemm(ctx, oracle, 0, 0, 1.0, m["A"], m["B"], 1.0, m["C"], (w.grid,) * 3)
    assert rel_fro(got, ref) <= TOL[dm.F32]


# per-element bound beside the norm: |got - ref| <= ELEM_C * tol * max|ref|
ELEM_C = 50


def assert_whole_result(got, ref, tol, what):
    """The whole result against the oracle's: relative Frobenius error and a per-element bound."""
    got = np.asarray(got, np.float64)
    assert got.shape == ref.shape, what
    err = rel_fro(got, ref)
    assert err <= tol, (what, err)
    worst = np.abs(got - ref).max()
    assert worst <= ELEM_C * tol * np.abs(ref).max(), (what, worst)


def _fc_workload(ctx, oracle, w, in_dt, policy=0, refs=None):
    """Every call of a fully-connected workload, the whole result of each against the oracle.
    `refs` (a dict) keeps the oracle's results by call name for a second pass over the same
    inputs with another output type (beta is 0 in these workloads)."""
    ctx.set_kernel_policy(policy)
    dev = {k: ctx.from_host(v, w.grid) for k, v in w.mats.items()}
    for call in w.calls:
        dm.gemm(ctx, int(call.transA), int(call.transB), call.alpha, dev[call.a], dev[call.b],
                call.beta, dev[call.c])
        got = dev[call.c].get()
        if refs is not None and call.name in refs:
            ref = refs[call.name]
        else:
            assert refs is None or call.beta == 0.0
            ref = oracle.gemm(call.transA, call.transB, call.alpha,
                              oracle.BlockMatrix(w.mats[call.a], w.grid),
                              oracle.BlockMatrix(w.mats[call.b], w.grid), call.beta,
                              oracle.BlockMatrix(w.mats[call.c], w.grid))
            if refs is not None:
                refs[call.name] = ref
        assert_whole_result(got, ref, TOL[in_dt], (w.name, call.name))
    for m in dev.values():
        m.destroy()


@pytest.mark.parametrize("policy", [0, 1])
def test_config2_scaled_whole_result(ctx, oracle, policy):
    _fc_workload(ctx, oracle, synth.config2(scale=8), dm.F32, policy)


def test_config2_full_size_whole_result(ctx, oracle):
    # forward, dW and dX at 1024 x 9216 x 4096 in the launch configuration the benchmark times
    _fc_workload(ctx, oracle, synth.config2(), dm.F32)


@pytest.mark.parametrize("out", ["f32", "f16"])
@pytest.mark.parametrize("policy", [0, 1])
def test_config3_scaled_whole_result(ctx, oracle, out, policy):
    _fc_workload(ctx, oracle, synth.config3(out, scale=8), dm.F16, policy)


def test_config3_full_size_whole_result(ctx, oracle):
    # both output types against one oracle run: the inputs are the same and beta is 0
    refs = {}
    for out in ("f32", "f16"):
        _fc_workload(ctx, oracle, synth.config3(out), dm.F16, refs=refs)
    assert len(refs) == 3


@pytest.mark.parametrize("policy", [0, 1])
def test_config4_scaled_whole_result(ctx, oracle, policy):
    w = synth.config4(scale=16)
    m = w.mats
    got, ref = run_gemm(ctx, oracle, 0, 0, 1.5, m["A"], m["B"], -0.5, m["C"], (w.grid,) * 3,
                        policy=policy)
    assert rel_fro(got, ref) <= TOL[dm.F64]


def test_config4_full_size_whole_result(ctx, oracle):
    w = synth.config4()
    m = w.mats
    got, ref = run_gemm(ctx, oracle, 0, 0, 1.5, m["A"], m["B"], -0.5, m["C"], (w.grid,) * 3)
    assert_whole_result(got, ref, TOL[dm.F64], w.name)


def test_fp16_path_agrees_with_fp32_path(ctx):
    # section 4.2: half mode "performs at par" with float.  Same fp16-representable data through
    # both paths: the only difference is the summation order of exact products.
    r = np.random.default_rng(204)
    A = r.uniform(0, 1, (256, 512)).astype(np.float16)
    B = r.normal(0, 1 / 16, (512, 128)).astype(np.float16)
    outs = []
    for dt in (np.float16, np.float32):
        dA, dB = ctx.from_host(A.astype(dt), (2, 2)), ctx.from_host(B.astype(dt), (2, 2))
        dC = ctx.matrix(256, 128, (2, 2), dm.F32)
        dm.gemm(ctx, 0, 0, 1.0, dA, dB, 0.0, dC)
        outs.append(dC.get())
        for m in (dA, dB, dC):
            m.destroy()
    assert rel_fro(outs[0], outs[1]) <= 1e-5


def test_pool_is_the_only_allocator(ctx):
    import torch
    before = torch.cuda.memory_allocated()
    A = ctx.from_host(np.ones((300, 300), np.float32), (2, 2))
    B = ctx.from_host(np.ones((300, 300), np.float32), (2, 2))
    C = ctx.matrix(300, 300, (2, 2), dm.F32)
    dm.gemm(ctx, 0, 0, 1.0, A, B, 0.0, C)
    assert np.array_equal(C.get(), np.full((300, 300), 300, np.float32))
    assert torch.cuda.memory_allocated() == before
    for m in (A, B, C):
        m.destroy()


FAST_CASES = [
    # dtype, (M, N, K), grids (A-as-op, B-as-op, C) chosen so that every segment is a whole
    # number of tiles and every k-segment a multiple of the k-step of the specialised kernels
    (dm.F32, (256, 384, 320), ((2, 2), (2, 2), (2, 2))),
    (dm.F32, (512, 256, 256), ((1, 1), (1, 1), (1, 1))),
    (dm.F32, (384, 256, 384), ((3, 2), (3, 2), (1, 2))),
    (dm.F16, (512, 256, 384), ((2, 2), (2, 2), (2, 2))),
    (dm.F16, (256, 384, 192), ((1, 3), (3, 1), (1, 1))),
    (dm.F16, (768, 256, 128), ((3, 1), (1, 2), (3, 2))),
    (dm.F64, (256, 384, 160), ((2, 2), (2, 2), (2, 2))),
    (dm.F64, (256, 128, 208), ((1, 1), (1, 1), (1, 1))),
    (dm.F64, (384, 256, 192), ((3, 2), (2, 2), (1, 2))),
    # K of one and two k-steps of the kernel: the load ring never fills (prologue and drain only)
    (dm.F32, (256, 256, 32), ((1, 1), (1, 1), (1, 1))),
    (dm.F32, (128, 256, 64), ((1, 2), (2, 1), (1, 1))),
    (dm.F16, (256, 256, 64), ((1, 1), (1, 1), (1, 1))),
    (dm.F16, (512, 256, 128), ((1, 2), (2, 1), (1, 1))),
    (dm.F64, (128, 128, 16), ((1, 1), (1, 1), (1, 1))),
    (dm.F64, (256, 128, 32), ((1, 2), (2, 1), (1, 1))),
    # K (or the K of a block) not a multiple of the kernel's k-step: the last elements of such a
    # segment go through zero-padded scratch panels (1000 output classes, 784 input pixels)
    (dm.F32, (256, 384, 1000), ((1, 1), (1, 1), (1, 1))),
    (dm.F32, (384, 256, 784), ((2, 2), (2, 2), (2, 2))),
    (dm.F32, (200, 300, 1000), ((1, 1), (1, 1), (1, 1))),
    (dm.F16, (256, 256, 1000), ((1, 1), (1, 1), (1, 1))),
    (dm.F16, (512, 256, 784), ((2, 1), (1, 2), (2, 2))),
    (dm.F16, (200, 296, 1000), ((1, 1), (1, 1), (1, 1))),
    (dm.F64, (256, 128, 200), ((1, 1), (1, 1), (1, 1))),
    (dm.F64, (128, 256, 1000), ((2, 1), (1, 2), (1, 1))),
]


@pytest.mark.parametrize("dt,mnk,grids", FAST_CASES)
@pytest.mark.parametrize("ta,tb", OPS)
def test_specialised_kernels_whole_result(ctx, oracle, dt, mnk, grids, ta, tb):
    """Sizes that satisfy the preconditions of the specialised kernels: the plan must pick one,
    the result must match the oracle within the precision's bar, and integer inputs must match
    bit for bit."""
    M, N, K = mnk
    r = np.random.default_rng(400 + M + N + K)
    ga, gb, gc = grids
    ga = ga[::-1] if ta else ga          # grids are given for op(A), op(B)
    gb = gb[::-1] if tb else gb
    for ints in (False, True):
        if ints:
            opA = r.integers(-3, 4, (M, K)).astype(NP[dt])
            opB = r.integers(-3, 4, (K, N)).astype(NP[dt])
            C0 = r.integers(-3, 4, (M, N)).astype(NP[dt])
        else:
            opA = r.uniform(-1, 1, (M, K)).astype(NP[dt])
            opB = r.uniform(-1, 1, (K, N)).astype(NP[dt])
            C0 = r.uniform(-1, 1, (M, N)).astype(NP[dt])
        ctx.set_kernel_policy(0)
        dA, dB, dC = ctx.from_host(stored(opA, ta), ga), ctx.from_host(stored(opB, tb), gb), ctx.from_host(C0, gc)
        assert dm.gemm_plan_info(ctx, ta, tb, dA, dB, dC)["kernel"] != 0
        for m in (dA, dB, dC):
            m.destroy()
        got, ref = run_gemm(ctx, oracle, ta, tb, 1.5 if not ints else 2.0, opA, opB,
                            -0.5 if not ints else 1.0, C0, (ga, gb, gc))
        if ints:
            assert np.array_equal(got.astype(np.float64), ref)
        else:
            assert rel_fro(got, ref) <= TOL[dt]


@pytest.mark.parametrize("dt,shape", [(dm.F16, "256x256"), (dm.F16, "256x128"), (dm.F16, "128x128"),
                                      (dm.F32, "128x128"), (dm.F32, "128x64"), (dm.F32, "128x96"),
                                      (dm.F64, "128x128"), (dm.F64, "128x64"),
                                      # the shapes offered to batches of at most 64 rows
                                      (dm.F16, "64x128"), (dm.F16, "64x64"), (dm.F32, "64x128"),
                                      (dm.F32, "64x256"), (dm.F64, "64x128")])
@pytest.mark.parametrize("ta,tb", OPS)
def test_every_tile_shape_of_the_specialised_kernels(ctx, oracle, dt, shape, ta, tb, monkeypatch):
    """The scheduler normally picks the tile shape by cost; DMATH_TILE pins it, so that every
    compiled shape is checked bit for bit on integer inputs (several k-tiles, several tiles,
    k-segments of different blocks)."""
    if shape == "128x96" and not tb:
        pytest.skip("the 128x96 fp32 tile needs a k-major B (transB = T)")
    monkeypatch.setenv("DMATH_TILE", shape)
    r = np.random.default_rng(500)
    M, N, K = 512, (576 if shape == "128x96" else 768), 448 if dt != dm.F16 else 448 + 64 * 3
    if shape.startswith("64x"):
        M = 128 - 16                     # two row blocks of 56 rows: ragged 64-row tiles, 16-byte aligned when stored transposed
    opA = r.integers(-2, 3, (M, K)).astype(NP[dt])
    opB = r.integers(-2, 3, (K, N)).astype(NP[dt])
    C0 = r.integers(-3, 4, (M, N)).astype(NP[dt])
    ga, gb, gc = (2, 1), (1, 3), (1, 1)
    ga = ga[::-1] if ta else ga
    gb = gb[::-1] if tb else gb
    ctx.set_kernel_policy(0)
    dA, dB, dC = ctx.from_host(stored(opA, ta), ga), ctx.from_host(stored(opB, tb), gb), ctx.from_host(C0, gc)
    info = dm.gemm_plan_info(ctx, ta, tb, dA, dB, dC)
    assert f"{info['tile_m']}x{info['tile_n']}" == shape and info["kernel"] != 0
    dm.gemm(ctx, ta, tb, 1.0, dA, dB, 1.0, dC)
    got = dC.get()
    ref = oracle.gemm(bool(ta), bool(tb), 1.0, oracle.BlockMatrix(stored(opA, ta), ga),
                      oracle.BlockMatrix(stored(opB, tb), gb), 1.0, oracle.BlockMatrix(C0, gc))
    assert np.array_equal(got.astype(np.float64), ref)
    for m in (dA, dB, dC):
        m.destroy()


@pytest.mark.parametrize("dt,out", [(dm.F64, dm.F64), (dm.F32, dm.F32), (dm.F16, dm.F32), (dm.F16, dm.F16)])
@pytest.mark.parametrize("ta,tb", [(0, 0), (1, 0), (0, 1)])
def test_specialised_kernels_with_split_k(ctx, oracle, dt, out, ta, tb):
    """Few C tiles, deep K: the specialised kernels split K over workgroups and a second kernel
    adds the partial sums in a fixed order.  Integer inputs: bit-for-bit; two runs: identical."""
    r = np.random.default_rng(600)
    M, N, K = 256, 384, 4096
    opA = r.integers(-1, 2, (M, K)).astype(NP[dt])
    opB = r.integers(-1, 2, (K, N)).astype(NP[dt])
    C0 = r.integers(-3, 4, (M, N)).astype(NP[out])
    ga, gb, gc = (1, 2), (2, 1), (1, 1)
    ga = ga[::-1] if ta else ga
    gb = gb[::-1] if tb else gb
    ctx.set_kernel_policy(0)
    dA, dB = ctx.from_host(stored(opA, ta), ga), ctx.from_host(stored(opB, tb), gb)
    ref = oracle.gemm(bool(ta), bool(tb), 1.0, oracle.BlockMatrix(stored(opA, ta), ga),
                      oracle.BlockMatrix(stored(opB, tb), gb), 1.0, oracle.BlockMatrix(C0, gc))
    outs = []
    for _ in range(2):
        dC = ctx.from_host(C0, gc)
        info = dm.gemm_plan_info(ctx, ta, tb, dA, dB, dC)
        assert info["kernel"] != 0 and info["split_k"] > 1 and info["workspace_bytes"] > 0
        dm.gemm(ctx, ta, tb, 1.0, dA, dB, 1.0, dC)
        outs.append(dC.get())
        dC.destroy()
    assert np.array_equal(outs[0].astype(np.float64), ref)
    assert np.array_equal(outs[0], outs[1])
    for m in (dA, dB):
        m.destroy()


@pytest.mark.parametrize("dt,out", [(dm.F64, dm.F64), (dm.F32, dm.F32), (dm.F16, dm.F32), (dm.F16, dm.F16)])
@pytest.mark.parametrize("ta,tb", OPS)
def test_specialised_kernels_on_ragged_tiles(ctx, oracle, dt, out, ta, tb):
    """M and N that are not multiples of any tile (but keep 16-byte alignment), K a multiple of the
    k-step: the specialised kernels run with a ragged last tile row/column.  Integer inputs:
    bit for bit; NaN-filled C with beta = 0 must not leak; neighbours of C must stay untouched."""
    r = np.random.default_rng(900)
    M, N, K = 152, 200, 192
    opA = r.integers(-2, 3, (M, K)).astype(NP[dt])
    opB = r.integers(-2, 3, (K, N)).astype(NP[dt])
    C0 = r.integers(-3, 4, (M, N)).astype(NP[out])
    ctx.set_kernel_policy(0)
    for grids in [((1, 1), (1, 1), (1, 1)), ((1, 3), (3, 1), (1, 1))]:
        ga, gb, gc = grids
        ga = ga[::-1] if ta else ga
        gb = gb[::-1] if tb else gb
        dA, dB, dC = ctx.from_host(stored(opA, ta), ga), ctx.from_host(stored(opB, tb), gb), ctx.from_host(C0, gc)
        guard = ctx.from_host(np.full((4, 64), 7, NP[out]))          # allocated right after C
        info = dm.gemm_plan_info(ctx, ta, tb, dA, dB, dC)
        assert info["kernel"] != 0, grids
        dm.gemm(ctx, ta, tb, 2.0, dA, dB, 1.0, dC)
        got = dC.get().astype(np.float64)
        ref = oracle.gemm(bool(ta), bool(tb), 2.0, oracle.BlockMatrix(stored(opA, ta), ga),
                          oracle.BlockMatrix(stored(opB, tb), gb), 1.0, oracle.BlockMatrix(C0, gc))
        assert np.array_equal(got, ref), grids
        dC.set(np.full((M, N), np.nan, NP[out]))
        dm.gemm(ctx, ta, tb, 1.0, dA, dB, 0.0, dC)
        ref0 = oracle.gemm(bool(ta), bool(tb), 1.0, stored(opA, ta), stored(opB, tb), 0.0)
        assert np.array_equal(dC.get().astype(np.float64), ref0), grids
        assert np.array_equal(guard.get(), np.full((4, 64), 7, NP[out]))
        for m in (dA, dB, dC, guard):
            m.destroy()


def test_block_beyond_4_gib_is_addressed_in_64_bits(ctx, oracle):
    """One block of B holds 4.6 GB: beyond the 32-bit lane offsets of the specialised kernels, so
    the plan must fall back to the kernel that indexes in 64 bits.  Small-integer data: rows of
    the result checked bit for bit, including k rows of B that lie beyond the 4 GiB mark."""
    M, K, N = 64, 8192, 278528
    assert K * N * 2 > 1 << 32
    A = ((np.arange(M * K, dtype=np.int64).reshape(M, K) * 7 + 3) % 5 - 2).astype(np.float16)
    B = np.empty((K, N), np.float16)
    col = (np.arange(N, dtype=np.int64) % 3 - 1).astype(np.float16)
    for k0 in range(0, K, 1024):                       # built in slices: no 18 GB int64 temporary
        kk = np.arange(k0, k0 + 1024, dtype=np.int64)
        B[k0:k0 + 1024] = ((kk % 4) - 1).astype(np.float16)[:, None] * col[None, :]
    ctx.set_kernel_policy(0)
    dA, dB = ctx.from_host(A), ctx.from_host(B)
    dC = ctx.matrix(M, N, (1, 1), dm.F32)
    info = dm.gemm_plan_info(ctx, 0, 0, dA, dB, dC)
    assert info["kernel"] == 0
    dm.gemm(ctx, 0, 0, 1.0, dA, dB, 0.0, dC)
    got = dC.get()
    rows = [0, 37, 63]
    ref = oracle.gemm(False, False, 1.0, A, B, 0.0, rows=rows)
    assert np.array_equal(got[rows].astype(np.float64), ref)
    # the same product restricted to the k rows beyond 4 GiB must not vanish (they are read)
    k_far = (1 << 32) // (N * 2) + 1
    far = A[rows][:, k_far:].astype(np.float64) @ B[k_far:, :4096].astype(np.float64)
    assert np.abs(far).max() > 0
    for m in (dA, dB, dC):
        m.destroy()


def test_cycle_probe_is_absent_from_the_product_library(ctx):
    with pytest.raises(dm.DmathError) as e:
        ctx.cycle_probe_read()
    assert e.value.code == 7                      # DMATH_ERR_UNSUPPORTED


def _valid_grid(r, n):
    """A random part count g for a dimension of length n that leaves no empty trailing part."""
    while True:
        g = int(r.integers(1, 5))
        step = -(-n // g)
        if (g - 1) * step < n:
            return g


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes_grids_ops_against_oracle(ctx, oracle, seed):
    """Seeded sweep over shapes (half of them multiples of 64 so that the specialised kernels and
    their ragged tiles are drawn, the rest arbitrary), independent random block grids for A, B
    and C, all ops, all precisions, random alpha and beta: small-integer data, bit for bit."""
    r = np.random.default_rng(7000 + seed)
    ctx.set_kernel_policy(0)
    for case in range(6):
        dt, out = [(dm.F64, dm.F64), (dm.F32, dm.F32), (dm.F16, dm.F32), (dm.F16, dm.F16)][int(r.integers(0, 4))]
        if r.integers(0, 2):
            M, N, K = (int(r.integers(1, 7)) * 64 + int(r.integers(0, 2)) * 8 for _ in range(3))
            K = K // 64 * 64
        else:
            M, N, K = (int(r.integers(1, 300)) for _ in range(3))
        ta, tb = int(r.integers(0, 2)), int(r.integers(0, 2))
        opA = r.integers(-2, 3, (M, K)).astype(NP[dt])
        opB = r.integers(-2, 3, (K, N)).astype(NP[dt])
        C0 = r.integers(-2, 3, (M, N)).astype(NP[out])
        A_st, B_st = stored(opA, ta), stored(opB, tb)
        ga = (_valid_grid(r, A_st.shape[0]), _valid_grid(r, A_st.shape[1]))
        gb = (_valid_grid(r, B_st.shape[0]), _valid_grid(r, B_st.shape[1]))
        gc = (_valid_grid(r, M), _valid_grid(r, N))
        alpha, beta = float(r.integers(-2, 3)), float(r.integers(-1, 2))
        dA, dB, dC = ctx.from_host(A_st, ga), ctx.from_host(B_st, gb), ctx.from_host(C0, gc)
        dm.gemm(ctx, ta, tb, alpha, dA, dB, beta, dC)
        ref = oracle.gemm(bool(ta), bool(tb), alpha, oracle.BlockMatrix(A_st, ga), oracle.BlockMatrix(B_st, gb),
                          beta, oracle.BlockMatrix(C0, gc))
        what = (seed, case, dt, out, (M, N, K), (ta, tb), ga, gb, gc, alpha, beta)
        if out == dm.F16 and np.abs(ref).max() > 2048:
            assert rel_fro(dC.get(), ref) <= TOL[dt], what
        else:
            assert np.array_equal(dC.get().astype(np.float64), ref), what
        for m in (dA, dB, dC):
            m.destroy()


@pytest.mark.parametrize("tile", ["256x256", "256x128", "128x128"])
@pytest.mark.parametrize("ta,tb", [(0, 1), (1, 0)])
def test_fp16_every_k_tile_count_per_tile_shape(oracle, monkeypatch, tile, ta, tb):
    """1 to 17 k-tiles of 64 on each tile shape of the 16x16x32 pipeline: the k-loop is unrolled
    into differently scheduled first, steady and last iterations, and every count takes another
    path through them (a stale accumulator register once showed only for some counts).  C is left
    as allocated, beta = 0; small integers, bit for bit."""
    monkeypatch.setenv("DMATH_TILE", tile)
    r = np.random.default_rng(270)
    c = make_context(0.5)
    try:
        M = N = 512
        for n in range(1, 18):
            K = 64 * n
            opA = r.integers(-3, 4, (M, K)).astype(np.float16)
            opB = r.integers(-3, 4, (K, N)).astype(np.float16)
            A, B = stored(opA, ta), stored(opB, tb)
            dA, dB = c.from_host(A), c.from_host(B)
            dC = c.matrix(M, N, (1, 1), dm.F32)
            info = dm.gemm_plan_info(c, ta, tb, dA, dB, dC)
            assert f"{info['tile_m']}x{info['tile_n']}" == tile and info["kernel"] > 0, info
            dm.gemm(c, ta, tb, 1.0, dA, dB, 0.0, dC)
            got = dC.get().astype(np.float64)
            ref = oracle.gemm(bool(ta), bool(tb), 1.0, A, B, 0.0)
            assert np.array_equal(got, ref), (tile, n, int((got != ref).sum()))
            for m in (dA, dB, dC):
                m.destroy()
    finally:
        c.close()


@pytest.mark.parametrize("tile", ["256x256", "256x128", "128x128"])
def test_fp16_k_segments_and_splits_per_tile_shape(oracle, monkeypatch, tile):
    """The k-loop of the 16x16x32 pipeline over several k-segments (block boundaries of A and B
    along k: the walk reloads its panel descriptors inside the loop) and split into parts, on
    each tile shape, beta = 0 and 1; small integers, bit for bit."""
    monkeypatch.setenv("DMATH_TILE", tile)
    r = np.random.default_rng(271)
    c = make_context(0.5)
    try:
        M = N = 512
        for K, gk in ((512, 4), (512, 1), (768, 3), (1024, 8), (256, 2), (512, 2), (1280, 5)):
            for beta in (0.0, 1.0):
                A = r.integers(-3, 4, (M, K)).astype(np.float16)
                B = r.integers(-3, 4, (K, N)).astype(np.float16)
                C0 = r.integers(-3, 4, (M, N)).astype(np.float32)
                dA, dB, dC = c.from_host(A, (1, gk)), c.from_host(B, (gk, 1)), c.from_host(C0)
                info = dm.gemm_plan_info(c, 0, 0, dA, dB, dC)
                assert f"{info['tile_m']}x{info['tile_n']}" == tile and info["kernel"] > 0, info
                dm.gemm(c, 0, 0, 1.0, dA, dB, beta, dC)
                got = dC.get().astype(np.float64)
                ref = oracle.gemm(False, False, 1.0, oracle.BlockMatrix(A, (1, gk)), oracle.BlockMatrix(B, (gk, 1)),
                                  beta, C0)
                assert np.array_equal(got, ref), (tile, K, gk, beta, info["split_k"], int((got != ref).sum()))
                for m in (dA, dB, dC):
                    m.destroy()
    finally:
        c.close()


@pytest.mark.parametrize("dt,out,tile,shape", [
    (dm.F32, dm.F32, "128x64", (1300, 4128, 256)),     # 11 x 65 = 715 tiles on 512 workgroup slots
    (dm.F64, dm.F64, "128x64", (1300, 4128, 256)),
    (dm.F16, dm.F32, "256x128", (2400, 4128, 512)),    # 10 x 33 = 330 tiles on 256 slots
    (dm.F16, dm.F16, "256x128", (2400, 4128, 512)),
])
@pytest.mark.parametrize("ta,tb", [(0, 0), (1, 0), (0, 1)])
def test_split_of_the_tiles_after_the_last_full_round(oracle, monkeypatch, dt, out, tile, shape, ta, tb):
    """More tiles than one round of workgroups holds: the tiles of the full rounds run the whole
    k-loop and store C, the rest are split into four parts with a compact workspace of their own
    and reduced in a fixed order (forced here; the cost model takes the same path where it pays).
    Ragged last tiles in both directions; small-integer data, bit for bit; sampled rows of a
    random case within the precision's bar."""
    monkeypatch.setenv("DMATH_TILE", tile)
    monkeypatch.setenv("DMATH_GEMM_SPLIT", "4t")
    M, N, K = shape
    r = np.random.default_rng(260)
    c = make_context(1.0)
    try:
        opA = r.integers(-2, 3, (M, K)).astype(NP[dt])
        opB = r.integers(-2, 3, (K, N)).astype(NP[dt])
        C0 = r.integers(-2, 3, (M, N)).astype(NP[out])
        A, B = stored(opA, ta), stored(opB, tb)
        dA, dB, dC = c.from_host(A), c.from_host(B), c.from_host(C0)
        info = dm.gemm_plan_info(c, ta, tb, dA, dB, dC)
        assert info["kernel"] > 0 and info["split_k"] == 4 and 0 < info["split_tiles"] < info["tiles"], info
        slots = 512 if dt != dm.F16 else 256
        assert info["tiles"] - info["split_tiles"] == info["tiles"] // slots * slots
        dm.gemm(c, ta, tb, 1.0, dA, dB, 1.0, dC)
        rows = list(range(0, M, 37)) + [M - 1]
        ref = oracle.gemm(bool(ta), bool(tb), 1.0, A, B, 1.0, C0, rows=rows)
        got = dC.get()[rows].astype(np.float64)
        if out == dm.F16 and np.abs(ref).max() > 2048:
            assert rel_fro(got, ref) <= TOL[dt]
        else:
            assert np.array_equal(got, ref)
        # random data, alpha and beta, on the same plan
        ra = r.uniform(-1, 1, A.shape).astype(NP[dt])
        rb = r.uniform(-1, 1, B.shape).astype(NP[dt])
        rc = r.uniform(-1, 1, (M, N)).astype(NP[out])
        dA.set(ra), dB.set(rb), dC.set(rc)
        dm.gemm(c, ta, tb, 1.5, dA, dB, -0.5, dC)
        ref = oracle.gemm(bool(ta), bool(tb), 1.5, ra, rb, -0.5, rc, rows=rows)
        assert rel_fro(dC.get()[rows], ref) <= TOL[dt]
    finally:
        c.close()


@pytest.mark.parametrize("seed", range(6))
def test_random_shapes_with_partial_last_rounds(ctx, oracle, seed):
    """Seeded shapes whose tile count is a little more than whole rounds of workgroups, ragged in
    both directions, random ops, grids and precisions, the cost model's own choices (which split
    the tiles after the last full round where that pays): small-integer data, bit for bit."""
    r = np.random.default_rng(9100 + seed)
    dt, out = [(dm.F32, dm.F32), (dm.F64, dm.F64), (dm.F16, dm.F32), (dm.F16, dm.F16)][seed % 4]
    rows, cols = (128, 64) if dt != dm.F16 else (256, 128)
    slots = 512 if dt != dm.F16 else 256
    tn = int(r.integers(24, 40))                             # column tiles
    tm = (slots * int(r.integers(1, 3)) + int(r.integers(8, 120))) // tn + 1
    M = tm * rows - int(r.integers(1, rows // 2)) // 8 * 8
    N = tn * cols - int(r.integers(1, cols // 2)) // 8 * 8
    K = 64 * int(r.integers(2, 9))
    ta, tb = int(r.integers(0, 2)), int(r.integers(0, 2))
    opA = r.integers(-2, 3, (M, K)).astype(NP[dt])
    opB = r.integers(-2, 3, (K, N)).astype(NP[dt])
    C0 = r.integers(-2, 3, (M, N)).astype(NP[out])
    A, B = stored(opA, ta), stored(opB, tb)
    ctx.set_kernel_policy(0)
    dA, dB, dC = ctx.from_host(A), ctx.from_host(B), ctx.from_host(C0)
    info = dm.gemm_plan_info(ctx, ta, tb, dA, dB, dC)
    assert info["kernel"] > 0, info
    dm.gemm(ctx, ta, tb, 1.0, dA, dB, 1.0, dC)
    sel = sorted(set(int(x) for x in r.integers(0, M, 48)) | {0, M - 1})
    ref = oracle.gemm(bool(ta), bool(tb), 1.0, A, B, 1.0, C0, rows=sel)
    got = dC.get()[sel].astype(np.float64)
    for m in (dA, dB, dC):
        m.destroy()
    what = (seed, dt, out, (M, N, K), (ta, tb), info)
    if out == dm.F16 and np.abs(ref).max() > 2048:
        assert rel_fro(got, ref) <= TOL[dt], what
    else:
        assert np.array_equal(got, ref), what
