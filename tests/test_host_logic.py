"""CPU-only tests of the library's host side: the C ABI exports what the header declares, the
pool, the block split rule, argument checks, and the tile scheduler (no kernel is launched)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1611_07819_amd as dm
from paper_1611_07819_amd import dmath as binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_SLAB = 0x7F0000000100      # never dereferenced by host logic


@pytest.fixture()
def ctx():
    c = dm.Context(FAKE_SLAB, 1 << 30)
    yield c
    c.close()


def test_library_exports_every_declared_symbol():
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if h.endswith(".h"):
            names |= set(re.findall(r"\b(dmath_[a-z_0-9]+)\s*\(", open(os.path.join(ROOT, "include", h)).read()))
    product = open(os.path.join(ROOT, "include", "dmath.h")).read()
    assert "probe" not in product          # measurement aids live in dmath_measure.h
    assert {"dmath_init", "dmath_matrix_create", "dmath_gemm", "dmath_conv_fwd",
            "dmath_conv_bwd_filter", "dmath_conv_bwd_data"} <= names
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_1611_07819_amd", "libdmath.so"))
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    assert binding.status_string(0) == "DMATH_OK"
    assert binding.status_string(6) == "DMATH_ERR_OOM"
    assert binding.status_string(99) == "DMATH_ERR_UNKNOWN"


def test_pool_accounting_alignment_and_reuse(ctx):
    s0 = ctx.pool_stats()
    assert s0["in_use"] == 0 and s0["capacity"] == (1 << 30) - 256   # 256-byte tail guard
    odd = dm.Context(FAKE_SLAB + 8, 1 << 20)         # unaligned slab: the head is given up
    assert odd.pool_stats()["capacity"] == (1 << 20) - 512
    assert odd.matrix(4, 4, (1, 1), dm.F32).block(0, 0)["ptr"] == FAKE_SLAB + 256
    odd.close()
    a = ctx.matrix(100, 100, (2, 2), dm.F32)        # 4 blocks of 50*50*4 = 10000 -> 10240 each
    assert ctx.pool_stats()["in_use"] == 4 * 10240
    ptrs = [a.block(i, j)["ptr"] for i in range(2) for j in range(2)]
    assert all(p % 256 == 0 for p in ptrs) and len(set(ptrs)) == 4
    b = ctx.matrix(10, 10, (1, 1), dm.F64)
    a.destroy()
    assert ctx.pool_stats()["in_use"] == 1024
    c = ctx.matrix(100, 100, (2, 2), dm.F32)        # first fit: reuses the hole left by a
    assert sorted(c.block(i, j)["ptr"] for i in range(2) for j in range(2)) == sorted(ptrs)
    assert ctx.pool_stats()["high_water"] == 4 * 10240 + 1024
    b.destroy()
    c.destroy()
    assert ctx.pool_stats()["in_use"] == 0
    big = ctx.matrix(16384, 16380, (1, 1), dm.F32)  # coalescing gave back one contiguous range
    big.destroy()


def test_pool_exhaustion_is_an_error_and_leaks_nothing():
    c = dm.Context(FAKE_SLAB, 1 << 20)
    with pytest.raises(dm.DmathError) as e:
        c.matrix(1024, 1024, (2, 2), dm.F32)         # 4 MiB > 1 MiB
    assert e.value.code == 6
    assert c.pool_stats()["in_use"] == 0
    c.close()


def test_split_rule_and_block_shapes(ctx):
    m = ctx.matrix(10, 7, (3, 2), dm.F16)
    assert [m.block(i, 0)["rows"] for i in range(3)] == [4, 4, 2]
    assert [m.block(0, j)["cols"] for j in range(2)] == [4, 3]
    assert m.block(2, 1)["ld"] == 3
    assert m.info() == {"rows": 10, "cols": 7, "grid": (3, 2), "dtype": dm.F16}
    with pytest.raises(dm.DmathError) as e:
        ctx.matrix(9, 4, (4, 1), dm.F32)             # ceil(9/4) = 3 leaves the 4th part empty
    assert e.value.code == 3
    for bad in [(0, 4, (1, 1)), (4, 4, (0, 1)), (4, -1, (1, 1))]:
        with pytest.raises(dm.DmathError) as e:
            ctx.matrix(bad[0], bad[1], bad[2], dm.F32)
        assert e.value.code == 1
    with pytest.raises(dm.DmathError):
        ctx.matrix(4, 4, (1, 1), 7)


def test_gemm_argument_checks(ctx):
    A = ctx.matrix(8, 6, (2, 2), dm.F32)
    B = ctx.matrix(6, 4, (1, 2), dm.F32)
    C = ctx.matrix(8, 4, (2, 1), dm.F32)
    assert dm.gemm_plan_info(ctx, 0, 0, A, B, C)["k"] == 6

    def code(fn):
        with pytest.raises(dm.DmathError) as e:
            fn()
        return e.value.code
    assert code(lambda: dm.gemm_plan_info(ctx, 1, 0, A, B, C)) == 2          # shape
    assert code(lambda: dm.gemm_plan_info(ctx, 0, 0, A, B, A)) == 5          # alias
    assert code(lambda: dm.gemm_plan_info(ctx, 0, 2, A, B, C)) == 1          # bad op
    Ch = ctx.matrix(8, 4, (1, 1), dm.F16)
    assert code(lambda: dm.gemm_plan_info(ctx, 0, 0, A, B, Ch)) == 4         # f32 in, f16 out
    Ah = ctx.matrix(8, 6, (1, 1), dm.F16)
    Bh = ctx.matrix(6, 4, (1, 1), dm.F16)
    assert dm.gemm_plan_info(ctx, 0, 0, Ah, Bh, C)["m"] == 8                 # f16 in, f32 out
    assert dm.gemm_plan_info(ctx, 0, 0, Ah, Bh, Ch)["m"] == 8                # f16 in, f16 out
    assert code(lambda: dm.gemm_plan_info(ctx, 0, 0, Ah, B, C)) == 4         # mixed inputs
    other = dm.Context(FAKE_SLAB + (1 << 31), 1 << 20)
    Co = other.matrix(8, 4, (1, 1), dm.F32)
    assert code(lambda: dm.gemm_plan_info(ctx, 0, 0, A, B, Co)) == 1         # foreign handle
    # the same checks guard the launching call; errors come back before any device work
    assert code(lambda: dm.gemm(ctx, 1, 0, 1.0, A, B, 0.0, C)) == 2
    assert code(lambda: dm.gemm(ctx, 0, 0, 1.0, A, B, 0.0, A)) == 5
    other.close()


def test_scheduler_refines_against_every_grid(ctx):
    # section 3.2: the grids of A, B and C need not agree.
    A = ctx.matrix(10, 7, (3, 2), dm.F32)   # rows cut at 4, 8; cols at 4
    B = ctx.matrix(7, 5, (2, 2), dm.F32)    # rows cut at 4;    cols at 3
    C = ctx.matrix(10, 5, (2, 1), dm.F32)   # rows cut at 5
    p = dm.gemm_plan_info(ctx, 0, 0, A, B, C)
    assert (p["m_segments"], p["n_segments"], p["k_segments"]) == (4, 2, 2)
    assert p["tiles"] == 8 and p["cached"] == 0
    assert dm.gemm_plan_info(ctx, 0, 0, A, B, C)["cached"] == 1
    B3 = ctx.matrix(7, 5, (3, 1), dm.F32)   # rows cut at 3, 6 -> k cuts {3,4,6}
    p = dm.gemm_plan_info(ctx, 0, 0, A, B3, C)
    assert (p["n_segments"], p["k_segments"]) == (1, 4)
    # transposed operands: op(A) = A^T swaps the roles of the two grids of A
    At = ctx.matrix(7, 10, (2, 3), dm.F32)
    p = dm.gemm_plan_info(ctx, 1, 0, At, B, C)
    assert (p["m_segments"], p["k_segments"]) == (4, 2)
    # destroying an operand drops the cached plan
    B.destroy()
    B = ctx.matrix(7, 5, (2, 2), dm.F32)
    assert dm.gemm_plan_info(ctx, 0, 0, A, B, C)["cached"] == 0


def test_scheduler_on_the_benchmark_configs(ctx):
    big = dm.Context(FAKE_SLAB, 8 << 30)
    X = big.matrix(1024, 9216, (4, 4), dm.F32)
    W = big.matrix(9216, 4096, (4, 4), dm.F32)
    Y = big.matrix(1024, 4096, (4, 4), dm.F32)
    dW = big.matrix(9216, 4096, (4, 4), dm.F32)
    dX = big.matrix(1024, 9216, (4, 4), dm.F32)
    for (ta, tb, a, b, c, mnk) in [(0, 0, X, W, Y, (1024, 4096, 9216)),
                                   (1, 0, X, Y, dW, (9216, 4096, 1024)),
                                   (0, 1, Y, W, dX, (1024, 9216, 4096))]:
        p = dm.gemm_plan_info(big, ta, tb, a, b, c)
        assert (p["m"], p["n"], p["k"]) == mnk
        assert (p["m_segments"], p["n_segments"], p["k_segments"]) == (4, 4, 4)
        assert p["tiles"] * p["tile_m"] * p["tile_n"] == mnk[0] * mnk[1]
    big.close()


def test_conv_argument_checks(ctx):
    d = dm.ConvDesc(n=4, c=3, h=8, w=8, k=5, r=3, s=3, pad_h=1, pad_w=1)
    X = ctx.matrix(4, 3 * 64, (2, 1), dm.F16)
    F = ctx.matrix(5, 27, (1, 1), dm.F16)
    Y = ctx.matrix(4, 5 * 64, (1, 1), dm.F32)

    def code(fn):
        with pytest.raises(dm.DmathError) as e:
            fn()
        return e.value.code
    Ybad = ctx.matrix(4, 5 * 63, (1, 1), dm.F32)
    assert code(lambda: dm.conv_fwd(ctx, d, 1.0, X, F, 0.0, Ybad)) == 2
    Xcols = ctx.matrix(4, 3 * 64, (1, 2), dm.F16)
    assert code(lambda: dm.conv_fwd(ctx, d, 1.0, Xcols, F, 0.0, Y)) == 3
    Y64 = ctx.matrix(4, 5 * 64, (1, 1), dm.F64)
    assert code(lambda: dm.conv_fwd(ctx, d, 1.0, X, F, 0.0, Y64)) == 4
    assert code(lambda: dm.conv_fwd(ctx, dm.ConvDesc(4, 3, 8, 8, 5, 3, 3, 1, 1, 0, 1), 1.0, X, F, 0.0, Y)) == 1
    assert code(lambda: dm.conv_fwd(ctx, dm.ConvDesc(4, 3, 2, 2, 5, 5, 5), 1.0, X, F, 0.0, Y)) == 2
    assert code(lambda: dm.conv_bwd_filter(ctx, d, 1.0, X, X, 0.0, F)) in (2, 5)


def test_pipeline_calls_without_a_capturable_stream(ctx):
    # the fixture's context uses the default stream, which cannot be captured
    with pytest.raises(dm.DmathError) as e:
        ctx.pipeline_begin()
    assert e.value.code == 7
    with pytest.raises(dm.DmathError) as e:
        ctx.pipeline_end()
    assert e.value.code == 1
    with pytest.raises(dm.DmathError) as e:
        ctx.pipeline_replay(3)
    assert e.value.code == 1


def test_size_limits(ctx):
    with pytest.raises(dm.DmathError) as e:
        ctx.matrix(1 << 31, 1, (1, 1), dm.F16)
    assert e.value.code == 7


def test_scheduler_pads_k_tails_and_counts_their_scratch(ctx):
    """K = 1000 is not a multiple of the fp32 kernels' k-step of 32: the plan keeps a specialised
    kernel, cuts the last 8 of K off as a segment of its own and reports the zero-padded scratch
    panels it reads them from ([M][32] for the k-major A, [32][N rounded up to 64] for B)."""
    A = ctx.matrix(256, 1000, (1, 1), dm.F32)
    B = ctx.matrix(1000, 384, (1, 1), dm.F32)
    C = ctx.matrix(256, 384, (1, 1), dm.F32)
    p = dm.gemm_plan_info(ctx, 0, 0, A, B, C)
    assert p["kernel"] != 0 and p["tile_k"] == 32
    # the segments are [0, 992) and [992, 1000), the first possibly cut further by split-K
    assert p["k_segments"] == p["split_k"] + 1
    partials = p["split_k"] * 256 * 384 * 4 if p["split_k"] > 1 else 0
    assert p["workspace_bytes"] == partials + (256 + 384) * 32 * 4
    # rows of 1001 floats are not 16-byte aligned: the guarded generic kernel, no scratch
    A1 = ctx.matrix(256, 1001, (1, 1), dm.F32)
    B1 = ctx.matrix(1001, 384, (1, 1), dm.F32)
    p = dm.gemm_plan_info(ctx, 0, 0, A1, B1, C)
    assert p["kernel"] == 0 and p["k_segments"] == 1
    # a K of fewer than four k-steps is left to the generic kernel as well
    A2 = ctx.matrix(256, 100, (1, 1), dm.F32)
    B2 = ctx.matrix(100, 384, (1, 1), dm.F32)
    assert dm.gemm_plan_info(ctx, 0, 0, A2, B2, C)["kernel"] == 0


def test_scheduler_choices_for_small_problems(ctx):
    """Where one round of tiles does not fill the 256 CUs the time model splits K (down to 128 of
    K per part), and a batch of at most 64 rows gets 64-row tiles."""
    A = ctx.matrix(512, 512, (1, 1), dm.F32)
    B = ctx.matrix(512, 512, (1, 1), dm.F32)
    C = ctx.matrix(512, 512, (1, 1), dm.F32)
    p = dm.gemm_plan_info(ctx, 0, 0, A, B, C)
    assert p["kernel"] != 0 and 2 <= p["split_k"] <= 4 and p["tiles"] * p["split_k"] <= 512
    big = dm.Context(FAKE_SLAB, 8 << 30)
    for dt in (dm.F16, dm.F32, dm.F64):
        X = big.matrix(64, 4096, (1, 1), dt)
        W = big.matrix(4096, 4096, (1, 1), dt)
        Y = big.matrix(64, 4096, (1, 1), dm.F32 if dt == dm.F16 else dt)
        p = dm.gemm_plan_info(big, 0, 0, X, W, Y)
        assert p["kernel"] != 0 and p["tile_m"] == 64 and p["split_k"] > 1
    big.close()


def test_scheduler_splits_only_the_tiles_after_the_last_full_round(ctx):
    """Tile counts that do not fill whole rounds of workgroups (256 CUs x workgroups per CU): the
    tiles of the full rounds run unsplit, the rest take partial sums in a compact workspace."""
    big = dm.Context(FAKE_SLAB, 8 << 30)
    # fp32, 128x64 tiles, two workgroups per CU: 640 tiles = one round of 512 + 128
    A, B, C = big.matrix(1280, 4096, (1, 1), dm.F32), big.matrix(4096, 4096, (1, 1), dm.F32), big.matrix(1280, 4096, (1, 1), dm.F32)
    p = dm.gemm_plan_info(big, 0, 0, A, B, C)
    assert (p["tile_m"], p["tile_n"], p["tiles"]) == (128, 64, 640)
    assert p["split_tiles"] == 128 and p["split_k"] >= 2
    assert p["workspace_bytes"] == p["split_k"] * 128 * 128 * 64 * 4      # only those tiles, not the whole C
    # exactly two rounds: nothing is split
    A2, C2 = big.matrix(2048, 4096, (1, 1), dm.F32), big.matrix(2048, 4096, (1, 1), dm.F32)
    p = dm.gemm_plan_info(big, 0, 0, A2, B, C2)
    assert p["tiles"] == 1024 and p["split_k"] == 1 and p["split_tiles"] == 0 and p["workspace_bytes"] == 0
    # fp16, 256x128 tiles, one workgroup per CU: 544 tiles = two rounds + 32
    Ah, Bh = big.matrix(4352, 4096, (1, 1), dm.F16), big.matrix(4096, 4096, (1, 1), dm.F16)
    Ch = big.matrix(4352, 4096, (1, 1), dm.F32)
    p = dm.gemm_plan_info(big, 0, 0, Ah, Bh, Ch)
    assert (p["tile_m"], p["tile_n"], p["tiles"], p["split_tiles"]) == (256, 128, 544, 32) and p["split_k"] >= 2
    # the data gradient of the benchmark's fp32 layer: 1152 tiles = 2.25 rounds
    Y, W, dX = big.matrix(1024, 4096, (4, 4), dm.F32), big.matrix(9216, 4096, (4, 4), dm.F32), big.matrix(1024, 9216, (4, 4), dm.F32)
    p = dm.gemm_plan_info(big, 0, 1, Y, W, dX)
    assert (p["tile_m"], p["tile_n"], p["tiles"], p["split_tiles"]) == (128, 64, 1152, 128)
    big.close()


def test_exceptions_do_not_cross_the_c_boundary():
    """A grid whose bookkeeping cannot be allocated must come back as DMATH_ERR_OOM, not as a C++
    exception that ends the process.  Run in a child whose address space is limited, so that the
    allocation fails quickly and this process is not disturbed."""
    import subprocess
    import sys
    code = r"""
import resource, sys
sys.path.insert(0, %r)
import paper_1611_07819_amd as dm
from paper_1611_07819_amd import dmath as binding
ctx = dm.Context(0x7F0000000100, 1 << 46)          # fake slab: host logic never dereferences it
resource.setrlimit(resource.RLIMIT_AS, (3 << 30, 3 << 30))
n = (1 << 31) - 1
for shape, grid in (((n, n), (n, n)),              # 2^62 block pointers: no container can hold them
                    ((n, 1), (n, 1))):             # 16 GiB of block pointers: bad_alloc under the limit
    try:
        ctx.matrix(shape[0], shape[1], grid, dm.F16)
    except binding.DmathError as e:
        assert e.code == 6, e.code                 # DMATH_ERR_OOM
    else:
        raise SystemExit("huge grid was accepted")
assert ctx.pool_stats()["in_use"] == 0             # nothing of the failed handles is left behind
m = ctx.matrix(64, 64, (2, 2), dm.F32)             # and the context still works
assert ctx.pool_stats()["in_use"] == 4 * 32 * 32 * 4
ctx.close()
print("barrier ok")
""" % ROOT
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "barrier ok" in r.stdout, (r.returncode, r.stdout[-400:], r.stderr[-800:])
