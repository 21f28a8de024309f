"""GPU parity of the implicit-GEMM convolutions against the CPU oracle, through the C ABI."""
import os

import numpy as np
import pytest

import paper_1611_07819_amd as dm
from paper_1611_07819_amd import synth
from gpu_util import TOL, make_context, rel_fro

pytestmark = pytest.mark.gpu
NP = {dm.F64: np.float64, dm.F32: np.float32, dm.F16: np.float16}

GEOMS = [
    dict(n=3, c=5, h=9, w=7, k=6, r=3, s=3, pad_h=1, pad_w=1),
    dict(n=2, c=4, h=12, w=10, k=70, r=3, s=2, pad_h=0, pad_w=1, stride_h=2, stride_w=1),
    dict(n=4, c=16, h=6, w=6, k=8, r=1, s=1),
    dict(n=2, c=3, h=11, w=9, k=5, r=5, s=3, pad_h=2, pad_w=0, stride_h=2, stride_w=3),
    dict(n=5, c=24, h=14, w=14, k=40, r=3, s=3, pad_h=1, pad_w=1),
]


@pytest.fixture(scope="module")
def ctx():
    c = make_context(3.0)
    yield c
    c.close()


def tensors(g, dt, seed, ints=False):
    d = dm.ConvDesc(**g)
    oh = (d.h + 2 * d.pad_h - d.r) // d.stride_h + 1
    ow = (d.w + 2 * d.pad_w - d.s) // d.stride_w + 1
    r = np.random.default_rng(seed)
    shapes = {"X": (d.n, d.c * d.h * d.w), "F": (d.k, d.c * d.r * d.s), "Y": (d.n, d.k * oh * ow)}
    if ints:
        t = {k: r.integers(-2, 3, s).astype(NP[dt]) for k, s in shapes.items()}
    else:
        t = {"X": r.uniform(0, 1, shapes["X"]).astype(NP[dt]),
             "F": r.normal(0, 0.2, shapes["F"]).astype(NP[dt]),
             "Y": r.normal(0, 0.1, shapes["Y"]).astype(NP[dt])}
    return d, t


def three_modes(ctx, oracle, g, dt, out_dt, alpha, beta, grids, ints=False, policy=0):
    d, t = tensors(g, dt, 300, ints)
    od = oracle.ConvDesc(**g)
    ctx.set_kernel_policy(policy)
    res = {}
    for mode in ("fwd", "bwd_filter", "bwd_data"):
        out_name = {"fwd": "Y", "bwd_filter": "F", "bwd_data": "X"}[mode]
        host = {k: (v.astype(NP[out_dt]) if k == out_name else v) for k, v in t.items()}
        dev = {k: ctx.from_host(v, grids[k]) for k, v in host.items()}
        blk = {k: oracle.BlockMatrix(v, grids[k]) for k, v in host.items()}
        if mode == "fwd":
            dm.conv_fwd(ctx, d, alpha, dev["X"], dev["F"], beta, dev["Y"])
            ref = oracle.conv_fwd(od, alpha, blk["X"], blk["F"], beta, blk["Y"])
        elif mode == "bwd_filter":
            dm.conv_bwd_filter(ctx, d, alpha, dev["X"], dev["Y"], beta, dev["F"])
            ref = oracle.conv_bwd_filter(od, alpha, blk["X"], blk["Y"], beta, blk["F"])
        else:
            dm.conv_bwd_data(ctx, d, alpha, dev["Y"], dev["F"], beta, dev["X"])
            ref = oracle.conv_bwd_data(od, alpha, blk["Y"], blk["F"], beta, blk["X"])
        res[mode] = (dev[out_name].get(), ref)
        for m in dev.values():
            m.destroy()
    return res


@pytest.mark.parametrize("policy", [0, 1])
@pytest.mark.parametrize("g", GEOMS)
@pytest.mark.parametrize("dt,out", [(dm.F64, dm.F64), (dm.F32, dm.F32), (dm.F16, dm.F32), (dm.F16, dm.F16)])
def test_geometries_all_modes(ctx, oracle, g, dt, out, policy):
    grids = {"X": (1, 1), "F": (1, 1), "Y": (1, 1)}
    for mode, (got, ref) in three_modes(ctx, oracle, g, dt, out, 1.5, -0.5, grids, policy=policy).items():
        assert rel_fro(got, ref) <= TOL[dt], mode


@pytest.mark.parametrize("g", GEOMS[:2] + GEOMS[4:])
@pytest.mark.parametrize("dt,out", [(dm.F64, dm.F64), (dm.F32, dm.F32), (dm.F16, dm.F32), (dm.F16, dm.F16)])
def test_integer_inputs_bitwise_with_row_blocked_tensors(ctx, oracle, g, dt, out):
    # |values| <= 2, at most c*r*s*4 <= 2048 per output in these geometries for the forward
    # pass; the weight gradient sums n*oh*ow*4 terms, also below 2048 here.
    grids = {"X": (g["n"], 1), "F": (2, 1), "Y": (2, 1)}
    for mode, (got, ref) in three_modes(ctx, oracle, g, dt, out, 1.0, 1.0, grids, ints=True).items():
        if out == dm.F16 and np.abs(ref).max() > 2048:
            assert rel_fro(got, ref) <= TOL[dt], mode
        else:
            assert np.array_equal(got.astype(np.float64), ref), mode


def test_delta_filters_fix_the_convention(ctx):
    g = dict(n=2, c=4, h=8, w=9, k=4, r=3, s=3, pad_h=1, pad_w=1)
    d = dm.ConvDesc(**g)
    X = np.random.default_rng(301).uniform(0, 1, (2, 4 * 72)).astype(np.float16)
    F = np.zeros((4, 4, 3, 3), np.float16)
    for k in range(4):
        F[k, k, 0, 2] = 1
    dX, dF = ctx.from_host(X), ctx.from_host(F.reshape(4, 36))
    dY = ctx.matrix(2, 4 * 72, (1, 1), dm.F16)
    dm.conv_fwd(ctx, d, 1.0, dX, dF, 0.0, dY)
    got = dY.get().reshape(2, 4, 8, 9)
    x = X.reshape(2, 4, 8, 9)
    want = np.zeros_like(x)
    want[:, :, 1:, :-1] = x[:, :, :-1, 1:]      # Y[oh,ow] = X[oh-1, ow+1]
    assert np.array_equal(got, want)
    for m in (dX, dF, dY):
        m.destroy()


@pytest.mark.parametrize("out", ["f32", "f16"])
def test_config5_reduced_whole_result(ctx, oracle, out):
    w = synth.config5(out, batch=4, channels=64, hw=28)
    _config5(ctx, oracle, w, None, None)


def test_config5_full_size_whole_result(ctx, oracle):
    # forward, weight gradient and data gradient at batch 64, every output element; both output
    # types against one oracle run (same inputs, beta = 0)
    refs = {}
    for out in ("f32", "f16"):
        _config5(ctx, oracle, synth.config5(out), None, None, refs=refs)
    assert sorted(refs) == ["bwd_data", "bwd_filter", "fwd"]


@pytest.mark.parametrize("dt", [dm.F32, dm.F64])
def test_config5_geometry_full_size_sampled_in_the_wider_precisions(ctx, oracle, dt):
    """The configuration-5 layer with its tensors widened to fp32 / fp64 (the launch
    configuration that the benchmark's cfg5_as_f32 lines time), sampled images and filters."""
    w = synth.config5("f32")
    mats = {k: v.astype(NP[dt]) for k, v in w.mats.items()}
    _config5(ctx, oracle, w, [0, 37, 63], [1, 200], mats=mats, dt=dt)


ELEM_C = 50    # per-element bound beside the norm: |got - ref| <= ELEM_C * tol * max|ref|


def _config5(ctx, oracle, w, images, filters, mats=None, dt=dm.F16, refs=None):
    """Forward, weight gradient and data gradient of the layer against the oracle (all outputs,
    or the sampled images / filters).  `refs` keeps the oracle's results by mode for a second
    pass over the same inputs with another output type."""
    mats = w.mats if mats is None else mats
    d = dm.ConvDesc(**w.conv)
    od = oracle.ConvDesc(**w.conv)
    dev = {k: ctx.from_host(v) for k, v in mats.items()}

    def check(mode, got, sel, make_ref):
        if refs is not None and mode in refs:
            ref = refs[mode]
        else:
            ref = make_ref()
            if refs is not None:
                refs[mode] = ref
        got = np.asarray(got if sel is None else got[sel], np.float64)
        assert got.shape == ref.shape, mode
        err = rel_fro(got, ref)
        assert err <= TOL[dt], (w.name, mode, err)
        worst = np.abs(got - ref).max()
        assert worst <= ELEM_C * TOL[dt] * np.abs(ref).max(), (w.name, mode, worst)

    dm.conv_fwd(ctx, d, 1.0, dev["X"], dev["F"], 0.0, dev["Y"])
    check("fwd", dev["Y"].get(), images,
          lambda: oracle.conv_fwd(od, 1.0, mats["X"], mats["F"], images=images))
    dm.conv_bwd_filter(ctx, d, 1.0, dev["X"], dev["dY"], 0.0, dev["dF"])
    check("bwd_filter", dev["dF"].get(), filters,
          lambda: oracle.conv_bwd_filter(od, 1.0, mats["X"], mats["dY"], filters=filters))
    dX = ctx.matrix(dev["X"].rows, dev["X"].cols, (1, 1), dev["Y"].dtype)
    dm.conv_bwd_data(ctx, d, 1.0, dev["dY"], dev["F"], 0.0, dX)
    check("bwd_data", dX.get(), images,
          lambda: oracle.conv_bwd_data(od, 1.0, mats["dY"], mats["F"], images=images))
    dX.destroy()
    for m in dev.values():
        m.destroy()


def runs_as_block_gemm(g, dt):
    """1x1, stride 1, no padding, 16-byte aligned planes and filter rows, planes that are whole
    64-element tiles or nearly: all three modes are block GEMMs on the tensors as they lie, with
    one column block (weight gradient: one k-segment) per image and no re-layout copies."""
    es = {dm.F16: 2, dm.F32: 4, dm.F64: 8}[dt]
    sp = g["h"] * g["w"]
    return (g["r"] == 1 and g["s"] == 1 and g.get("stride_h", 1) == 1 and g.get("stride_w", 1) == 1 and
            g.get("pad_h", 0) == 0 and g.get("pad_w", 0) == 0 and (sp * es) % 16 == 0 and
            (g["c"] * es) % 16 == 0 and (sp + 63) // 64 * 64 * 100 <= sp * 135)


def out_plane(g):
    oh = (g["h"] + 2 * g.get("pad_h", 0) - g["r"]) // g.get("stride_h", 1) + 1
    ow = (g["w"] + 2 * g.get("pad_w", 0) - g["s"]) // g.get("stride_w", 1) + 1
    return oh, ow


def dy_read_in_place(g, dt, y_grid=(1, 1)):
    """The weight gradient reads dY where it lies (no channels-last copy of it): dY is one block,
    a plane is a whole number of 16-byte chunks, all pixels a whole number of k-tiles, the filter
    count a multiple of 64, and a plane holds at least one k-tile."""
    es, pt = {dm.F16: (2, 64), dm.F32: (4, 32), dm.F64: (8, 16)}[dt]
    oh, ow = out_plane(g)
    sp = oh * ow
    return (y_grid[0] == 1 and "DMATH_CONV_DY_COPY" not in os.environ and (sp * es) % 16 == 0 and
            (g["n"] * sp) % pt == 0 and g["k"] % 64 == 0 and pt <= sp)


def copies_written(g, dt, y_grid=(1, 1)):
    """Re-layout copies the three modes write on the specialised kernels: two each, except that
    the weight gradient may read dY in place."""
    return 5 if dy_read_in_place(g, dt, y_grid) else 6


FAST_GEOMS = [
    # geometries that run on the specialised kernels
    dict(n=4, c=128, h=16, w=16, k=256, r=3, s=3, pad_h=1, pad_w=1),
    dict(n=8, c=128, h=16, w=8, k=256, r=1, s=1),
    dict(n=2, c=256, h=16, w=16, k=256, r=5, s=3, pad_h=2, pad_w=1),
    dict(n=16, c=128, h=12, w=12, k=256, r=3, s=3, pad_h=1, pad_w=1),
    dict(n=4, c=128, h=16, w=16, k=512, r=3, s=3, pad_h=1, pad_w=1),      # two row tiles of filters
    dict(n=4, c=256, h=16, w=16, k=128, r=3, s=3, pad_h=1, pad_w=1),      # 128 filters: 128x128 tiles
    dict(n=4, c=64, h=16, w=16, k=64, r=3, s=3, pad_h=1, pad_w=1),        # 64 channels and filters: narrow tiles
    dict(n=4, c=192, h=16, w=16, k=128, r=5, s=5, pad_h=2, pad_w=2),      # channels a multiple of 64 only
    dict(n=8, c=64, h=8, w=8, k=256, r=1, s=1),
    dict(n=2, c=64, h=40, w=40, k=64, r=3, s=3, pad_h=1, pad_w=1),        # planes of more than 1024 pixels
    dict(n=16, c=64, h=34, w=34, k=64, r=1, s=1),                         # ... whose size is 4 mod 8
    # strides: rows and columns left over at the end (22+2-3 and 16+2-3 are odd), 1x1 filter, mixed
    dict(n=8, c=64, h=22, w=16, k=64, r=3, s=3, pad_h=1, pad_w=1, stride_h=2, stride_w=2),
    dict(n=4, c=128, h=16, w=16, k=256, r=1, s=1, stride_h=2, stride_w=2),
    dict(n=4, c=64, h=16, w=32, k=128, r=3, s=5, pad_h=1, pad_w=2, stride_h=1, stride_w=2),
    dict(n=4, c=64, h=24, w=24, k=64, r=5, s=5, pad_h=2, pad_w=2, stride_h=3, stride_w=3),
    # channel and filter counts rounded up to 64 inside the copies, planes of an odd number of
    # pixels, n*oh*ow not a multiple of 64 (the weight gradient's last pixel tile reads zeros)
    dict(n=4, c=96, h=13, w=13, k=96, r=3, s=3, pad_h=1, pad_w=1),
    dict(n=3, c=128, h=7, w=7, k=384, r=3, s=3, pad_h=1, pad_w=1),        # planes of fewer than 64 pixels
    dict(n=2, c=64, h=27, w=27, k=128, r=5, s=5, pad_h=2, pad_w=2),
    dict(n=5, c=120, h=9, w=11, k=120, r=3, s=2, pad_h=1, pad_w=0, stride_h=2, stride_w=1),
    dict(n=16, c=64, h=13, w=13, k=64, r=3, s=3, pad_h=1, pad_w=1),       # 43 pixel tiles in 5 uneven parts
    dict(n=8, c=64, h=6, w=4, k=64, r=3, s=3, pad_h=1, pad_w=1),          # planes of 24 pixels: fp64 reads dY in place, a plane ends inside two k-tiles of three
    dict(n=2, c=64, h=16, w=16, k=64, r=12, s=12),                        # 144 taps: fp64 filter permute / reduction without LDS staging
    # 1x1, stride 1, no padding: block GEMMs with one column block per image (planes of 576 pixels:
    # ragged last column tile, and a k-tail per image in the weight gradient; 56 channels: a k-tail
    # in the forward pass)
    dict(n=3, c=128, h=24, w=24, k=192, r=1, s=1),
    dict(n=2, c=56, h=32, w=16, k=120, r=1, s=1),
]


@pytest.mark.parametrize("g", FAST_GEOMS)
@pytest.mark.parametrize("dt,out", [(dm.F16, dm.F32), (dm.F16, dm.F16), (dm.F32, dm.F32), (dm.F64, dm.F64)])
def test_specialised_conv_whole_result(ctx, oracle, g, dt, out):
    """All three modes on the specialised path (fp16, fp32 and fp64 pipelines) against the oracle:
    within the precision's bar on random data (alpha/beta exercised) and bit for bit on
    small-integer data with a row-blocked layout of every tensor."""
    grids = {"X": (1, 1), "F": (1, 1), "Y": (1, 1)}
    before = ctx.relayout_stats()["written"]
    res = three_modes(ctx, oracle, g, dt, out, 1.5, -0.5, grids, policy=0)
    # every mode went through the specialised kernels: each re-laid-out its two operands
    assert ctx.relayout_stats()["written"] - before == (0 if runs_as_block_gemm(g, dt) else copies_written(g, dt))
    for mode in ("fwd", "bwd_filter", "bwd_data"):
        got, ref = res[mode]
        assert rel_fro(got, ref) <= TOL[dt], mode
    d, t = tensors(g, dt, 300, ints=True)
    t = {k: np.sign(v).astype(NP[dt]) if k != "F" else v for k, v in t.items()}   # keep sums small
    od = oracle.ConvDesc(**g)
    ctx.set_kernel_policy(0)
    blocked, whole = {"X": (g["n"], 1), "F": (2, 1), "Y": (2, 1)}, {"X": (1, 1), "F": (1, 1), "Y": (1, 1)}
    # the weight gradient a second time on one-block tensors, where it may read dY in place
    for mode, grids in (("fwd", blocked), ("bwd_filter", blocked), ("bwd_data", blocked), ("bwd_filter", whole)):
        out_name = {"fwd": "Y", "bwd_filter": "F", "bwd_data": "X"}[mode]
        host = {k: (v.astype(NP[out]) if k == out_name else v) for k, v in t.items()}
        dev = {k: ctx.from_host(v, grids[k]) for k, v in host.items()}
        if mode == "fwd":
            dm.conv_fwd(ctx, d, 1.0, dev["X"], dev["F"], 1.0, dev["Y"])
            ref = oracle.conv_fwd(od, 1.0, host["X"], host["F"], 1.0, host["Y"])
        elif mode == "bwd_filter":
            dm.conv_bwd_filter(ctx, d, 1.0, dev["X"], dev["Y"], 1.0, dev["F"])
            ref = oracle.conv_bwd_filter(od, 1.0, host["X"], host["Y"], 1.0, host["F"])
        else:
            dm.conv_bwd_data(ctx, d, 1.0, dev["Y"], dev["F"], 1.0, dev["X"])
            ref = oracle.conv_bwd_data(od, 1.0, host["Y"], host["F"], 1.0, host["X"])
        got = dev[out_name].get().astype(np.float64)
        if out == dm.F16 and np.abs(ref).max() > 2048:
            assert rel_fro(got, ref) <= TOL[dm.F16], mode
        else:
            assert np.array_equal(got, ref), mode
        for m in dev.values():
            m.destroy()


SPLIT_GEOMS = [
    dict(n=3, c=128, h=14, w=14, k=256, r=3, s=3, pad_h=1, pad_w=1),                  # ragged last row tile
    dict(n=5, c=120, h=9, w=11, k=120, r=3, s=2, pad_h=1, pad_w=0, stride_h=2, stride_w=1),  # padded channels, odd planes
    dict(n=2, c=192, h=16, w=16, k=64, r=5, s=5, pad_h=2, pad_w=2),
]


@pytest.mark.parametrize("split", ["1", "3", "8"])
@pytest.mark.parametrize("g", SPLIT_GEOMS)
@pytest.mark.parametrize("dt,out", [(dm.F16, dm.F32), (dm.F16, dm.F16), (dm.F32, dm.F32), (dm.F64, dm.F64)])
def test_forward_and_data_gradient_with_a_split_k_loop(oracle, monkeypatch, g, dt, out, split):
    """The forward pass and the data gradient with the (r, s, c) loop whole and cut into 3 (uneven)
    and 8 parts whose partial sums a second kernel adds: bit for bit on small-integer data, within
    the precision's bar on random data with alpha and beta."""
    monkeypatch.setenv("DMATH_CONV_SPLIT", split)
    c = make_context(1.0)
    try:
        grids = {"X": (g["n"], 1), "F": (2, 1), "Y": (1, 1)}
        before = c.relayout_stats()["written"]
        res = three_modes(c, oracle, g, dt, out, 1.0, 1.0, grids, ints=True, policy=0)
        assert c.relayout_stats()["written"] - before == copies_written(g, dt)   # every mode on the specialised kernels
        for mode in ("fwd", "bwd_data"):
            got, ref = res[mode]
            if out == dm.F16 and np.abs(ref).max() > 2048:
                assert rel_fro(got, ref) <= TOL[dm.F16], mode
            else:
                assert np.array_equal(got.astype(np.float64), ref), mode
        res = three_modes(c, oracle, g, dt, out, 1.5, -0.5, {"X": (1, 1), "F": (1, 1), "Y": (1, 1)}, policy=0)
        for mode in ("fwd", "bwd_data"):
            got, ref = res[mode]
            assert rel_fro(got, ref) <= TOL[dt], mode
    finally:
        c.close()


@pytest.mark.parametrize("split", ["1", "3"])
@pytest.mark.parametrize("g", [
    dict(n=5, c=128, h=14, w=14, k=256, r=3, s=3, pad_h=1, pad_w=1),   # 18 k-tiles (parts of 6), ragged last row tile
    dict(n=4, c=64, h=16, w=16, k=256, r=3, s=1, pad_h=1, pad_w=0),    # 3 k-tiles (parts of 1)
    dict(n=4, c=64, h=16, w=16, k=256, r=2, s=2, pad_h=1, pad_w=1),    # 4 k-tiles, even filter (parts of 2, 2: two parts)
    dict(n=4, c=192, h=16, w=16, k=256, r=3, s=3, pad_h=1, pad_w=1),   # 27 k-tiles
])
@pytest.mark.parametrize("tile", ["224x256", "256x256", "256x128", "256x64"])
@pytest.mark.parametrize("out", [dm.F32, dm.F16])
def test_fp16_forward_tile_shapes_and_k_tile_counts(oracle, monkeypatch, out, tile, g, split):
    """Every fp16 tile shape of the forward pass / data gradient (16x16x32 fragments: 224x256,
    256x256, 256x128; 32x32x16: 256x64) over k-loops of 3 to 27 k-tiles, whole and in three parts
    (down to one k-tile per part): bit for bit on small-integer data with beta = 1."""
    monkeypatch.setenv("DMATH_CONV_TILE", tile)
    monkeypatch.setenv("DMATH_CONV_SPLIT", split)
    c = make_context(1.0)
    try:
        grids = {"X": (g["n"], 1), "F": (2, 1), "Y": (1, 1)}
        before = c.relayout_stats()["written"]
        res = three_modes(c, oracle, g, dm.F16, out, 1.0, 1.0, grids, ints=True, policy=0)
        assert c.relayout_stats()["written"] - before == copies_written(g, dm.F16)   # every mode on the specialised kernels
        for mode in ("fwd", "bwd_filter", "bwd_data"):
            got, ref = res[mode]
            if out == dm.F16 and np.abs(ref).max() > 2048:
                assert rel_fro(got, ref) <= TOL[dm.F16], mode
            else:
                assert np.array_equal(got.astype(np.float64), ref), mode
    finally:
        c.close()


@pytest.mark.parametrize("dt,out,tile", [(dm.F16, dm.F32, "256x64"), (dm.F32, dm.F32, "128x64"),
                                         (dm.F64, dm.F64, "128x64")])
def test_split_of_the_tiles_after_the_last_full_round(oracle, monkeypatch, dt, out, tile):
    """18000 pixels x 256 channels are 284 tiles of 256x64 (fp16: 256 workgroup slots) or 564 of
    128x64 (fp32, fp64: 512 slots): the tiles of the first full round run the whole (r, s, c)
    loop, the 28 / 52 left over run it in four parts.  Forward and data gradient, small-integer
    data, bit for bit on images of both kinds (the split tiles start at pixel 16384, in image 18)."""
    monkeypatch.setenv("DMATH_CONV_TILE", tile)
    monkeypatch.setenv("DMATH_CONV_SPLIT", "4t")
    g = dict(n=20, c=256, h=30, w=30, k=256, r=3, s=3, pad_h=1, pad_w=1)
    images = [0, 10, 18, 19]
    c = make_context(1.5)
    try:
        d, t = tensors(g, dt, 302, ints=True)
        od = oracle.ConvDesc(**g)
        X, F, dY = c.from_host(t["X"]), c.from_host(t["F"]), c.from_host(t["Y"])
        Y = c.from_host(np.ones(t["Y"].shape, NP[out]))
        dX = c.from_host(np.ones(t["X"].shape, NP[out]))
        dm.conv_fwd(c, d, 1.0, X, F, 1.0, Y)
        ref = oracle.conv_fwd(od, 1.0, t["X"], t["F"], images=images) + 1.0
        assert np.array_equal(Y.get()[images].astype(np.float64), ref)
        dm.conv_bwd_data(c, d, 1.0, dY, F, 1.0, dX)
        ref = oracle.conv_bwd_data(od, 1.0, t["Y"], t["F"], images=images) + 1.0
        assert np.array_equal(dX.get()[images].astype(np.float64), ref)
    finally:
        c.close()


def test_repeated_calls_rewrite_the_channels_last_copy(ctx, oracle):
    # the specialised path keeps a channels-last copy of X in the pool; a second call with new
    # contents of X must not see the old copy
    g = FAST_GEOMS[0]
    d, t = tensors(g, dm.F16, 301)
    od = oracle.ConvDesc(**g)
    dX, dF = ctx.from_host(t["X"]), ctx.from_host(t["F"])
    dY = ctx.matrix(*t["Y"].shape, (1, 1), dm.F32)
    dm.conv_fwd(ctx, d, 1.0, dX, dF, 0.0, dY)
    first = dY.get()
    x2 = (1 - t["X"].astype(np.float32)).astype(np.float16)
    dX.set(x2)
    dm.conv_fwd(ctx, d, 1.0, dX, dF, 0.0, dY)
    assert rel_fro(dY.get(), oracle.conv_fwd(od, 1.0, x2, t["F"])) <= TOL[dm.F16]
    assert rel_fro(first, oracle.conv_fwd(od, 1.0, t["X"], t["F"])) <= TOL[dm.F16]
    for m in (dX, dF, dY):
        m.destroy()


@pytest.mark.parametrize("seed", range(8))
def test_random_geometries_against_oracle(ctx, oracle, seed):
    """Seeded sweep over geometries (filter sizes 1..5, strides 1..3, pads up to the filter size
    minus one, odd channel counts; two cases in four are geometries that the specialised
    kernels accept), row-blocked tensors, all three modes, small-integer data compared bit for
    bit."""
    r = np.random.default_rng(8000 + seed)
    ctx.set_kernel_policy(0)
    for case in range(4):
        if case == 3:
            # any precision with channel and filter counts just below multiples of 64, any plane
            # size, strides and pads: the specialised kernels with padded copies and ragged tiles
            rr, ss = int(r.integers(1, 5)), int(r.integers(1, 5))
            g = dict(n=int(r.integers(1, 6)), c=int(r.integers(54, 65)) * int(r.integers(1, 3)),
                     h=int(r.integers(rr, rr + 12)), w=int(r.integers(ss, ss + 12)),
                     k=int(r.integers(54, 65)) * int(r.integers(1, 3)), r=rr, s=ss,
                     pad_h=int(r.integers(0, rr)), pad_w=int(r.integers(0, ss)),
                     stride_h=int(r.integers(1, 3)), stride_w=int(r.integers(1, 3)))
            dt, out = [(dm.F16, dm.F32), (dm.F16, dm.F16), (dm.F32, dm.F32), (dm.F64, dm.F64)][int(r.integers(0, 4))]
        elif case == 2:
            rr, ss = int(r.integers(1, 4)), int(r.integers(1, 4))
            hw = [(8, 8), (16, 8), (16, 16), (12, 12), (14, 14), (10, 10)][int(r.integers(0, 6))]
            g = dict(n=int(r.integers(1, 4)) * 4, c=int(r.integers(1, 3)) * 128, h=hw[0], w=hw[1], k=256, r=rr, s=ss,
                     pad_h=(rr - 1) // 2, pad_w=(ss - 1) // 2)
            if rr % 2 == 0 or ss % 2 == 0:       # even filters shrink the output: keep n*oh*ow a multiple of 256
                g["pad_h"], g["pad_w"] = rr // 2, ss // 2
            dt, out = dm.F16, [dm.F32, dm.F16][int(r.integers(0, 2))]
        else:
            rr, ss = int(r.integers(1, 6)), int(r.integers(1, 6))
            g = dict(n=int(r.integers(1, 5)), c=int(r.integers(1, 20)), h=int(r.integers(rr, rr + 12)),
                     w=int(r.integers(ss, ss + 12)), k=int(r.integers(1, 70)), r=rr, s=ss,
                     pad_h=int(r.integers(0, rr)), pad_w=int(r.integers(0, ss)),
                     stride_h=int(r.integers(1, 4)), stride_w=int(r.integers(1, 4)))
            dt, out = [(dm.F64, dm.F64), (dm.F32, dm.F32), (dm.F16, dm.F32), (dm.F16, dm.F16)][int(r.integers(0, 4))]
        grids = {"X": (min(2, g["n"]), 1), "F": (min(3, g["k"]), 1), "Y": (1, 1)}
        for mode, (got, ref) in three_modes(ctx, oracle, g, dt, out, 1.0, 1.0, grids, ints=True).items():
            what = (seed, case, mode, g, dt, out)
            if out == dm.F16 and np.abs(ref).max() > 2048:
                assert rel_fro(got, ref) <= TOL[dt], what
            else:
                assert np.array_equal(got.astype(np.float64), ref), what


@pytest.mark.parametrize("g", [dict(n=3, c=128, h=14, w=14, k=256, r=3, s=3, pad_h=1, pad_w=1),
                               dict(n=5, c=256, h=12, w=6, k=128, r=1, s=1)])
@pytest.mark.parametrize("dt,out", [(dm.F16, dm.F32), (dm.F16, dm.F16), (dm.F32, dm.F32), (dm.F64, dm.F64)])
def test_specialised_conv_ragged_last_row_tile(ctx, oracle, g, dt, out):
    """n*oh*ow is not a multiple of the row tile, nor of the weight gradient's pixel tile:
    the last tile of the forward and of the data gradient is ragged (clamped gathers, masked
    stores), the weight gradient's last pixel tile reads zeros past the end.  Small-integer data,
    bit for bit."""
    grids = {"X": (g["n"], 1), "F": (2, 1), "Y": (1, 1)}
    before = ctx.relayout_stats()["written"]
    res = three_modes(ctx, oracle, g, dt, out, 1.0, 1.0, grids, ints=True, policy=0)
    assert ctx.relayout_stats()["written"] - before == copies_written(g, dt)   # every mode on the specialised kernels
    for mode, (got, ref) in res.items():
        if out == dm.F16 and np.abs(ref).max() > 2048:
            assert rel_fro(got, ref) <= TOL[dm.F16], mode
        else:
            assert np.array_equal(got.astype(np.float64), ref), mode


@pytest.mark.parametrize("y_grid", [(1, 1), (2, 1)])
def test_fp16_weight_gradient_with_a_k_range_too_long_for_the_offset_table(oracle, monkeypatch, y_grid):
    """The fp16 weight gradient on 256x128 tiles keeps the pixel offsets of a part's k-range in an
    LDS table beside the pipeline's stages when they fit (up to 63 k-tiles per part); unsplit, the
    4608 pixels of this layer are 72 k-tiles, so the kernel steps its pixel counters instead.
    With dY read in place (one block) and through its channels-last copy (two blocks): bit for bit
    on small-integer data."""
    monkeypatch.setenv("DMATH_CONV_SPLIT", "1")
    g = dict(n=8, c=128, h=24, w=24, k=256, r=3, s=3, pad_h=1, pad_w=1)
    c = make_context(1.0)
    try:
        grids = {"X": (1, 1), "F": (1, 1), "Y": y_grid}
        res = three_modes(c, oracle, g, dm.F16, dm.F32, 1.0, 1.0, grids, ints=True, policy=0)
        got, ref = res["bwd_filter"]
        assert np.array_equal(got.astype(np.float64), ref)
    finally:
        c.close()
