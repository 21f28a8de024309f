"""Pins of the CPU convolution oracles (forward, weight gradient, data gradient), CPU only.

The paper names convolution (abstract) and its use in back-propagation (section 1) without a
formula; expectations here are hand-worked literals, exact special cases and identities that
fix the flip convention, the (r,s)->(h,w) axis order, the padding and the stride."""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "conv_hand_cases.txt")


def rng(seed):
    return np.random.default_rng(seed)


def parse_rows(s):
    return np.array([[float(v) for v in row.split()] for row in s.strip().split(";")])


def hand_cases():
    out = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = [x.strip() for x in line.split("|")]
        h, w = map(int, f[1].split())
        r, s = map(int, f[2].split())
        ph, pw = map(int, f[3].split())
        sh, sw = map(int, f[4].split())
        out.append((f[0], h, w, r, s, ph, pw, sh, sw, parse_rows(f[5]), parse_rows(f[6]),
                    parse_rows(f[7])))
    return out


@pytest.mark.parametrize("case", hand_cases(), ids=lambda c: c[0])
@pytest.mark.parametrize("dt", [np.float64, np.float32, np.float16])
def test_hand_worked_literals(oracle, case, dt):
    _, h, w, r, s, ph, pw, sh, sw, X, F, want = case
    d = oracle.ConvDesc(1, 1, h, w, 1, r, s, ph, pw, sh, sw)
    got = oracle.conv_fwd(d, 1.0, X.reshape(1, -1).astype(dt), F.reshape(1, -1).astype(dt))
    assert got.shape == (1, want.size)
    assert np.array_equal(got.reshape(want.shape), want)


def im2col(d, X):
    """Explicit lowering, written independently of the C loops: rows (n,oh,ow), cols (c,r,s)."""
    oh, ow = d.out_hw()
    x = X.reshape(d.n, d.c, d.h, d.w).astype(np.float64)
    xp = np.zeros((d.n, d.c, d.h + 2 * d.pad_h, d.w + 2 * d.pad_w))
    xp[:, :, d.pad_h:d.pad_h + d.h, d.pad_w:d.pad_w + d.w] = x
    cols = np.empty((d.n, oh, ow, d.c, d.r, d.s))
    for r in range(d.r):
        for s in range(d.s):
            cols[:, :, :, :, r, s] = xp[:, :, r:r + (oh - 1) * d.stride_h + 1:d.stride_h,
                                        s:s + (ow - 1) * d.stride_w + 1:d.stride_w].transpose(0, 2, 3, 1)
    return cols.reshape(d.n * oh * ow, d.c * d.r * d.s)


GEOMS = [
    dict(n=2, c=3, h=6, w=5, k=4, r=3, s=3, pad_h=1, pad_w=1),
    dict(n=3, c=2, h=7, w=8, k=3, r=3, s=2, pad_h=0, pad_w=1, stride_h=2, stride_w=1),
    dict(n=1, c=4, h=5, w=5, k=2, r=1, s=1),
    dict(n=2, c=2, h=9, w=7, k=3, r=5, s=3, pad_h=2, pad_w=0, stride_h=2, stride_w=3),
]


@pytest.mark.parametrize("g", GEOMS)
def test_direct_loops_equal_im2col_gemm(oracle, g):
    d = oracle.ConvDesc(**g)
    oh, ow = d.out_hw()
    r = rng(21)
    X = r.uniform(0, 1, (d.n, d.c * d.h * d.w)).astype(np.float32)
    F = r.normal(0, 0.3, (d.k, d.c * d.r * d.s)).astype(np.float32)
    Y0 = r.normal(0, 1, (d.n, d.k * oh * ow)).astype(np.float32)
    got = oracle.conv_fwd(d, 1.5, X, F, -0.5, Y0)
    cols = im2col(d, X)
    # second route: the lowered matrix through the oracle GEMM (N,T): [n*oh*ow x crs] * F^T
    y = oracle.gemm(False, True, 1.0, cols, F.astype(np.float64), 0.0)
    y = y.reshape(d.n, oh * ow, d.k).transpose(0, 2, 1).reshape(d.n, -1)
    want = 1.5 * y - 0.5 * Y0.astype(np.float64)
    assert oracle.rel_frobenius(got, want) < 1e-13
    # weight gradient = cols^T-contraction: dF[k, crs] = sum_m dY[m,k] cols[m,crs]
    dY = r.normal(0, 0.1, (d.n, d.k * oh * ow)).astype(np.float32)
    dF0 = r.normal(0, 1, (d.k, d.c * d.r * d.s)).astype(np.float32)
    gotF = oracle.conv_bwd_filter(d, 2.0, X, dY, 1.0, dF0)
    dy_m = dY.astype(np.float64).reshape(d.n, d.k, oh * ow).transpose(0, 2, 1).reshape(-1, d.k)
    wantF = 2.0 * oracle.gemm(True, False, 1.0, dy_m, cols, 0.0) + dF0.astype(np.float64)
    assert oracle.rel_frobenius(gotF, wantF) < 1e-13


def test_one_by_one_conv_is_a_gemm(oracle):
    d = oracle.ConvDesc(n=3, c=5, h=4, w=6, k=7, r=1, s=1)
    r = rng(22)
    X = r.integers(-3, 4, (d.n, d.c * 24)).astype(np.float32)
    F = r.integers(-3, 4, (d.k, d.c)).astype(np.float32)
    got = oracle.conv_fwd(d, 1.0, X, F)
    for n in range(d.n):
        yn = oracle.gemm(False, False, 1.0, F, X[n].reshape(d.c, 24), 0.0)   # [k x hw]
        assert np.array_equal(got[n].reshape(d.k, 24), yn)


@pytest.mark.parametrize("dt", [np.float64, np.float32, np.float16])
def test_centre_delta_filter_is_identity(oracle, dt):
    d = oracle.ConvDesc(n=2, c=3, h=5, w=4, k=3, r=3, s=3, pad_h=1, pad_w=1)
    X = rng(23).uniform(0, 1, (2, 60)).astype(dt)
    F = np.zeros((3, 3, 3, 3), dt)
    for k in range(3):
        F[k, k, 1, 1] = 1
    got = oracle.conv_fwd(d, 1.0, X, F.reshape(3, 27))
    assert np.array_equal(got, X.astype(np.float64))


def test_off_centre_delta_fixes_flip_and_axis_order(oracle):
    # only F[k,k,0,2] = 1  =>  Y[oh,ow] = X[oh-1, ow+1], zero where that falls outside.
    d = oracle.ConvDesc(n=1, c=2, h=4, w=5, k=2, r=3, s=3, pad_h=1, pad_w=1)
    X = np.arange(40, dtype=np.float64).reshape(1, 40) + 1
    F = np.zeros((2, 2, 3, 3))
    F[0, 0, 0, 2] = 1
    F[1, 1, 0, 2] = 1
    got = oracle.conv_fwd(d, 1.0, X, F.reshape(2, 18)).reshape(2, 4, 5)
    x = X.reshape(2, 4, 5)
    want = np.zeros((2, 4, 5))
    want[:, 1:, :-1] = x[:, :-1, 1:]
    assert np.array_equal(got, want)


def test_all_ones_counts_taps(oracle):
    d = oracle.ConvDesc(n=1, c=6, h=5, w=7, k=2, r=3, s=3, pad_h=1, pad_w=1)
    got = oracle.conv_fwd(d, 1.0, np.ones((1, 6 * 35), np.float16), np.ones((2, 54), np.float16))
    taps = np.full((5, 7), 9.0)
    taps[0, :] = taps[-1, :] = 6
    taps[:, 0] = taps[:, -1] = 6
    taps[0, 0] = taps[0, -1] = taps[-1, 0] = taps[-1, -1] = 4
    assert np.array_equal(got.reshape(2, 5, 7), np.broadcast_to(6 * taps, (2, 5, 7)))


@pytest.mark.parametrize("g", GEOMS)
def test_adjoint_identities_pin_both_gradients(oracle, g):
    # <dY, conv(X,F)> = <dF(X,dY), F> = <dX(dY,F), X>
    d = oracle.ConvDesc(**g)
    oh, ow = d.out_hw()
    r = rng(24)
    X = r.uniform(0, 1, (d.n, d.c * d.h * d.w))
    F = r.normal(0, 0.3, (d.k, d.c * d.r * d.s))
    dY = r.normal(0, 0.1, (d.n, d.k * oh * ow))
    Y = oracle.conv_fwd(d, 1.0, X, F)
    dF = oracle.conv_bwd_filter(d, 1.0, X, dY)
    dX = oracle.conv_bwd_data(d, 1.0, dY, F)
    s0 = float((dY * Y).sum())
    assert abs(float((dF * F).sum()) - s0) <= 1e-12 * abs(s0)
    assert abs(float((dX * X).sum()) - s0) <= 1e-12 * abs(s0)


def test_brute_force_tiny_all_three(oracle):
    d = oracle.ConvDesc(n=2, c=2, h=4, w=3, k=2, r=2, s=3, pad_h=1, pad_w=1, stride_h=2, stride_w=1)
    oh, ow = d.out_hw()
    r = rng(25)
    X = r.integers(-3, 4, (2, 2, 4, 3)).astype(np.float64)
    F = r.integers(-3, 4, (2, 2, 2, 3)).astype(np.float64)
    dY = r.integers(-3, 4, (2, 2, oh, ow)).astype(np.float64)
    Y = np.zeros((2, 2, oh, ow))
    dF = np.zeros_like(F)
    dX = np.zeros_like(X)
    for n in range(2):
        for k in range(2):
            for a in range(oh):
                for b in range(ow):
                    for c in range(2):
                        for p in range(2):
                            for q in range(3):
                                ih, iw = a * 2 + p - 1, b * 1 + q - 1
                                if 0 <= ih < 4 and 0 <= iw < 3:
                                    Y[n, k, a, b] += X[n, c, ih, iw] * F[k, c, p, q]
                                    dF[k, c, p, q] += dY[n, k, a, b] * X[n, c, ih, iw]
                                    dX[n, c, ih, iw] += dY[n, k, a, b] * F[k, c, p, q]
    assert np.array_equal(oracle.conv_fwd(d, 1.0, X.reshape(2, -1), F.reshape(2, -1)), Y.reshape(2, -1))
    assert np.array_equal(oracle.conv_bwd_filter(d, 1.0, X.reshape(2, -1), dY.reshape(2, -1)),
                          dF.reshape(2, -1))
    assert np.array_equal(oracle.conv_bwd_data(d, 1.0, dY.reshape(2, -1), F.reshape(2, -1)),
                          dX.reshape(2, -1))


def test_selection_and_block_rows(oracle):
    d = oracle.ConvDesc(n=4, c=2, h=5, w=5, k=3, r=3, s=3, pad_h=1, pad_w=1)
    r = rng(26)
    X = r.uniform(0, 1, (4, 50)).astype(np.float16)
    F = r.normal(0, 0.3, (3, 18)).astype(np.float16)
    dY = r.normal(0, 0.1, (4, 75)).astype(np.float16)
    full = oracle.conv_fwd(d, 1.0, X, F)
    assert np.array_equal(oracle.conv_fwd(d, 1.0, oracle.BlockMatrix(X, (2, 1)), F, images=[3, 1]),
                          full[[3, 1]])
    fullF = oracle.conv_bwd_filter(d, 1.0, X, dY)
    assert np.array_equal(oracle.conv_bwd_filter(d, 1.0, oracle.BlockMatrix(X, (4, 1)),
                                                 oracle.BlockMatrix(dY, (2, 1)), filters=[2]), fullF[[2]])
    fullX = oracle.conv_bwd_data(d, 1.0, dY, F)
    assert np.array_equal(oracle.conv_bwd_data(d, 1.0, dY, F, images=[0, 2]), fullX[[0, 2]])


def test_alpha_beta_and_nan_rules(oracle):
    d = oracle.ConvDesc(n=1, c=1, h=3, w=3, k=1, r=3, s=3, pad_h=1, pad_w=1)
    X = rng(27).uniform(0, 1, (1, 9))
    F = rng(28).uniform(0, 1, (1, 9))
    Y0 = rng(29).uniform(0, 1, (1, 9))
    y = oracle.conv_fwd(d, 1.0, X, F)
    assert np.array_equal(oracle.conv_fwd(d, 1.0, X, F, 0.0, np.full((1, 9), np.nan)), y)
    assert np.array_equal(oracle.conv_fwd(d, 0.0, np.full((1, 9), np.nan), F, 2.0, Y0), 2.0 * Y0)
    assert np.array_equal(oracle.conv_fwd(d, 2.0, X, F, 1.0, Y0), 2.0 * y + Y0)
