"""Pins of the CPU GEMM oracle against what the definition fixes (CPU only).

The paper (abstract; section 2.1 for blocks; section 3.2 for layout independence) names the
operation but prints no values, so every expectation here is a closed form, an exact special
case, an algebraic identity or a hand-expanded literal."""
import itertools
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "gemm_hand_cases.txt")
DT = [np.float64, np.float32, np.float16]
GRIDS = [(1, 1), (2, 2), (3, 2), (1, 4)]


def rng(seed):
    return np.random.default_rng(seed)


def ints(r, shape, dt, lo=-3, hi=3):
    return r.integers(lo, hi + 1, size=shape).astype(dt)


def op(x, t):
    return x.T if t else x


def parse_rows(s):
    return np.array([[float(v) for v in row.split()] for row in s.strip().split(";")])


def hand_cases():
    out = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = [x.strip() for x in line.split("|")]
        ta, tb = f[1].split()
        al, be = (float(v) for v in f[2].split())
        out.append((f[0], ta == "T", tb == "T", al, be, parse_rows(f[3]), parse_rows(f[4]),
                    parse_rows(f[5]), parse_rows(f[6])))
    return out


@pytest.mark.parametrize("case", hand_cases(), ids=lambda c: c[0])
@pytest.mark.parametrize("dt", DT)
def test_hand_expanded_literals(oracle, case, dt):
    _, ta, tb, al, be, A, B, C, want = case
    got = oracle.gemm(ta, tb, al, A.astype(dt), B.astype(dt), be, C.astype(dt))
    assert np.array_equal(got, want)


def test_half_decode_matches_ieee(oracle):
    # every one of the 65536 bit patterns, against numpy's float16 -> float64 widening
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    same = (got == want) | (np.isnan(got) & np.isnan(want))
    assert same.all()
    assert np.array_equal(np.signbit(got), np.signbit(want))


def test_split_rule(oracle):
    assert oracle.split_bounds(10, 3) == [(0, 4), (4, 8), (8, 10)]
    assert oracle.split_bounds(8, 4) == [(0, 2), (2, 4), (4, 6), (6, 8)]
    with pytest.raises(ValueError):
        oracle.BlockMatrix(np.zeros((9, 4)), (4, 1))     # ceil(9/4)=3: 4th part would be empty
    m = np.arange(35, dtype=np.float64).reshape(5, 7)
    bm = oracle.BlockMatrix(m, (2, 3))
    assert [b.shape for b in bm.blocks] == [(3, 3), (3, 3), (3, 1), (2, 3), (2, 3), (2, 1)]
    assert np.array_equal(bm.blocks[4], m[3:5, 3:6])


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("grid", GRIDS)
@pytest.mark.parametrize("ta,tb", list(itertools.product([False, True], repeat=2)))
def test_identity_is_bitwise(oracle, dt, grid, ta, tb):
    r = rng(1)
    n = 12
    A = r.uniform(-1, 1, (n, n)).astype(dt)
    I = np.eye(n, dtype=dt)
    got = oracle.gemm(ta, tb, 1.0, oracle.BlockMatrix(A, grid), oracle.BlockMatrix(I, grid), 0.0)
    assert np.array_equal(got, op(A, ta).astype(np.float64))
    got = oracle.gemm(ta, tb, 1.0, oracle.BlockMatrix(I, grid), oracle.BlockMatrix(A, grid), 0.0)
    assert np.array_equal(got, op(A, tb).astype(np.float64))


@pytest.mark.parametrize("dt", DT)
def test_permutation_is_bitwise(oracle, dt):
    r = rng(2)
    A = r.uniform(-1, 1, (9, 6)).astype(dt)
    p = r.permutation(9)
    P = np.zeros((9, 9), dt)
    P[np.arange(9), p] = 1          # (P A)[i] = A[p[i]]
    got = oracle.gemm(False, False, 1.0, oracle.BlockMatrix(P, (3, 3)),
                      oracle.BlockMatrix(A, (3, 2)), 0.0)
    assert np.array_equal(got, A[p].astype(np.float64))
    q = r.permutation(6)
    Q = np.zeros((6, 6), dt)
    Q[q, np.arange(6)] = 1          # (A Q)[:, j] = A[:, q[j]]
    got = oracle.gemm(False, False, 1.0, A, Q, 0.0)
    assert np.array_equal(got, A[:, q].astype(np.float64))


@pytest.mark.parametrize("dt", DT)
def test_power_of_two_diagonal_is_bitwise(oracle, dt):
    r = rng(3)
    A = r.uniform(-1, 1, (8, 5)).astype(dt)
    d = (2.0 ** r.integers(-3, 4, size=8)).astype(dt)
    got = oracle.gemm(False, False, 1.0, np.diag(d), A, 0.0)
    assert np.array_equal(got, d[:, None].astype(np.float64) * A.astype(np.float64))
    e = (2.0 ** r.integers(-3, 4, size=5)).astype(dt)
    got = oracle.gemm(False, False, 1.0, A, np.diag(e), 0.0)
    assert np.array_equal(got, A.astype(np.float64) * e[None, :].astype(np.float64))


def test_rank_one_closed_form(oracle):
    r = rng(4)
    u = r.uniform(-1, 1, (7, 1))
    v = r.uniform(-1, 1, (1, 5))
    C0 = r.uniform(-1, 1, (7, 5))
    got = oracle.gemm(False, False, 1.5, u, v, -0.5, C0)
    want = 1.5 * (u * v) + (-0.5) * C0
    assert np.allclose(got, want, rtol=4e-16, atol=0)
    # the same through the transposed operands
    got = oracle.gemm(True, True, 1.5, u.T.copy(), v.T.copy(), -0.5, C0)
    assert np.allclose(got, want, rtol=4e-16, atol=0)


@pytest.mark.parametrize("dt", DT)
def test_constant_matrices(oracle, dt):
    M, N, K = 6, 10, 37
    A = np.full((M, K), 2, dt)
    B = np.full((K, N), -3, dt)
    got = oracle.gemm(False, False, 1.0, oracle.BlockMatrix(A, (2, 4)),
                      oracle.BlockMatrix(B, (4, 3)), 0.0)
    assert np.array_equal(got, np.full((M, N), K * 2 * -3, np.float64))


@pytest.mark.parametrize("dt", DT)
@pytest.mark.parametrize("ta,tb", list(itertools.product([False, True], repeat=2)))
def test_all_ops_vs_explicit_transposes_exact_on_integers(oracle, dt, ta, tb):
    # integer inputs: every order of summation gives the same bits, so "==" is the bar.
    r = rng(5)
    M, N, K = 11, 13, 17
    opA, opB = ints(r, (M, K), dt), ints(r, (K, N), dt)
    A = np.ascontiguousarray(op(opA, ta))        # stored so that op(A) == opA
    B = np.ascontiguousarray(op(opB, tb))
    C0 = ints(r, (M, N), dt)
    want = 2.0 * (opA.astype(np.int64) @ opB.astype(np.int64)) + 3.0 * C0.astype(np.float64)
    for ga, gb, gc in [((1, 1), (1, 1), (1, 1)), ((2, 3), (3, 2), (2, 2)), ((4, 1), (2, 5), (3, 4))]:
        got = oracle.gemm(ta, tb, 2.0, oracle.BlockMatrix(A, ga), oracle.BlockMatrix(B, gb), 3.0,
                          oracle.BlockMatrix(C0, gc))
        assert np.array_equal(got, want)


def test_transpose_identity(oracle):
    # (A B)^T = B^T A^T : gemm(T,T; B, A) is the transpose of gemm(N,N; A, B)
    r = rng(6)
    A = r.uniform(-1, 1, (9, 14))
    B = r.uniform(-1, 1, (14, 6))
    ab = oracle.gemm(False, False, 1.0, A, B, 0.0)
    bt_at = oracle.gemm(True, True, 1.0, B, A, 0.0)
    assert np.array_equal(bt_at, ab.T)      # same products, same summation order: bitwise


def test_block_decomposed_equals_monolithic(oracle):
    # section 3.2: results are independent of the layout.  Same arithmetic order => bitwise.
    r = rng(7)
    A = r.uniform(-1, 1, (23, 31)).astype(np.float32)
    B = r.uniform(-1, 1, (31, 19)).astype(np.float32)
    C = r.uniform(-1, 1, (23, 19)).astype(np.float32)
    mono = oracle.gemm(False, False, 1.0, A, B, 1.0, C)
    for ga, gb, gc in [((2, 2), (2, 2), (2, 2)), ((5, 3), (4, 7), (3, 3)), ((23, 1), (1, 19), (1, 1))]:
        got = oracle.gemm(False, False, 1.0, oracle.BlockMatrix(A, ga), oracle.BlockMatrix(B, gb),
                          1.0, oracle.BlockMatrix(C, gc))
        assert np.array_equal(got, mono)


def test_alpha_beta_algebra_and_nan_rules(oracle):
    r = rng(8)
    A = r.uniform(-1, 1, (5, 4))
    B = r.uniform(-1, 1, (4, 6))
    C = r.uniform(-1, 1, (5, 6))
    ab = oracle.gemm(False, False, 1.0, A, B, 0.0)
    assert np.array_equal(oracle.gemm(False, False, 0.0, A, B, 0.0, C), np.zeros((5, 6)))
    assert np.array_equal(oracle.gemm(False, False, 0.0, A, B, 1.0, C), C)
    assert np.array_equal(oracle.gemm(False, False, 1.0, A, B, 1.0, C), ab + C)
    assert np.array_equal(oracle.gemm(False, False, 1.5, A, B, -0.5, C), 1.5 * ab + (-0.5) * C)
    # beta == 0: old C is not read; alpha == 0: A and B are not read
    nanC = np.full((5, 6), np.nan)
    assert np.array_equal(oracle.gemm(False, False, 1.0, A, B, 0.0, nanC), ab)
    nanA = np.full((5, 4), np.nan)
    assert np.array_equal(oracle.gemm(False, False, 0.0, nanA, B, 2.0, C), 2.0 * C)
    # and they do propagate when they are read
    assert np.isnan(oracle.gemm(False, False, 1.0, nanA, B, 0.0)).all()


def test_linearity(oracle):
    r = rng(9)
    A = r.uniform(-1, 1, (8, 16))
    B1 = r.uniform(-1, 1, (16, 5))
    B2 = r.uniform(-1, 1, (16, 5))
    lhs = oracle.gemm(False, False, 1.0, A, B1 + B2, 0.0)
    rhs = oracle.gemm(False, False, 1.0, A, B1, 0.0) + oracle.gemm(False, False, 1.0, A, B2, 0.0)
    assert oracle.rel_frobenius(lhs, rhs) < 1e-15


def test_adjoint_identity_pins_tn_and_nt(oracle):
    # <dY, X W> = <X^T dY, W> = <dY W^T, X>: fixes the back-propagation variants from NN.
    r = rng(10)
    X = r.uniform(0, 1, (12, 20))
    W = r.normal(0, 0.2, (20, 9))
    dY = r.normal(0, 0.1, (12, 9))
    g = ((2, 2), (2, 3), (3, 1))
    Y = oracle.gemm(False, False, 1.0, oracle.BlockMatrix(X, g[0]), oracle.BlockMatrix(W, g[1]), 0.0)
    dW = oracle.gemm(True, False, 1.0, oracle.BlockMatrix(X, g[0]), oracle.BlockMatrix(dY, g[2]), 0.0)
    dX = oracle.gemm(False, True, 1.0, oracle.BlockMatrix(dY, g[2]), oracle.BlockMatrix(W, g[1]), 0.0)
    s0 = float((dY * Y).sum())
    assert abs(float((dW * W).sum()) - s0) <= 1e-12 * abs(s0)
    assert abs(float((dX * X).sum()) - s0) <= 1e-12 * abs(s0)
    assert dW.shape == W.shape and dX.shape == X.shape


def test_brute_force_tiny(oracle):
    r = rng(11)
    for (M, N, K) in [(1, 1, 1), (2, 3, 1), (3, 2, 8), (8, 8, 8), (5, 7, 3)]:
        for ta, tb in itertools.product([False, True], repeat=2):
            opA = r.uniform(-1, 1, (M, K))
            opB = r.uniform(-1, 1, (K, N))
            C0 = r.uniform(-1, 1, (M, N))
            want = np.empty((M, N))
            for i in range(M):
                for j in range(N):
                    acc = 0.0
                    for k in range(K):
                        acc += opA[i, k] * opB[k, j]
                    want[i, j] = 0.75 * acc + 0.25 * C0[i, j]
            got = oracle.gemm(ta, tb, 0.75, np.ascontiguousarray(op(opA, ta)),
                              np.ascontiguousarray(op(opB, tb)), 0.25, C0)
            assert np.array_equal(got, want)


@pytest.mark.parametrize("dt,tol", [(np.float64, 1e-13), (np.float32, 1e-13), (np.float16, 1e-13)])
def test_against_numpy_matmul(oracle, dt, tol):
    # the inputs are widened exactly, so numpy's float64 matmul of the widened inputs is the
    # same mathematical quantity; only the summation order differs.
    r = rng(12)
    A = r.uniform(-1, 1, (64, 200)).astype(dt)
    B = r.uniform(-1, 1, (200, 48)).astype(dt)
    got = oracle.gemm(False, False, 1.0, oracle.BlockMatrix(A, (4, 4)),
                      oracle.BlockMatrix(B, (4, 3)), 0.0)
    assert oracle.rel_frobenius(got, A.astype(np.float64) @ B.astype(np.float64)) < tol


def test_row_selection(oracle):
    r = rng(13)
    A = r.uniform(-1, 1, (20, 9)).astype(np.float32)
    B = r.uniform(-1, 1, (9, 11)).astype(np.float32)
    C = r.uniform(-1, 1, (20, 11)).astype(np.float32)
    full = oracle.gemm(False, False, 1.5, oracle.BlockMatrix(A, (3, 2)), B, -0.5,
                       oracle.BlockMatrix(C, (2, 2)))
    rows = [19, 0, 7, 7]
    part = oracle.gemm(False, False, 1.5, oracle.BlockMatrix(A, (3, 2)), B, -0.5,
                       oracle.BlockMatrix(C, (2, 2)), rows=rows)
    assert np.array_equal(part, full[rows])
    fullT = oracle.gemm(True, False, 1.0, np.ascontiguousarray(A.T), B, 0.0)
    partT = oracle.gemm(True, False, 1.0, np.ascontiguousarray(A.T), B, 0.0, rows=rows)
    assert np.array_equal(partT, fullT[rows])


def test_shape_errors(oracle):
    with pytest.raises(ValueError):
        oracle.gemm(False, False, 1.0, np.zeros((3, 4)), np.zeros((5, 2)), 0.0)
    with pytest.raises(ValueError):
        oracle.gemm(False, False, 1.0, np.zeros((3, 4)), np.zeros((4, 2)), 1.0, np.zeros((3, 3)))
    with pytest.raises(ValueError):
        oracle.gemm(False, False, 1.0, np.zeros((3, 4)), np.zeros((4, 2)), 1.0, None)


def test_fp64_accuracy_on_deep_k(oracle):
    # the oracle's own rounding error at K = 8192 stays far below the 1e-12 fp64 parity bar:
    # compare a few rows against exact rational arithmetic rounded once (math.fsum of exact
    # products of fp32-representable inputs, whose products are exact in fp64).
    import math
    r = rng(14)
    K = 8192
    A = r.uniform(-1, 1, (2, K)).astype(np.float32).astype(np.float64)
    B = r.uniform(-1, 1, (K, 3)).astype(np.float32).astype(np.float64)
    got = oracle.gemm(False, False, 1.0, A, B, 0.0)
    want = np.array([[math.fsum(A[i] * B[:, j]) for j in range(3)] for i in range(2)])
    assert np.abs(got - want).max() <= 1e-13 * np.abs(want).max() + 1e-13


def test_convert_rounds_once_to_nearest_even(oracle):
    # ties and a double-rounding trap, checked against hand-computed binary16 / binary32 values
    h = np.float64
    ulp16 = 2.0 ** -10                       # spacing of binary16 in [1, 2)
    src = np.array([[1 + ulp16 / 2,          # tie -> even (1.0)
                     1 + 3 * ulp16 / 2,      # tie -> even (1 + 2 ulp)
                     1 + ulp16 / 2 + 2.0 ** -40,   # just above the tie: must round UP (a detour over
                                                   # binary32 would first land on the tie, then go down)
                     65504.0, 65520.0, 1e-8, -2.0 ** -25]], dtype=h)
    with np.errstate(over="ignore"):
        got = oracle.convert(src, np.float16).astype(h)
    want = np.array([[1.0, 1 + 2 * ulp16, 1 + ulp16, 65504.0, np.inf, 0.0, -0.0]])
    assert np.array_equal(got, want)
    assert np.signbit(got[0, 6])
    f = oracle.convert(np.array([[1 + 2.0 ** -24, 1 + 3 * 2.0 ** -24]]), np.float32).astype(h)
    assert np.array_equal(f, np.array([[1.0, 1 + 2.0 ** -22]]))
    # widening is exact
    x = np.random.default_rng(30).uniform(-1, 1, (5, 7)).astype(np.float16)
    assert np.array_equal(oracle.convert(x, np.float64), x.astype(np.float64))
