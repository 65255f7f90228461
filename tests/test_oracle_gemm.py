"""Pins for the GEMM oracle (CPU only): closed forms, identities and brute force.

The oracle implements Eq. 1 of Section 2.2 (C = alpha*op(A)*op(B) + beta*C).
Nothing here compares the oracle with itself through the same formula: each
check is a case whose answer is known independently (identity / permutation
operands, all-ones, rank-1, exact integer arithmetic, exact rational
arithmetic, numpy's fp64 matmul) or an identity between differently-indexed
calls (transposes, layouts), so that a wrong index, a swapped operand, a
dropped beta or alpha term or a transposed leading dimension fails at least one.
"""
from fractions import Fraction
import itertools

import numpy as np
import pytest

from oracle import gemm_oracle as go
from paper_1806_07060_amd import workloads as wl

CM, RM = go.COL_MAJOR, go.ROW_MAJOR
NT, TR, CT = go.NO_TRANS, go.TRANS, go.CONJ_TRANS


def store(mat, layout, ld=None, fill=np.nan):
    """Flat fp32 buffer holding logical matrix `mat` in the given layout with leading dimension ld."""
    rows, cols = mat.shape
    min_ld = max(1, rows if layout == CM else cols)
    ld = ld or min_ld
    assert ld >= min_ld
    buf = np.full(wl.buffer_len(layout, (rows, cols), ld), fill, np.float32)
    v = wl.matrix_view(buf, layout, (rows, cols), ld)
    if v.size:
        v[...] = mat
    return buf, ld


def run(opA_mat, opB_mat, C0, alpha=1.0, beta=0.0, tA=NT, tB=NT, layout=CM, pad=(0, 0, 0), scalar=False):
    """Call the oracle on logical op(A) [MxK], op(B) [KxN], C0 [MxN]; returns the logical result matrix."""
    M, K = opA_mat.shape
    N = opB_mat.shape[1]
    Ast = opA_mat.T if tA != NT else opA_mat
    Bst = opB_mat.T if tB != NT else opB_mat
    a, lda = store(Ast, layout, (max(1, Ast.shape[0] if layout == CM else Ast.shape[1]) + pad[0]))
    b, ldb = store(Bst, layout, (max(1, Bst.shape[0] if layout == CM else Bst.shape[1]) + pad[1]))
    c, ldc = store(C0, layout, (max(1, M if layout == CM else N) + pad[2]), fill=wl.C_SENTINEL)
    before = c.copy()
    st = go.sgemm(layout, tA, tB, M, N, K, alpha, a, lda, b, ldb, beta, c, ldc, scalar=scalar)
    assert st == 0
    # padding of C must be untouched
    mask = np.ones(c.shape, bool)
    idx = wl.matrix_view(np.arange(c.size), layout, (M, N), ldc)
    mask[idx.ravel()] = False
    assert np.array_equal(c[mask], before[mask])
    return wl.matrix_view(c, layout, (M, N), ldc).copy()


def rnd(shape, seed, lo=-1, hi=1):
    return np.random.default_rng(seed).uniform(lo, hi, size=shape).astype(np.float32)


ALL_T = list(itertools.product((NT, TR), (NT, TR)))
ALL_L = (CM, RM)


@pytest.mark.parametrize("layout", ALL_L)
@pytest.mark.parametrize("tA,tB", ALL_T)
def test_identity_left_and_right(layout, tA, tB):
    # I * B = B and A * I = A; with alpha = 2 and beta = 0.5 every value is exact in fp64 and
    # (float)(2 b + 0.5 c) is the correctly rounded closed form.
    B = rnd((7, 5), 1)
    C0 = rnd((7, 5), 2)
    got = run(np.eye(7, dtype=np.float32), B, C0, 2.0, 0.5, tA, tB, layout, pad=(3, 2, 1))
    want = (2.0 * B.astype(np.float64) + 0.5 * C0.astype(np.float64)).astype(np.float32)
    assert np.array_equal(got, want)
    A = rnd((6, 9), 3)
    C0 = rnd((6, 9), 4)
    got = run(A, np.eye(9, dtype=np.float32), C0, -4.0, 1.0, tA, tB, layout, pad=(1, 0, 2))
    want = (-4.0 * A.astype(np.float64) + C0.astype(np.float64)).astype(np.float32)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("layout", ALL_L)
@pytest.mark.parametrize("tA,tB", ALL_T)
def test_permutation_matrices(layout, tA, tB):
    # P with P[i, p[i]] = 1:  (P B)[i, :] = B[p[i], :]   and   (A P)[:, p[j]] = A[:, j]
    rng = np.random.default_rng(5)
    p = rng.permutation(8)
    P = np.zeros((8, 8), np.float32)
    P[np.arange(8), p] = 1.0
    B = rnd((8, 11), 6)
    got = run(P, B, np.zeros((8, 11), np.float32), 1.0, 0.0, tA, tB, layout, pad=(2, 3, 0))
    assert np.array_equal(got, B[p, :])
    A = rnd((5, 8), 7)
    got = run(A, P, np.zeros((5, 8), np.float32), 1.0, 0.0, tA, tB, layout)
    want = np.empty_like(A)
    want[:, p] = A
    assert np.array_equal(got, want)


@pytest.mark.parametrize("layout", ALL_L)
@pytest.mark.parametrize("tA,tB", ALL_T)
@pytest.mark.parametrize("M,N,K", [(3, 4, 5), (17, 1, 129), (1, 9, 1000), (33, 31, 64)])
def test_all_ones(layout, tA, tB, M, N, K):
    C0 = rnd((M, N), 8)
    got = run(np.ones((M, K), np.float32), np.ones((K, N), np.float32), C0, 0.5, 0.25, tA, tB, layout)
    want = (0.5 * K + 0.25 * C0.astype(np.float64)).astype(np.float32)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("layout", ALL_L)
@pytest.mark.parametrize("tA,tB", ALL_T)
def test_rank_one(layout, tA, tB):
    u = rnd((13, 1), 9)
    v = rnd((1, 10), 10)
    C0 = rnd((13, 10), 11)
    got = run(u, v, C0, 2.0, -1.0, tA, tB, layout, pad=(1, 1, 1))
    want = (2.0 * (u.astype(np.float64) * v.astype(np.float64)) - C0.astype(np.float64)).astype(np.float32)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("layout", ALL_L)
@pytest.mark.parametrize("tA,tB", ALL_T)
def test_small_integers_exact(layout, tA, tB):
    # integer-valued inputs: every partial sum is an integer far below 2^53 -> result equals integer arithmetic
    rng = np.random.default_rng(12)
    M, N, K = 19, 23, 301
    A = rng.integers(-8, 9, (M, K))
    B = rng.integers(-8, 9, (K, N))
    C0 = rng.integers(-8, 9, (M, N))
    got = run(A.astype(np.float32), B.astype(np.float32), C0.astype(np.float32), 3.0, -2.0, tA, tB, layout,
              pad=(2, 0, 5))
    want = 3 * (A @ B) - 2 * C0
    assert np.array_equal(got.astype(np.int64), want)
    assert np.array_equal(got, want.astype(np.float32))


def test_asymmetric_operands_not_swapped():
    # A B != B A and (A B)^T != A B for these; integer-exact, catches swapped operands / transposed output
    A = np.array([[1, 2], [3, 4], [5, 6]], np.float32)  # 3x2
    B = np.array([[1, 0, 2, 0], [0, 1, 0, 3]], np.float32)  # 2x4
    want = np.array([[1, 2, 2, 6], [3, 4, 6, 12], [5, 6, 10, 18]], np.float32)
    for layout in ALL_L:
        for tA, tB in ALL_T:
            assert np.array_equal(run(A, B, np.zeros((3, 4), np.float32), 1.0, 0.0, tA, tB, layout), want)


@pytest.mark.parametrize("layout", ALL_L)
def test_transpose_flags_are_pure_storage(layout):
    # the same logical op(A), op(B) stored four ways must give bit-identical results
    A = rnd((21, 34), 13)
    B = rnd((34, 15), 14)
    C0 = rnd((21, 15), 15)
    ref = run(A, B, C0, 1.25, 0.75, NT, NT, layout)
    for tA, tB in ALL_T:
        assert np.array_equal(run(A, B, C0, 1.25, 0.75, tA, tB, layout, pad=(1, 2, 3)), ref)
    assert np.array_equal(run(A, B, C0, 1.25, 0.75, CT, CT, layout), ref)


def test_layouts_agree_and_swap_identity():
    # row-major call == column-major call on the same logical matrices, and
    # C^T = op(B)^T op(A)^T: a column-major call on swapped operands yields the transpose, bit for bit.
    A = rnd((12, 29), 16)
    B = rnd((29, 18), 17)
    C0 = rnd((12, 18), 18)
    ref = run(A, B, C0, 0.5, 2.0, NT, TR, CM)
    assert np.array_equal(run(A, B, C0, 0.5, 2.0, TR, NT, RM), ref)
    swapped = run(B.T.copy(), A.T.copy(), C0.T.copy(), 0.5, 2.0, NT, NT, CM)
    assert np.array_equal(swapped.T, ref)


def test_power_of_two_linearity():
    A = rnd((9, 40), 19)
    B = rnd((40, 7), 20)
    C0 = rnd((9, 7), 21)
    base = run(A, B, C0, 1.0, 0.0)
    assert np.array_equal(run(A, B, C0, 4.0, 0.0), 4.0 * base)
    assert np.array_equal(run(A, B, C0, -0.125, 0.0), -0.125 * base)
    # beta term alone (alpha = 0)
    assert np.array_equal(run(A, B, C0, 0.0, 8.0), 8.0 * C0)


def test_special_scalars_and_degenerate_sizes():
    A = rnd((6, 5), 22)
    B = rnd((5, 4), 23)
    C0 = rnd((6, 4), 24)
    # beta = 0: C0 is not read, NaN / Inf do not propagate
    bad = np.full((6, 4), np.nan, np.float32)
    bad[0, 0] = np.inf
    assert np.array_equal(run(A, B, bad, 1.0, 0.0), run(A, B, np.zeros_like(C0), 1.0, 0.0))
    # alpha = 0: A and B are not read
    nanA = np.full_like(A, np.nan)
    assert np.array_equal(run(nanA, B, C0, 0.0, 0.5), 0.5 * C0)
    assert np.array_equal(run(nanA, B, C0, 0.0, 0.0), np.zeros_like(C0))
    # beta = 1: C0 added exactly (integers)
    Ai = np.round(4 * A)
    Bi = np.round(4 * B)
    Ci = np.round(4 * C0)
    assert np.array_equal(run(Ai, Bi, Ci, 1.0, 1.0), (Ai.astype(np.float64) @ Bi.astype(np.float64) + Ci).astype(np.float32))
    # K = 0: C = beta * C0
    assert np.array_equal(run(np.empty((6, 0), np.float32), np.empty((0, 4), np.float32), C0, 1.0, 0.5), 0.5 * C0)
    # M = 0 or N = 0: success, nothing touched
    for M, N in ((0, 4), (6, 0), (0, 0)):
        c = np.full(8, 3.0, np.float32)
        for fn_scalar in (False, True):
            assert go.sgemm(CM, NT, NT, M, N, 5, 1.0, A.ravel(), max(1, M), B.ravel(), 5, 1.0, c, max(1, M),
                            scalar=fn_scalar) == 0
            assert np.all(c == 3.0)


def test_argument_errors():
    a = np.zeros(64, np.float32)
    ok = dict(layout=CM, transA=NT, transB=NT, M=4, N=4, K=4, alpha=1.0, A=a, lda=4, B=a, ldb=4, beta=0.0, C=a.copy(),
              ldc=4)

    def call(**kw):
        d = dict(ok)
        d.update(kw)
        return go.sgemm(**d)

    assert call() == 0
    assert call(layout=100) == -1
    assert call(transA=0) == -2
    assert call(transB=114) == -3
    assert call(M=-1) == -4
    assert call(N=-1) == -5
    assert call(K=-1) == -6
    assert call(lda=3) == -9
    assert call(ldb=3) == -11
    assert call(ldc=3) == -14
    # leading dimension follows the stored shape: A^T stored is K x M
    assert call(transA=TR, M=8, K=2, lda=2, ldc=8, C=np.zeros(64, np.float32)) == 0
    assert call(transA=TR, M=8, K=2, lda=1, ldc=8, C=np.zeros(64, np.float32)) == -9
    assert call(layout=RM, M=2, N=8, K=4, lda=4, ldb=8, ldc=8) == 0
    assert call(layout=RM, M=2, N=8, K=4, lda=4, ldb=7, ldc=8) == -11
    assert call(layout=RM, M=2, N=8, K=4, lda=4, ldb=8, ldc=7) == -14
    # zero-sized problems still need ld >= 1
    assert call(M=0, lda=0) == -9


def exact_reference(A, B, C0, alpha, beta):
    """Exact rational value of alpha*A*B + beta*C0, rounded once to fp32 (tiny sizes only)."""
    M, K = A.shape
    N = B.shape[1]
    out = np.empty((M, N), np.float32)
    fa, fb = Fraction(float(np.float32(alpha))), Fraction(float(np.float32(beta)))
    for i in range(M):
        for j in range(N):
            s = Fraction(0)
            for k in range(K):
                s += Fraction(float(A[i, k])) * Fraction(float(B[k, j]))
            r = fa * s + (fb * Fraction(float(C0[i, j])) if beta != 0 else 0)
            # round exact rational to fp32 through fp64 (double rounding could differ only in
            # near-tie cases; the comparison below allows one ulp)
            out[i, j] = np.float32(float(r))
    return out


def test_against_exact_rational_arithmetic():
    rng = np.random.default_rng(25)
    for M, N, K in [(1, 1, 1), (2, 3, 4), (5, 4, 7), (3, 3, 33)]:
        A = rng.uniform(-1, 1, (M, K)).astype(np.float32)
        B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
        C0 = rng.uniform(-1, 1, (M, N)).astype(np.float32)
        for tA, tB in ALL_T:
            got = run(A, B, C0, 1.5, -0.3, tA, tB, CM, scalar=True)
            want = exact_reference(A, B, C0, 1.5, -0.3)
            ulp = np.spacing(np.abs(want))
            assert np.all(np.abs(got.astype(np.float64) - want.astype(np.float64)) <= ulp)


def test_against_numpy_fp64_matmul():
    # special case "no padding, plain matrices": the library routine is numpy's fp64 matmul
    for (M, N, K), seed in zip([(64, 64, 64), (130, 67, 515), (257, 3, 1024)], (26, 27, 28)):
        A, B, C0 = rnd((M, K), seed), rnd((K, N), seed + 100), rnd((M, N), seed + 200)
        got = run(A, B, C0, 1.0, 0.5).astype(np.float64)
        want = A.astype(np.float64) @ B.astype(np.float64) + 0.5 * C0.astype(np.float64)
        # fp64 summation-order differences (<= K * 2^-53 relative to sum |a b|) plus one fp32 rounding
        bound = np.spacing(np.abs(want).astype(np.float32)).astype(np.float64) * 0.5 + K * 2.0 ** -52
        assert np.all(np.abs(got - want) <= bound)


@pytest.mark.parametrize("layout", ALL_L)
def test_fast_loop_order_equals_scalar_loops_on_all_tiny_shapes(layout):
    # the interchanged / threaded loops must be bit-identical to the three nested loops
    dims = (1, 2, 3, 5, 8, 17)
    rng = np.random.default_rng(29)
    for M, N, K in itertools.product(dims, dims, dims):
        A = rng.uniform(-1, 1, (M, K)).astype(np.float32)
        B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
        C0 = rng.uniform(-1, 1, (M, N)).astype(np.float32)
        for tA, tB in ALL_T:
            pad = tuple(int(x) for x in rng.integers(0, 3, 3))
            f = run(A, B, C0, 1.1, 0.6, tA, tB, layout, pad=pad)
            s = run(A, B, C0, 1.1, 0.6, tA, tB, layout, pad=pad, scalar=True)
            assert np.array_equal(f, s), (M, N, K, tA, tB, pad)


def test_fast_equals_scalar_medium_and_elements_entry():
    case = wl.GemmCase(150, 77, 260, TR, TR, 0.7, -0.4, lda=263, ldb=80, ldc=155, seed=31)
    A, B, C0 = wl.make_operands(case)
    c1, c2 = C0.copy(), C0.copy()
    args = (CM, TR, TR, 150, 77, 260, 0.7, A, 263, B, 80, -0.4)
    assert go.sgemm(*args, c1, 155) == 0
    assert go.sgemm(*args, c2, 155, scalar=True) == 0
    assert np.array_equal(c1, c2, equal_nan=True)
    assert not np.any(np.isnan(wl.matrix_view(c1, CM, (150, 77), 155)))  # NaN padding of A, B never read
    ii = np.array([0, 149, 75, 3], np.int64)
    jj = np.array([0, 76, 40, 76], np.int64)
    e = go.sgemm_elements(*args, C0, 155, ii, jj)
    assert np.array_equal(e, wl.matrix_view(c1, CM, (150, 77), 155)[ii, jj])
    with pytest.raises(ValueError):
        go.sgemm_elements(*args, C0, 155, np.array([150]), np.array([0]))


def test_tolerance_formula():
    t = go.tolerance(1000, 2.0, 0.5, 0.5, np.array([4.0, -8.0]))
    assert np.allclose(t, [1e-3 + 2e-6, 1e-3 + 4e-6])
