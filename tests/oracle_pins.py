"""Pins for a matrix-product routine, written so they can be run against the C oracle
and against deliberately wrong variants of it (see test_oracle_pins.py).

Every pin takes ``gemm(a, b) -> fp64 array``: a, b are fp32 numpy matrices (m,k),(k,n).
Each pin raises AssertionError when the routine disagrees with what the definition
C[i][j] = sum_p A[i][p] B[p][j] (matmul, Sec. 5.2 of the paper) or plain mathematics
fixes.  None of them re-derives the expected value by calling the routine under test
or by retyping its loop; expected values are closed forms, exact rational brute force,
an independent library product, or algebraic identities.
"""
from __future__ import annotations

import numpy as np

from oracle import py_exact
from paper_1904_03383_amd import inputgen as ig


def pin_identity(gemm):
    b = ig.uniform(21, (9, 13))
    a = ig.uniform(22, (11, 9))
    assert np.array_equal(gemm(np.eye(9, dtype=np.float32), b), b.astype(np.float64))
    assert np.array_equal(gemm(a, np.eye(9, dtype=np.float32)), a.astype(np.float64))


def pin_all_ones(gemm):
    for m, n, k in [(3, 5, 1), (4, 2, 7), (2, 3, 1000), (1, 1, 1 << 20)]:
        c = gemm(np.ones((m, k), np.float32), np.ones((k, n), np.float32))
        assert c.shape == (m, n) and np.all(c == float(k)), (m, n, k)


def pin_empty_k(gemm):
    c = gemm(np.zeros((3, 0), np.float32), np.zeros((0, 4), np.float32))
    assert c.shape == (3, 4) and np.all(c == 0.0)


def pin_exact_bruteforce(gemm):
    """All shapes m,n,k in 0..4 plus a few larger ones; integer and 2^-23-grid inputs.

    For grid inputs every product is a multiple of 2^-46 bounded by 1, so the sum of
    k <= 128 of them has at most 53 significant bits: an fp64 running sum is exact and
    must equal the rational result exactly.
    """
    shapes = [(m, n, k) for m in range(0, 5) for n in range(0, 5) for k in range(0, 5)]
    shapes += [(5, 6, 7), (2, 9, 33), (7, 3, 64)]
    seed = 100
    for (m, n, k) in shapes:
        for gen in (ig.small_int, ig.uniform):
            seed += 1
            a = gen(seed, (m, k))
            b = gen(seed + 5000, (k, n))
            want = py_exact.to_float_grid(py_exact.matmul_exact(a.tolist(), b.tolist(), n))
            got = gemm(a, b)
            assert got.shape == (m, n)
            if m and n:
                assert np.array_equal(got, np.array(want, dtype=np.float64).reshape(m, n)), (m, n, k, gen.__name__)


def pin_closed_forms(gemm):
    # rank one: A[i][p] = u_i, B[p][j] = v_j  =>  C = k * u_i * v_j
    u = np.array([1, -2, 3, 0, 4], np.float32)
    v = np.array([2, 1, -3, 5], np.float32)
    k = 37
    c = gemm(np.repeat(u[:, None], k, 1), np.repeat(v[None, :], k, 0))
    assert np.array_equal(c, k * np.outer(u, v).astype(np.float64))
    # A[i][p] = p + 1, B = 1  =>  C = k (k + 1) / 2
    k = 300
    a = np.tile(np.arange(1, k + 1, dtype=np.float32), (3, 1))
    assert np.all(gemm(a, np.ones((k, 2), np.float32)) == k * (k + 1) / 2)
    # A[i][p] = (i + 1) [p == 2], B[p][j] = (p + 1) * 10 + j  => picks row 2 of B scaled by i + 1;
    # distinguishes A[i][p] from A[p][i] and B[p][j] from B[j][p] on non-symmetric data
    a = np.zeros((4, 5), np.float32)
    a[:, 2] = np.arange(1, 5)
    b = (np.arange(1, 6, dtype=np.float32)[:, None] * 10 + np.arange(6, dtype=np.float32)[None, :])
    want = np.arange(1, 5, dtype=np.float64)[:, None] * (30 + np.arange(6, dtype=np.float64))[None, :]
    assert np.array_equal(gemm(a, b), want)
    # permutation matrix: rows of B permuted, bit exact
    perm = np.array([3, 0, 4, 1, 2])
    p = np.zeros((5, 5), np.float32)
    p[np.arange(5), perm] = 1
    bb = ig.uniform(31, (5, 7))
    assert np.array_equal(gemm(p, bb), bb[perm].astype(np.float64))
    # diagonal power-of-two scaling is exact
    e = np.array([-3, 0, 5, 1], dtype=np.float64)
    d = np.diag(2.0 ** e).astype(np.float32)
    bb = ig.uniform(32, (4, 6))
    assert np.array_equal(gemm(d, bb), bb.astype(np.float64) * (2.0 ** e)[:, None])
    # signs: (-A) B = -(A B) exactly and a single negative entry gives a negative product
    assert gemm(np.array([[-2.0]], np.float32), np.array([[3.0]], np.float32))[0, 0] == -6.0


def pin_invariants(gemm):
    a = ig.uniform(41, (17, 29))
    b = ig.uniform(42, (29, 23))
    c = gemm(a, b)
    # transpose identity: (A B)^T = B^T A^T; the same products in the same p order => identical bits
    ct = gemm(np.ascontiguousarray(b.T), np.ascontiguousarray(a.T))
    assert np.array_equal(c, ct.T)
    # K additivity (k = 29 <= 128 grid inputs: all sums exact, so equality is exact)
    k1 = 12
    c1 = gemm(np.ascontiguousarray(a[:, :k1]), np.ascontiguousarray(b[:k1]))
    c2 = gemm(np.ascontiguousarray(a[:, k1:]), np.ascontiguousarray(b[k1:]))
    assert np.array_equal(c, c1 + c2)
    # linearity in A on operands whose sum is exact in fp32, and homogeneity under 2^e scaling
    a1 = ig.small_int(43, (17, 29))
    a2 = ig.small_int(44, (17, 29)) * np.float32(0.125)
    assert np.array_equal(gemm(a1 + a2, b), gemm(a1, b) + gemm(a2, b))
    assert np.array_equal(gemm(a * np.float32(4), b), 4.0 * c)
    # each output depends only on its own row of A and column of B
    a3 = a.copy()
    a3[5] = 0
    c3 = gemm(a3, b)
    assert np.all(c3[5] == 0) and np.array_equal(np.delete(c3, 5, 0), np.delete(c, 5, 0))


def pin_library_dgemm(gemm, size=(96, 80, 300)):
    """Independent library product on fp64-cast inputs (never the oracle itself)."""
    m, n, k = size
    for gen, seed in ((ig.uniform, 51), (ig.normal, 52)):
        a = gen(seed, (m, k))
        b = gen(seed + 1, (k, n))
        ref = a.astype(np.float64) @ b.astype(np.float64)
        s = np.abs(a).astype(np.float64) @ np.abs(b).astype(np.float64)
        assert np.all(np.abs(gemm(a, b) - ref) <= 1e-12 * s)


def pin_freivalds(gemm, m=300, n=280, k=520, reps=4):
    """Freivalds' check: C x == A (B x) for random sign vectors x, O(n^2) work, different code path."""
    a = ig.normal(61, (m, k))
    b = ig.normal(62, (k, n))
    c = gemm(a, b)
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    for r in range(reps):
        x = np.where(ig.raw_bits(63 + r, n) >> np.uint64(63), 1.0, -1.0)
        lhs = c @ x
        rhs = a64 @ (b64 @ x)
        bound = 1e-10 * (np.abs(a64) @ (np.abs(b64) @ np.ones(n)))
        assert np.all(np.abs(lhs - rhs) <= bound)


ALL_PINS = [pin_identity, pin_all_ones, pin_empty_k, pin_exact_bruteforce, pin_closed_forms,
            pin_invariants, pin_library_dgemm, pin_freivalds]


# ---- axpy (Sec. 5.2: z = alpha.x + y) ------------------------------------------------------------

def axpy_pin_special_values(axpy):
    x = ig.uniform(81, (1000,))
    y = ig.uniform(82, (1000,))
    assert np.array_equal(axpy(0.0, x, y), y.astype(np.float64))                    # alpha = 0
    assert np.array_equal(axpy(1.0, x, np.zeros_like(x)), x.astype(np.float64))     # y = 0, alpha = 1
    assert np.all(axpy(-1.0, x, x) == 0.0)                                          # x - x
    assert np.array_equal(axpy(1.0, x, y), axpy(1.0, y, x))                         # commutes at alpha = 1
    assert axpy(3.0, np.array([2.0], np.float32), np.array([-1.0], np.float32))[0] == 5.0
    assert axpy(-0.5, np.array([4.0], np.float32), np.array([1.0], np.float32))[0] == -1.0


def axpy_pin_exact_cases(axpy):
    xi = ig.small_int(83, (5000,), -100, 100)
    yi = ig.small_int(84, (5000,), -1000, 1000)
    got = axpy(7.0, xi, yi)
    want = [7 * int(a) + int(b) for a, b in zip(xi.tolist(), yi.tolist())]          # integer arithmetic
    assert got.tolist() == [float(v) for v in want]
    # power-of-two alpha: alpha*x is an exact scaling, and on the 2^-23 grid the sum is exact in fp64
    x = ig.uniform(85, (4096,))
    y = ig.uniform(86, (4096,))
    from fractions import Fraction
    got = axpy(0.25, x, y)
    for i in (0, 1, 17, 4095):
        assert Fraction(got[i]) == Fraction(1, 4) * Fraction(float(x[i])) + Fraction(float(y[i]))


def axpy_pin_elementwise_and_empty(axpy):
    x = ig.normal(87, (257,))
    y = ig.normal(88, (257,))
    z = axpy(1.5, x, y)
    x2 = x.copy()
    x2[100] = 0.0
    z2 = axpy(1.5, x2, y)
    assert z2[100] == float(y[100]) and np.array_equal(np.delete(z, 100), np.delete(z2, 100))
    assert axpy(2.0, x[:0], y[:0]).shape == (0,)
    assert np.array_equal(axpy(2.0, x, y)[::-1], axpy(2.0, x[::-1].copy(), y[::-1].copy()))   # order free


AXPY_PINS = [axpy_pin_special_values, axpy_pin_exact_cases, axpy_pin_elementwise_and_empty]
