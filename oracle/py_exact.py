"""Exact brute-force matrix product for tiny sizes -- TEST INFRASTRUCTURE ONLY.

Evaluates C[i][j] = sum_p A[i][p] * B[p][j] (matmul of Sec. 5.2 of the paper) in exact
rational arithmetic with pure-Python loops, in the order j, i, p (deliberately not the
order of the C oracle).  fp32/fp64 inputs convert to Fractions without error, so the
result is the mathematically exact product; it pins the C oracle on small cases.
"""
from __future__ import annotations

from fractions import Fraction


def matmul_exact(a, b, n=None):
    """a: m x k nested sequence, b: k x n nested sequence -> m x n list of Fractions.

    n must be given when k == 0 (an empty b carries no column count)."""
    m = len(a)
    k = len(b)
    if n is None:
        n = len(b[0]) if k else 0
    if any(len(row) != k for row in a):
        raise ValueError("inner dimensions differ")
    c = [[Fraction(0) for _ in range(n)] for _ in range(m)]
    for j in range(n):
        for i in range(m):
            acc = Fraction(0)
            for p in range(k):
                acc += Fraction(a[i][p]) * Fraction(b[p][j])
            c[i][j] = acc
    return c


def to_float_grid(c):
    """Round each exact entry to the nearest fp64 (Fraction -> float is correctly rounded)."""
    return [[float(x) for x in row] for row in c]
