"""Exact rational arithmetic helpers for pinning the oracle (tests only).

Everything here works on *logical* matrices given as lists of lists of
``fractions.Fraction``; it is written as dot products over explicit index
ranges (row, column, inner index), independently of the oracle's loops, and is
only usable on tiny inputs.
"""
from fractions import Fraction

import numpy as np


def frac(a):
    """numpy 2-D array (any storage order) -> list of lists of exact Fractions."""
    return [[Fraction(float(a[i, j])) for j in range(a.shape[1])] for i in range(a.shape[0])]


def transpose(X):
    if not X:
        return []
    return [[X[i][j] for i in range(len(X))] for j in range(len(X[0]))]


def matmul(X, Y):
    m, k, n = len(X), len(Y), len(Y[0]) if Y else 0
    return [[sum((X[i][l] * Y[l][j] for l in range(k)), Fraction(0)) for j in range(n)] for i in range(m)]


def abs_matmul(X, Y):
    m, k, n = len(X), len(Y), len(Y[0]) if Y else 0
    return [[sum((abs(X[i][l] * Y[l][j]) for l in range(k)), Fraction(0)) for j in range(n)] for i in range(m)]


def triangle(A, lower, unit):
    """The triangular matrix an (uplo, diag) pair makes of square A; other entries exact zero."""
    n = len(A)
    out = [[Fraction(0)] * n for _ in range(n)]
    for r in range(n):
        for c in range(n):
            if r == c:
                out[r][c] = Fraction(1) if unit else A[r][c]
            elif (r > c) == lower:
                out[r][c] = A[r][c]
    return out


def solve_triangular(Tm, Bm):
    """Exact X with Tm X = Bm for a triangular (either kind) nonsingular Tm, by elimination."""
    n = len(Tm)
    ncol = len(Bm[0])
    lower = all(Tm[r][c] == 0 for r in range(n) for c in range(n) if c > r)
    X = [[Fraction(0)] * ncol for _ in range(n)]
    rows = range(n) if lower else range(n - 1, -1, -1)
    for j in range(ncol):
        for i in rows:
            s = Bm[i][j]
            for l in range(n):
                if l != i:
                    s -= Tm[i][l] * X[l][j]
            X[i][j] = s / Tm[i][i]
    return X


def to_float(X):
    return np.array([[float(v) for v in row] for row in X], dtype=np.float64).reshape(len(X), len(X[0]) if X else 0)
