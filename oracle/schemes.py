"""Bilinear schemes <m,k,n;R;U,V,W> for the oracle.  TEST INFRASTRUCTURE ONLY.

A scheme is written the way a textbook prints it: R products of a signed sum of
blocks of A with a signed sum of blocks of B, and one signed sum of products per
block of C.  `from_formulas` turns that text into the coefficient tensors of the
paper's LCMA tuple (Sec. 2.1): U[r,i,l] multiplies A_{i,l} in the r-th left
operand (Eq. 3), V[r,l,j] multiplies B_{l,j} in the r-th right operand (Eq. 4),
W[r,i,j] multiplies the r-th product in C_{i,j} (Eq. 6).

Nothing here is shared with the GPU library: it carries its own tables.
"""
from __future__ import annotations

import re
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Scheme:
    m: int
    k: int
    n: int
    R: int
    U: np.ndarray  # (R, m, k) int32
    V: np.ndarray  # (R, k, n) int32
    W: np.ndarray  # (R, m, n) int32
    name: str = ""

    def nnz(self):
        return (int(np.count_nonzero(self.U)), int(np.count_nonzero(self.V)),
                int(np.count_nonzero(self.W)))


_TERM = re.compile(r"([+-]?)\s*([a-zA-Z]+)(\d+)")


def _signed_terms(expr: str):
    """'a11 + a22 - b3' -> [(+1,'a','11'), (+1,'a','22'), (-1,'b','3')]."""
    expr = expr.strip()
    out, pos = [], 0
    while pos < len(expr):
        mt = _TERM.match(expr, pos)
        if not mt:
            raise ValueError(f"cannot parse {expr!r} at {pos}")
        out.append((-1 if mt.group(1) == "-" else 1, mt.group(2), mt.group(3)))
        pos = mt.end()
        while pos < len(expr) and expr[pos].isspace():
            pos += 1
    return out


def from_formulas(m: int, k: int, n: int, products: list[str], outputs: list[str],
                  name: str = "") -> Scheme:
    """products[r] = '(sum of a<i><l>) * (sum of b<l><j>)'; outputs = 'c<i><j> = sum of h<r>'.

    Block indices are the paper's 1-based single digits; product numbers are 1-based.
    """
    R = len(products)
    U = np.zeros((R, m, k), np.int32)
    V = np.zeros((R, k, n), np.int32)
    W = np.zeros((R, m, n), np.int32)
    for r, text in enumerate(products):
        left, right = text.split("*")
        left = left.strip().strip("()")
        right = right.strip().strip("()")
        for s, sym, idx in _signed_terms(left):
            assert sym == "a" and len(idx) == 2
            U[r, int(idx[0]) - 1, int(idx[1]) - 1] += s
        for s, sym, idx in _signed_terms(right):
            assert sym == "b" and len(idx) == 2
            V[r, int(idx[0]) - 1, int(idx[1]) - 1] += s
    seen = set()
    for text in outputs:
        lhs, rhs = text.split("=")
        (s0, sym0, idx0), = _signed_terms(lhs)
        assert sym0 == "c" and s0 == 1 and len(idx0) == 2
        i, j = int(idx0[0]) - 1, int(idx0[1]) - 1
        seen.add((i, j))
        for s, sym, idx in _signed_terms(rhs):
            assert sym == "h"
            W[int(idx) - 1, i, j] += s
    assert len(seen) == m * n, "every block of C needs a formula"
    return Scheme(m, k, n, R, U, V, W, name)


def classical(m: int, k: int, n: int) -> Scheme:
    """The definition of block matrix multiplication as a scheme of rank m*k*n."""
    R = m * k * n
    U = np.zeros((R, m, k), np.int32)
    V = np.zeros((R, k, n), np.int32)
    W = np.zeros((R, m, n), np.int32)
    r = 0
    for i in range(m):
        for j in range(n):
            for l in range(k):
                U[r, i, l] = 1
                V[r, l, j] = 1
                W[r, i, j] = 1
                r += 1
    return Scheme(m, k, n, R, U, V, W, f"classical{m}{k}{n}")


def strassen() -> Scheme:
    """Strassen's <2,2,2;7> (paper Sec. 2.1; numbering in which C11 = H1+H4-H5+H7)."""
    products = [
        "(a11 + a22) * (b11 + b22)",
        "(a21 + a22) * (b11)",
        "(a11) * (b12 - b22)",
        "(a22) * (b21 - b11)",
        "(a11 + a12) * (b22)",
        "(a21 - a11) * (b11 + b12)",
        "(a12 - a22) * (b21 + b22)",
    ]
    outputs = [
        "c11 = h1 + h4 - h5 + h7",
        "c12 = h3 + h5",
        "c21 = h2 + h4",
        "c22 = h1 - h2 + h3 + h6",
    ]
    return from_formulas(2, 2, 2, products, outputs, "strassen")


def laderman() -> Scheme:
    """Laderman's <3,3,3;23> (named in paper Sec. 2.1)."""
    products = [
        "(a11 + a12 + a13 - a21 - a22 - a32 - a33) * (b22)",
        "(a11 - a21) * (-b12 + b22)",
        "(a22) * (-b11 + b12 + b21 - b22 - b23 - b31 + b33)",
        "(-a11 + a21 + a22) * (b11 - b12 + b22)",
        "(a21 + a22) * (-b11 + b12)",
        "(a11) * (b11)",
        "(-a11 + a31 + a32) * (b11 - b13 + b23)",
        "(-a11 + a31) * (b13 - b23)",
        "(a31 + a32) * (-b11 + b13)",
        "(a11 + a12 + a13 - a22 - a23 - a31 - a32) * (b23)",
        "(a32) * (-b11 + b13 + b21 - b22 - b23 - b31 + b32)",
        "(-a13 + a32 + a33) * (b22 + b31 - b32)",
        "(a13 - a33) * (b22 - b32)",
        "(a13) * (b31)",
        "(a32 + a33) * (-b31 + b32)",
        "(-a13 + a22 + a23) * (b23 + b31 - b33)",
        "(a13 - a23) * (b23 - b33)",
        "(a22 + a23) * (-b31 + b33)",
        "(a12) * (b21)",
        "(a23) * (b32)",
        "(a21) * (b13)",
        "(a31) * (b12)",
        "(a33) * (b33)",
    ]
    outputs = [
        "c11 = h6 + h14 + h19",
        "c12 = h1 + h4 + h5 + h6 + h12 + h14 + h15",
        "c13 = h6 + h7 + h9 + h10 + h14 + h16 + h18",
        "c21 = h2 + h3 + h4 + h6 + h14 + h16 + h17",
        "c22 = h2 + h4 + h5 + h6 + h20",
        "c23 = h14 + h16 + h17 + h18 + h21",
        "c31 = h6 + h7 + h8 + h11 + h12 + h13 + h14",
        "c32 = h12 + h13 + h14 + h15 + h22",
        "c33 = h6 + h7 + h8 + h9 + h23",
    ]
    return from_formulas(3, 3, 3, products, outputs, "laderman")


def kronecker(outer: Scheme, inner: Scheme, name: str = "") -> Scheme:
    """One flat scheme equal to applying `inner` to every block product of `outer`.

    Flat indices: r = r1*R2 + r2, i = i1*m2 + i2, l = l1*k2 + l2, j = j1*n2 + j2,
    and each coefficient is the product of the two levels' coefficients.  This is
    the reading of the paper's "two-level recursive Strassen <4,4,4>, R=49".
    """
    m, k, n, R = outer.m * inner.m, outer.k * inner.k, outer.n * inner.n, outer.R * inner.R
    U = np.einsum("ail,bjm->abijlm", outer.U, inner.U).reshape(R, m, k)
    V = np.einsum("ail,bjm->abijlm", outer.V, inner.V).reshape(R, k, n)
    W = np.einsum("ail,bjm->abijlm", outer.W, inner.W).reshape(R, m, n)
    return Scheme(m, k, n, R, U.astype(np.int32), V.astype(np.int32), W.astype(np.int32),
                  name or f"{outer.name}x{inner.name}")


def strassen2() -> Scheme:
    s = strassen()
    return kronecker(s, s, "strassen2")


def strassen_wide() -> Scheme:
    """A rectangular scheme <2,2,4;14>: Strassen with every block column of B and C cut in two
    (Strassen composed with the definition of a 1 x 1 by 1 x 2 block product)."""
    return kronecker(strassen(), classical(1, 1, 2), "strassen_wide")


def winograd() -> Scheme:
    """The Winograd form of Strassen's algorithm, <2,2,2;7> with 15 additions when common sums are
    shared (S1 = a21 + a22, S2 = S1 - a11, S3 = a11 - a21, S4 = a12 - S2; T1 = b12 - b11, T2 = b22 - T1,
    T3 = b22 - b12, T4 = T2 - b21), written out flat here.  Not one of the paper's named schemes: it
    exercises the generator's sharing of common sums."""
    products = [
        "(a11) * (b11)",
        "(a12) * (b21)",
        "(a12 - a21 - a22 + a11) * (b22)",                      # S4 * b22
        "(a22) * (b22 - b12 + b11 - b21)",                      # a22 * T4
        "(a21 + a22) * (b12 - b11)",                            # S1 * T1
        "(a21 + a22 - a11) * (b22 - b12 + b11)",                # S2 * T2
        "(a11 - a21) * (b22 - b12)",                            # S3 * T3
    ]
    outputs = [
        "c11 = h1 + h2",
        "c12 = h1 + h6 + h5 + h3",
        "c21 = h1 + h6 + h7 - h4",
        "c22 = h1 + h6 + h7 + h5",
    ]
    return from_formulas(2, 2, 2, products, outputs, "winograd")


def by_name(name: str) -> Scheme:
    return {"strassen": strassen, "strassen2": strassen2, "laderman": laderman,
            "strassen_wide": strassen_wide, "winograd": winograd}[name]()


def to_text(s: Scheme) -> str:
    """Scheme text format: 'm k n R', then R rows of U, R rows of V, R rows of W."""
    lines = [f"{s.m} {s.k} {s.n} {s.R}"]
    for T in (s.U, s.V, s.W):
        for r in range(s.R):
            lines.append(" ".join(str(int(x)) for x in T[r].reshape(-1)))
    return "\n".join(lines) + "\n"
