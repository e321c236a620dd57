"""Exact (E_X, E_W, D) triples used as fixtures -- TEST INFRASTRUCTURE ONLY.

The paper names, but does not print, the rank-49 "Strassen's construction" for
4x4 tiles (appendix on initialising the tile-level optimisation; caption of the
speed-up figure: r=49 imitates exact multiplication).  It is built here from the
textbook seven-product scheme for 2x2 blocks applied twice.  All matrices are
r x t^2 for the row-major tile vectorisation vec(T)[a*t+b] = T[a][b].
"""
from __future__ import annotations

import numpy as np

# Seven-product scheme for [[A11,A12],[A21,A22]] * [[B11,B12],[B21,B22]],
# columns ordered (11, 12, 21, 22).
#   M1=(A11+A22)(B11+B22)  M2=(A21+A22)B11   M3=A11(B12-B22)   M4=A22(B21-B11)
#   M5=(A11+A12)B22        M6=(A21-A11)(B11+B12)               M7=(A12-A22)(B21+B22)
#   C11=M1+M4-M5+M7  C12=M3+M5  C21=M2+M4  C22=M1-M2+M3+M6
_U = np.array([[1, 0, 0, 1],
               [0, 0, 1, 1],
               [1, 0, 0, 0],
               [0, 0, 0, 1],
               [1, 1, 0, 0],
               [-1, 0, 1, 0],
               [0, 1, 0, -1]], dtype=np.float64)      # coefficients of A in M_p
_V = np.array([[1, 0, 0, 1],
               [1, 0, 0, 0],
               [0, 1, 0, -1],
               [-1, 0, 1, 0],
               [0, 0, 0, 1],
               [1, 1, 0, 0],
               [0, 0, 1, 1]], dtype=np.float64)       # coefficients of B in M_p
_Z = np.array([[1, 0, 0, 1],
               [0, 0, 1, -1],
               [0, 1, 0, 1],
               [1, 0, 1, 0],
               [-1, 1, 0, 0],
               [0, 0, 0, 1],
               [1, 0, 0, 0]], dtype=np.float64)       # coefficient of M_p in (C11,C12,C21,C22)


def strassen_2x2():
    """(E_X, E_W, D), each 7 x 4: exact 2x2 product with t=2, r=7."""
    return _U.copy(), _V.copy(), _Z.copy()


def _nest(F):
    """Two-level factor matrix for 4x4 tiles.

    Row 7*p + p' ; column of the row-major 4x4 vec: 4*(2*bi+si) + (2*bj+sj), where
    (bi,bj) picks the 2x2 block and (si,sj) the entry inside it.  A Kronecker
    product would order columns (block, inner); the row-major vec interleaves them.
    """
    out = np.zeros((49, 16))
    for p in range(7):
        for pp in range(7):
            for bi in range(2):
                for bj in range(2):
                    for si in range(2):
                        for sj in range(2):
                            col = 4 * (2 * bi + si) + (2 * bj + sj)
                            out[7 * p + pp, col] = F[p, 2 * bi + bj] * F[pp, 2 * si + sj]
    return out


def strassen_4x4():
    """(E_X, E_W, D), each 49 x 16: the seven-product scheme applied at both levels."""
    return _nest(_U), _nest(_V), _nest(_Z)


def trivial(t: int = 4):
    """Rank-t^3 basis of the schoolbook product: row (a,l,b) multiplies X[a,l]*W[l,b]
    and adds it to C[a,b]."""
    r, tt = t ** 3, t * t
    E_X = np.zeros((r, tt))
    E_W = np.zeros((r, tt))
    D = np.zeros((r, tt))
    for a in range(t):
        for l in range(t):
            for b in range(t):
                p = (a * t + l) * t + b
                E_X[p, a * t + l] = 1.0
                E_W[p, l * t + b] = 1.0
                D[p, a * t + b] = 1.0
    return E_X, E_W, D
