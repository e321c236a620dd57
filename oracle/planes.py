"""Second oracle formulation: the three-step plane algorithm -- TEST INFRASTRUCTURE ONLY.

Follows Algorithm 1 ("STL pseudo-code") and Claim 3.4 in the paper's order:
(i) encode every X tile with E_X, (ii) one ordinary matrix product per plane p,
(iii) decode every output tile with D^T.  numpy's fp64 ``matmul`` is the library
primitive used for each step; nothing else is blocked or fused.  This is written
independently of ``stl_oracle.c`` (which evaluates Eq. (2) tile by tile) and the
two are required to agree (tests/test_oracle_pins.py).

The gradients are the chain rule through those three linear steps (the paper
gives no formulas; Section "Strassen-Tile Operator" only asserts they exist).
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf


def tiles(A, t: int = 4):
    """Tiled view of Section "Strassen-Tile Operator": (a, b) matrix -> (a/t, b/t, t^2),
    each tile vectorised row-major."""
    A = np.asarray(A, dtype=np.float64)
    a, b = A.shape
    if a % t or b % t:
        raise ValueError("matrix dimensions must be divisible by t")
    return A.reshape(a // t, t, b // t, t).transpose(0, 2, 1, 3).reshape(a // t, b // t, t * t)


def untile(T, t: int = 4):
    """Inverse of :func:`tiles`."""
    T = np.asarray(T, dtype=np.float64)
    A, B, tt = T.shape
    assert tt == t * t
    return T.reshape(A, B, t, t).transpose(0, 2, 1, 3).reshape(A * t, B * t)


def encode(A, E, t: int = 4):
    """Step (i): planes[p] = p-th entry of every encoded tile.  Returns (r, a/t, b/t)."""
    hat = tiles(A, t) @ np.asarray(E, dtype=np.float64).T          # hatX = X @ E^T
    return np.ascontiguousarray(hat.transpose(2, 0, 1))


def plane_products(Xhat, What):
    """Step (ii), Claim 3.4: Yhat[p] = Xhat[p] @ What[p], r independent products."""
    return np.matmul(np.asarray(Xhat, dtype=np.float64), np.asarray(What, dtype=np.float64))


def decode(Yhat, D, t: int = 4):
    """Step (iii): every output tile is D^T applied to its r encoded entries."""
    Y = np.asarray(Yhat, dtype=np.float64).transpose(1, 2, 0) @ np.asarray(D, dtype=np.float64)
    return untile(Y, t)


def forward(X, What, E_X, D, t: int = 4, return_yhat: bool = False):
    Xhat = encode(X, E_X, t)
    Yhat = plane_products(Xhat, What)
    C = decode(Yhat, D, t)
    return (C, Yhat) if return_yhat else C


def backward(X, What, E_X, D, dC, t: int = 4):
    """Gradients of <dC, C> w.r.t. X, What, E_X, D (same order as oracle.backward)."""
    E_X = np.asarray(E_X, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64)
    What = np.asarray(What, dtype=np.float64)
    x = tiles(X, t)                                   # (M, K, t^2)
    dc = tiles(dC, t)                                 # (M, N, t^2)
    Xhat = encode(X, E_X, t)                          # (r, M, K)
    Yhat = plane_products(Xhat, What)                 # (r, M, N)
    dD = np.tensordot(Yhat, dc, axes=([1, 2], [0, 1]))             # (r, t^2)
    dYhat = np.ascontiguousarray((dc @ D.T).transpose(2, 0, 1))    # (r, M, N)
    dXhat = np.matmul(dYhat, What.transpose(0, 2, 1))              # (r, M, K)
    dWhat = np.matmul(Xhat.transpose(0, 2, 1), dYhat)              # (r, K, N)
    dX = untile(dXhat.transpose(1, 2, 0) @ E_X, t)
    dE_X = np.tensordot(dXhat, x, axes=([1, 2], [0, 1]))           # (r, t^2)
    return dX, dWhat, dE_X, dD


def encode_weight_backward(W, E_W, dWhat, t: int = 4):
    """Gradients through the weight encoding What[p,L,J] = sum_q E_W[p,q] w[L,J,q] (the "true encoding" of the
    paper's plane definition, as opposed to training What directly): with dWhat the gradient of the loss w.r.t.
    the encoded planes,
        dw[L,J,q]  = sum_p E_W[p,q] dWhat[p,L,J]          (a decode of dWhat with E_W as decoder)  -> dW (k x n)
        dE_W[p,q]  = sum_{L,J} dWhat[p,L,J] w[L,J,q].
    The paper only states that these gradients exist (Section "Strassen-Tile Operator"); this is the chain rule."""
    dWhat = np.asarray(dWhat, dtype=np.float64)
    dW = decode(dWhat, E_W, t)
    dE_W = np.tensordot(dWhat, tiles(W, t), axes=([1, 2], [0, 1]))
    return dW, dE_W


def gelu(h):
    """Exact (erf) GELU, used between the two layers of the MLP-shaped pair."""
    h = np.asarray(h, dtype=np.float64)
    return 0.5 * h * (1.0 + erf(h / np.sqrt(2.0)))


def recode(Yhat, D, E_next, activation: str | None = "gelu", t: int = 4):
    """Inter-layer step of Algorithm 2 (its Steps 3 and 1 taken together): decode the encoded output of
    one layer with D, apply the activation entrywise (``None``: the paper's purely linear case, where the
    step collapses to one (r_next x r) map per tile), encode the result with the next layer's E_X.
    Output tile (I, J) of the first layer is input tile (I, L = J) of the second."""
    H = decode(Yhat, D, t)
    if activation == "gelu":
        H = gelu(H)
    elif activation is not None:
        raise ValueError("activation must be 'gelu' or None")
    return encode(H, E_next, t)


def mlp_pair(X, What1, E_X1, D1, What2, E_X2, D2, t: int = 4, activation: str | None = "gelu"):
    """STL up-projection, activation (exact GELU, or none), STL down-projection; fp64 end to end.
    Written as Algorithm 2 does it: the hidden activation only exists between decode and encode."""
    Yhat1 = plane_products(encode(X, E_X1, t), What1)
    Xhat2 = recode(Yhat1, D1, E_X2, activation, t)
    return decode(plane_products(Xhat2, What2), D2, t)
