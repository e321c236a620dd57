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


# ------------------------------------------------------------------ both operands encoded at run time
def aa_forward(A, B, E_A, E_B, D, nbatch: int = 1, t: int = 4, b_transposed: bool = False):
    """STL of two activations (the attention products of the Class-1 discussion, where neither operand is a
    weight): the second operand is encoded at run time with E_B exactly as a weight is with E_W,
        Bhat[p, L, J] = sum_q E_B[p, q] b[L, J, q],   C = decode_D( encode_{E_A}(A)[p] @ Bhat[p] ).
    `nbatch` independent products (heads x images) are stacked along the rows: A is (nbatch*m, k), B is
    (nbatch*k, n), C is (nbatch*m, n); the bases are shared by the whole batch.
    b_transposed: B holds the transposes, (nbatch*n, k) -- the Q K^T case with K stored tokens x width; the
    operator is applied to B_b^T."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    m, rb = A.shape[0] // nbatch, B.shape[0] // nbatch
    k = A.shape[1]
    if A.shape[0] != nbatch * m or B.shape[0] != nbatch * rb or (B.shape[1] if b_transposed else rb) != k:
        raise ValueError("stacked operands do not match nbatch")
    out = []
    for b in range(nbatch):
        Bb = B[b * rb:(b + 1) * rb]
        Bhat = encode(Bb.T if b_transposed else Bb, E_B, t)
        out.append(forward(A[b * m:(b + 1) * m], Bhat, E_A, D, t))
    return np.concatenate(out, axis=0)


def aa_backward(A, B, E_A, E_B, D, dC, nbatch: int = 1, t: int = 4, b_transposed: bool = False):
    """Gradients of sum_b <dC_b, C_b> for :func:`aa_forward`: (dA, dB, dE_A, dE_B, dD).  Chain rule through the
    three steps for A (as for an activation) and through the run-time encoding for B (as for a weight); the
    shared bases collect the sum over the batch.  dB has the shape B was given in."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    dC = np.asarray(dC, dtype=np.float64)
    m, rb = A.shape[0] // nbatch, B.shape[0] // nbatch
    dA, dB = np.zeros_like(A), np.zeros_like(B)
    dE_A, dE_B, dD = (np.zeros((np.asarray(D).shape[0], t * t)) for _ in range(3))
    for b in range(nbatch):
        Ab, Bs = A[b * m:(b + 1) * m], B[b * rb:(b + 1) * rb]
        Bb = Bs.T if b_transposed else Bs
        Bhat = encode(Bb, E_B, t)
        dAb, dBhat, dEa, dDb = backward(Ab, Bhat, E_A, D, dC[b * m:(b + 1) * m], t)
        dBb, dEb = encode_weight_backward(Bb, E_B, dBhat, t)
        dA[b * m:(b + 1) * m] = dAb
        dB[b * rb:(b + 1) * rb] = dBb.T if b_transposed else dBb
        dE_A += dEa
        dE_B += dEb
        dD += dDb
    return dA, dB, dE_A, dE_B, dD


# ------------------------------------------------------------------ row counts that t does not divide
def pad_rows(X, rows: int, t: int = 4):
    """Appendix "More Details on STL Replacement in T2T-ViT", item 1: every image contributes `rows` token rows
    (197 in the paper) and is extended with null rows to the next multiple of t (200).  X is the stack
    (nimg*rows, k); returns (nimg*rows_pad, k)."""
    X = np.asarray(X, dtype=np.float64)
    nimg = X.shape[0] // rows
    if X.shape[0] != nimg * rows:
        raise ValueError("row count is not a multiple of the per-image rows")
    rows_pad = -(-rows // t) * t
    out = np.zeros((nimg, rows_pad, X.shape[1]))
    out[:, :rows] = X.reshape(nimg, rows, -1)
    return out.reshape(nimg * rows_pad, -1)


def fold_rows(Y, fold, rows: int, t: int = 4):
    """Same passage, the way back: the padded output (nimg*rows_pad, n) returns to (nimg*rows, n) rows.  Rows of
    complete tile rows are kept; the last t padded rows of an image are combined linearly into its remaining
    rho = rows - t*floor(rows/t) rows with the trainable coefficients `fold` (rho x t): the paper's case is
    rho = 1 with 4 coefficients, and one combination per remaining row is the reading taken for rho = 2, 3.
    With rows divisible by t nothing is folded."""
    Y = np.asarray(Y, dtype=np.float64)
    rows_pad = -(-rows // t) * t
    nimg = Y.shape[0] // rows_pad
    Y3 = Y.reshape(nimg, rows_pad, -1)
    if rows_pad == rows:
        return Y.copy()
    fold = np.asarray(fold, dtype=np.float64)
    body = rows_pad - t
    if fold.shape != (rows - body, t):
        raise ValueError("fold must be (rows mod t) x t")
    out = np.empty((nimg, rows, Y3.shape[2]))
    out[:, :body] = Y3[:, :body]
    out[:, body:] = np.einsum("ra,iaj->irj", fold, Y3[:, body:])
    return out.reshape(nimg * rows, -1)


def ragged_forward(X, What, E_X, D, fold, rows: int, t: int = 4):
    """STL layer on images of `rows` tokens each: pad with null rows, apply the operator, fold back."""
    return fold_rows(forward(pad_rows(X, rows, t), What, E_X, D, t), fold, rows, t)


def ragged_backward(X, What, E_X, D, fold, dC, rows: int, t: int = 4):
    """Gradients of <dC, ragged_forward(...)>: (dX, dWhat, dE_X, dD, dfold).  The fold is linear, so its adjoint
    spreads dC over the padded rows and dfold pairs the padded output with dC; gradients of null rows are
    dropped."""
    X = np.asarray(X, dtype=np.float64)
    dC = np.asarray(dC, dtype=np.float64)
    rows_pad = -(-rows // t) * t
    nimg = X.shape[0] // rows
    body = rows_pad - t
    Xp = pad_rows(X, rows, t)
    dC3 = dC.reshape(nimg, rows, -1)
    dY = np.zeros((nimg, rows_pad, dC3.shape[2]))
    if rows_pad == rows:
        dY[:] = dC3
        dfold = None
    else:
        fold = np.asarray(fold, dtype=np.float64)
        Y3 = forward(Xp, What, E_X, D, t).reshape(nimg, rows_pad, -1)
        dY[:, :body] = dC3[:, :body]
        dY[:, body:] = np.einsum("ra,irj->iaj", fold, dC3[:, body:])
        dfold = np.einsum("irj,iaj->ra", dC3[:, body:], Y3[:, body:])
    dXp, dWhat, dE_X, dD = backward(Xp, What, E_X, D, dY.reshape(nimg * rows_pad, -1), t)
    dX = dXp.reshape(nimg, rows_pad, -1)[:, :rows].reshape(nimg * rows, -1)
    return dX, dWhat, dE_X, dD, dfold
