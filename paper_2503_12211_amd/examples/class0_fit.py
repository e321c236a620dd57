"""Fit the STL bases (E_X, E_W, D) to plain matrix multiplication of Gaussian 4x4 tiles -- the paper's
"Class 0" experiment (Section "Class 0 Experiments", appendix paragraphs "Estimates of alpha_STL" and
"Initialization Issues") -- with the library's own forward and backward passes.

    alpha_STL(r) = min over bases of (1/16) E || X W - STL(X, W) ||_F^2      over 4x4 Gaussian tiles X, W.

One call of the operator on random X (m x k) and W (k x n) evaluates M*K*N independent tile pairs at once: the
residual of output tile (I, J) is the sum over L of the residuals of the pairs (X_{I,L}, W_{L,J}), which are
uncorrelated for i.i.d. Gaussian tiles, so ||C - X W||_F^2 / (m n K) estimates the per-entry error alpha.
Training uses true encoding (What = encode(W, E_W)), so all three bases get gradients:
stl_backward gives dE_X, dD and dWhat; stl_encode_weight_backward turns dWhat into dE_W.
Initialisation: `strassen` takes r random rows of the two-level seven-product basis (r = 49 is exact),
`gauss` draws N(0, 1/16) entries.  fp32 storage.  PyTorch supplies device memory, the target product and Adam.

    python -m paper_2503_12211_amd.examples.class0_fit --r 16 24 32 42 49 --steps 400
"""
from __future__ import annotations

import argparse

import numpy as np


def seven_product_basis_4x4():
    """(E_X, E_W, D), each 49 x 16, of the two-level seven-product scheme for 4x4 tiles vectorised row-major."""
    # one level, operands ordered (11, 12, 21, 22): rows = the seven products
    U = np.array([[1, 0, 0, 1], [0, 0, 1, 1], [1, 0, 0, 0], [0, 0, 0, 1], [1, 1, 0, 0], [-1, 0, 1, 0], [0, 1, 0, -1]], float)
    V = np.array([[1, 0, 0, 1], [1, 0, 0, 0], [0, 1, 0, -1], [-1, 0, 1, 0], [0, 0, 0, 1], [1, 1, 0, 0], [0, 0, 1, 1]], float)
    Z = np.array([[1, 0, 0, 1], [0, 0, 1, -1], [0, 1, 0, 1], [1, 0, 1, 0], [-1, 1, 0, 0], [0, 0, 0, 1], [1, 0, 0, 0]], float)

    def two_level(F):
        out = np.zeros((49, 16))
        for p in range(7):
            for q in range(7):
                for bi in range(2):
                    for bj in range(2):
                        for si in range(2):
                            for sj in range(2):
                                out[7 * p + q, 4 * (2 * bi + si) + (2 * bj + sj)] = F[p, 2 * bi + bj] * F[q, 2 * si + sj]
        return out
    return two_level(U), two_level(V), two_level(Z)


def fit(r: int, steps: int = 300, init: str = "strassen", seed: int = 0, size: int = 128, lr: float = 3e-3,
        log_every: int = 0, trace: list | None = None, trace_steps: int = 0):
    """Returns the list of per-step estimates of alpha (before each update).  With `trace` (a list) the first
    `trace_steps` steps append a dict of host copies of what the step saw and produced -- X, W, the three bases before
    the update, alpha, the upstream gradient dC and the three basis gradients -- so that a test can recompute the step independently."""
    import torch

    import paper_2503_12211_amd as stl

    rng = np.random.default_rng(seed)
    if init == "strassen":
        rows = np.sort(rng.choice(49, size=r, replace=False)) if r <= 49 else None
        if rows is None:
            raise ValueError("strassen initialisation needs r <= 49")
        bases = [b[rows] for b in seven_product_basis_4x4()]
    elif init == "gauss":
        bases = [rng.standard_normal((r, 16)) * 0.25 for _ in range(3)]
    else:
        raise ValueError("init must be 'strassen' or 'gauss'")
    dev = dict(device="cuda", dtype=torch.float32)
    E_X, E_W, D = (torch.tensor(b, **dev).contiguous() for b in bases)
    params = [E_X, E_W, D]
    for p_ in params:
        p_.grad = torch.zeros_like(p_)
    opt = torch.optim.Adam(params, lr=lr)

    m = k = n = size
    M, K, N = m // 4, k // 4, n // 4
    prob = stl.Problem(m, k, n, r, stl.STL_F32)
    What = torch.empty((r, K, N), **dev)
    C = torch.empty((m, n), **dev)
    Xhat = torch.empty(stl.stl_plane_elems(M, K, r), **dev)    # saved planes, layout private to the library
    Yhat = torch.empty(stl.stl_plane_elems(M, N, r), **dev)
    dWhat = torch.empty((r, K, N), **dev)
    sizes = [stl.stl_workspace_bytes(prob, op) for op in (stl.STL_OP_FORWARD, stl.STL_OP_BACKWARD, stl.STL_OP_ENCODE_WEIGHT_BACKWARD)]
    ws = torch.empty(max(max(sizes), 16), dtype=torch.uint8, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(seed + 1)
    history = []
    for step in range(steps):
        X = torch.randn((m, k), generator=gen, **dev)
        W = torch.randn((k, n), generator=gen, **dev)
        stl.stl_encode_weight(prob, W, E_W, What)
        stl.stl_forward(prob, X, What, E_X, D, C, Xhat, Yhat, ws, sizes[0])
        resid = C - X @ W
        alpha = float((resid * resid).sum() / (m * n * K))
        history.append(alpha)
        dC = (resid * (2.0 / (m * n * K))).contiguous()
        stl.stl_backward(prob, X, What, E_X, D, dC, Xhat, Yhat, None, dWhat, E_X.grad, D.grad, 0, ws, sizes[1])
        stl.stl_encode_weight_backward(prob, W, E_W, dWhat, None, E_W.grad, 0, ws, sizes[2])
        if trace is not None and step < trace_steps:
            host = lambda t_: t_.detach().cpu().numpy().astype(np.float64)
            trace.append({"X": host(X), "W": host(W), "E_X": host(E_X), "E_W": host(E_W), "D": host(D), "alpha": alpha, "dC": host(dC),
                          "dE_X": host(E_X.grad), "dE_W": host(E_W.grad), "dD": host(D.grad)})
        opt.step()
        if log_every and step % log_every == 0:
            print(f"  r={r} {init}: step {step:5d}  alpha {alpha:.4f}", flush=True)
    torch.cuda.synchronize()
    return history


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--r", type=int, nargs="+", default=[16, 24, 32, 42, 49])
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--size", type=int, default=128)
    ap.add_argument("--lr", type=float, default=3e-3)
    args = ap.parse_args()
    print("r   init      alpha(start)  alpha(end, mean of last 20 steps)")
    for r in args.r:
        for init in ("strassen", "gauss"):
            if init == "strassen" and r > 49:
                continue
            h = fit(r, args.steps, init, size=args.size, lr=args.lr)
            print(f"{r:<3d} {init:9s} {h[0]:12.4f}  {np.mean(h[-20:]):12.4f}", flush=True)


if __name__ == "__main__":
    main()
