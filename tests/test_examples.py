"""The Class-0 fitting example: its own basis generator (CPU) and a short training run through the library (GPU)."""
import numpy as np
import pytest

from paper_2503_12211_amd.examples import class0_fit


def test_example_basis_is_exact_and_matches_the_oracle_fixture():
    """The example builds its own r=49 basis (product code shares nothing with the oracle): it must multiply 4x4
    tiles exactly and equal the oracle's fixture row for row."""
    from oracle import bases
    E_X, E_W, D = class0_fit.seven_product_basis_4x4()
    rng = np.random.default_rng(0)
    X, W = rng.standard_normal((4, 4)), rng.standard_normal((4, 4))
    c = D.T @ ((E_X @ X.reshape(-1)) * (E_W @ W.reshape(-1)))
    assert np.abs(c.reshape(4, 4) - X @ W).max() < 1e-14
    for mine, ref in zip((E_X, E_W, D), bases.strassen_4x4()):
        assert np.array_equal(mine, ref)


@pytest.mark.gpu
def test_class0_fit_trains_through_the_library():
    # exact basis: the residual of the first step is fp32 rounding noise (Adam then moves the bases by about its
    # step size whatever the gradient's magnitude, so later steps only have to stay small)
    h = class0_fit.fit(49, steps=3, init="strassen", size=64)
    assert h[0] < 1e-9 and max(h) < 1e-2, h
    # pruned basis and Gaussian start: the error estimate must fall (per-entry variance of X W is 4)
    for init in ("strassen", "gauss"):
        h = class0_fit.fit(32, steps=120, init=init, size=64, seed=3)
        assert np.isfinite(h).all()
        assert np.mean(h[-10:]) < 0.6 * np.mean(h[:3]), (init, h[:3], h[-10:])
    # and more planes fit better than fewer, from the same kind of start
    h16 = class0_fit.fit(16, steps=120, init="gauss", size=64, seed=3)
    h48 = class0_fit.fit(48, steps=120, init="gauss", size=64, seed=3)
    assert np.mean(h48[-10:]) < np.mean(h16[-10:])


@pytest.mark.gpu
@pytest.mark.parametrize("init,r", [("strassen", 32), ("gauss", 24), ("strassen", 49)])
def test_class0_steps_against_the_oracle(init, r):
    """The first training steps of the Class-0 fit recomputed by the oracle on the same tiles and the same bases: the
    error estimate alpha, and the gradients of all three bases (dE_X and dD from the backward oracle, dE_W through the
    oracle of the weight encoding), fp32 storage."""
    import oracle
    from oracle import planes
    trace = []
    class0_fit.fit(r, steps=3, init=init, size=64, seed=11, trace=trace, trace_steps=3)
    assert len(trace) == 3
    for i, t in enumerate(trace):
        m, k = t["X"].shape
        n = t["W"].shape[1]
        What = oracle.encode_weight(t["W"], t["E_W"])
        C = oracle.forward(t["X"], What, t["E_X"], t["D"])
        resid = C - t["X"] @ t["W"]
        alpha = float((resid * resid).sum() / (m * n * (k // 4)))
        dC = resid * (2.0 / (m * n * (k // 4)))
        if alpha > 1e-3:                                         # away from the exact basis the fp32 residual is accurate
            assert np.linalg.norm(t["dC"] - dC) <= 1e-4 * np.linalg.norm(dC), i
        # gradients for the upstream gradient the step actually used (near the exact basis the fp32 residual C - X W
        # is mostly rounding of its two terms, which is the example's arithmetic, not the library's)
        _, dWhat, dE_X, dD = oracle.backward(t["X"], What, t["E_X"], t["D"], t["dC"])
        _, dE_W = planes.encode_weight_backward(t["W"], t["E_W"], dWhat)
        if init == "strassen" and r == 49 and i == 0:
            assert alpha < 1e-20 and t["alpha"] < 1e-9           # exact basis: nothing but rounding
            continue
        assert abs(t["alpha"] - alpha) <= 1e-4 * alpha + 1e-9, (i, t["alpha"], alpha)
        for name, ref in (("dE_X", dE_X), ("dE_W", dE_W), ("dD", dD)):
            err = np.linalg.norm(t[name] - ref) / np.linalg.norm(ref)
            assert err <= 2e-5, (i, name, err)       # two chained fp32 passes (backward, then the weight encoding's)
        if i:
            for name in ("E_X", "E_W", "D"):                     # the optimiser moved the bases between the steps
                assert not np.array_equal(t[name], trace[i - 1][name])


@pytest.mark.gpu
def test_autograd_layer_matches_the_oracle_gradients():
    """The PyTorch layer built on the C ABI: outputs and all four autograd gradients against the fp64 oracle, and a few
    optimiser steps that lower a regression loss."""
    import torch
    import gpu_util as gu
    import stl_synth
    from oracle import planes
    from paper_2503_12211_amd.examples.stl_linear import STLLinear, stl_linear
    for dtype, tdt in (("bf16", torch.bfloat16), ("f32", torch.float32)):
        p = stl_synth.stl_problem(64, 96, 128, 24, seed=41, dtype=dtype, with_dC=True)
        X, What, E_X, D = (gu.dev(p[s], dtype).requires_grad_() for s in ("X", "What", "E_X", "D"))
        C = stl_linear(X, What, E_X, D)
        C.backward(gu.dev(p["dC"], dtype))
        assert gu.rel(gu.host(C), planes.forward(p["X"], p["What"], p["E_X"], p["D"])) <= gu.TOL[dtype]
        ref = planes.backward(p["X"], p["What"], p["E_X"], p["D"], p["dC"])
        for t, g in zip((X, What, E_X, D), ref):
            assert t.grad.dtype == tdt
            assert gu.rel(gu.host(t.grad), g) <= 1.5 * gu.TOL[dtype]      # parameter gradients are rounded to the storage type
    layer = STLLinear(64, 32, 16, dtype=torch.float32).cuda()
    opt = torch.optim.Adam(layer.parameters(), lr=1e-2)
    gen = torch.Generator(device="cuda").manual_seed(5)
    x = torch.randn((4, 32, 64), device="cuda", generator=gen)
    target = torch.randn((4, 32, 32), device="cuda", generator=gen)
    losses = []
    for _ in range(30):
        opt.zero_grad()
        loss = ((layer(x) - target) ** 2).mean()
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    assert losses[-1] < 0.9 * losses[0], losses
