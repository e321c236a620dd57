"""GPU parity: stl_backward (dX, dWhat, dE_X, dD) against the fp64 oracle and finite differences."""
import numpy as np
import pytest

import oracle
import stl_synth
from oracle import planes

pytestmark = pytest.mark.gpu
NAMES = ("dX", "dWhat", "dE_X", "dD")


@pytest.fixture(scope="module")
def gu():
    import gpu_util
    return gpu_util


def oracle_grads(p, use_planes=False):
    f = planes.backward if use_planes else oracle.backward
    return dict(zip(NAMES, f(p["X"], p["What"], p["E_X"], p["D"], p["dC"])))


SHAPES = [(4, 4, 4, 1), (20, 36, 28, 7), (68, 132, 76, 24), (160, 96, 224, 32), (32, 32, 32, 64)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_backward_small(gu, dtype, shape):
    m, k, n, r = shape
    p = stl_synth.stl_problem(m, k, n, r, seed=31 + m + r, dtype=dtype, with_dC=True)
    got = gu.backward(p, dtype)
    ref = oracle_grads(p)
    for name in NAMES:
        assert gu.rel(got[name], ref[name]) <= gu.TOL[dtype], name


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_finite_differences_32(gu, dtype):
    """m=k=n=32: <grad, V> from the GPU equals the central difference of the fp64 forward along V
    (the loss is linear in each argument, so the difference quotient has no truncation error)."""
    p = stl_synth.stl_problem(32, 32, 32, 32, seed=41, dtype=dtype, with_dC=True)
    got = gu.backward(p, dtype)
    rng = np.random.default_rng(1)
    keys = {"dX": "X", "dWhat": "What", "dE_X": "E_X", "dD": "D"}

    def loss(q):
        return float(np.sum(q["dC"].astype(np.float64) * oracle.forward(q["X"], q["What"], q["E_X"], q["D"])))

    for g, a in keys.items():
        V = rng.standard_normal(p[a].shape)
        plus = {k_: v.astype(np.float64) for k_, v in p.items()}
        minus = {k_: v.astype(np.float64) for k_, v in p.items()}
        plus[a] = plus[a] + 1e-3 * V
        minus[a] = minus[a] - 1e-3 * V
        fd = (loss(plus) - loss(minus)) / 2e-3
        an = float(np.sum(got[g] * V))
        scale = np.linalg.norm(got[g]) * np.linalg.norm(V)
        assert abs(fd - an) <= gu.TOL[dtype] * scale, (g, fd, an)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_256_slice(gu, dtype):
    """The 256 x 256 x 256 sub-problem with the workload's distributions, r=32."""
    p = stl_synth.stl_problem(256, 256, 256, 32, seed=51, dtype=dtype, with_dC=True)
    got = gu.backward(p, dtype)
    ref = oracle_grads(p)
    for name in NAMES:
        assert gu.rel(got[name], ref[name]) <= gu.TOL[dtype], name
    # Euler identities: the loss is homogeneous of degree one in every argument
    lhs = [np.sum(got["dX"] * p["X"]), np.sum(got["dWhat"] * p["What"]), np.sum(got["dE_X"] * p["E_X"]),
           np.sum(got["dD"] * p["D"])]
    val = np.sum(p["dC"].astype(np.float64) * oracle.forward(p["X"], p["What"], p["E_X"], p["D"]))
    scale = np.linalg.norm(p["dC"]) * np.linalg.norm(oracle.forward(p["X"], p["What"], p["E_X"], p["D"]))
    for v in lhs:
        assert abs(v - val) <= gu.TOL[dtype] * scale


def test_backward_saved_yhat_accumulate_and_skips(gu):
    dtype = "bf16"
    p = stl_synth.stl_problem(96, 160, 128, 16, seed=61, dtype=dtype, with_dC=True)
    ref = oracle_grads(p)
    C, Xh, Y = gu.forward(p, dtype, save_yhat=True, save_xhat=True)
    with_saved = gu.backward(p, dtype, yhat=Y)
    both_saved = gu.backward(p, dtype, yhat=Y, xhat=Xh)
    for name in NAMES:
        assert gu.rel(with_saved[name], ref[name]) <= gu.TOL[dtype], name
        assert np.array_equal(with_saved[name], both_saved[name]), name
    rng = np.random.default_rng(2)
    init = [rng.standard_normal(ref[nm].shape).astype(np.float32) for nm in ("dWhat", "dE_X", "dD")]
    acc = gu.backward(p, dtype, accumulate=1, init=init)
    for nm, i0 in zip(("dWhat", "dE_X", "dD"), init):
        assert gu.rel(acc[nm] - i0, ref[nm]) <= gu.TOL[dtype], nm
    part = gu.backward(p, dtype, skip=("dX", "dD"))
    assert np.isnan(part["dX"]).all() and np.isnan(part["dD"]).all()       # untouched
    assert gu.rel(part["dWhat"], ref["dWhat"]) <= gu.TOL[dtype]
    assert gu.rel(part["dE_X"], ref["dE_X"]) <= gu.TOL[dtype]


@pytest.mark.parametrize("shape", [(1056, 544, 800, 8), (1152, 1152, 1152, 3), (1184, 1152, 1216, 2)])
def test_backward_matrix_core_shapes_bf16(gu, shape):
    """Plane sizes that take the MFMA kernels (register-staged and LDS-DMA pipelined) in all three
    products, with blocks that hang over the edge."""
    m, k, n, r = shape
    p = stl_synth.stl_problem(m, k, n, r, seed=71 + r, dtype="bf16", with_dC=True)
    got = gu.backward(p, "bf16")
    ref = oracle_grads(p, use_planes=True)
    for name in NAMES:
        assert gu.rel(got[name], ref[name]) <= gu.TOL["bf16"], name
    again = gu.backward(p, "bf16")
    for name in NAMES:
        assert np.array_equal(got[name], again[name]), name        # bitwise reproducible


def test_config5_full_size(gu):
    """bf16, m=8192, k=n=4096, r=32, backward at full size with nothing saved (Xhat and Yhat recomputed inside
    stl_backward) against the plane oracle: whole-tensor norm, every entry, every 256 x 256 block and tile row."""
    cfg, p = stl_synth.config_problem("C5", with_dC=True)
    got = gu.backward(p, "bf16")
    ref = oracle_grads(p, use_planes=True)
    for name in NAMES:
        gu.check(got[name], ref[name], "bf16", f"C5 recompute {name}")


def test_config5_step_as_benchmarked(gu):
    """The step bench.py times, at its size (bf16, m=8192, k=n=4096, r=32): stl_forward handing Xhat and Yhat to
    stl_backward through Xhat_save / Yhat_save.  Everything the step produces -- C, the two saved plane tensors and
    the four gradients -- against the plane oracle: whole-tensor norm, every entry, every 256 x 256 block and every
    tile row (see gpu_util.check)."""
    cfg, p = stl_synth.config_problem("C5", with_dC=True)
    got = gu.step(p, "bf16")
    Cref, Yref = planes.forward(p["X"], p["What"], p["E_X"], p["D"], return_yhat=True)
    gu.check(got["C"], Cref, "bf16", "C5 step C")
    gu.check(got["Yhat"], Yref, "bf16", "C5 step Yhat", slab=1)
    del Cref, Yref
    gu.check(got["Xhat"], planes.encode(p["X"], p["E_X"]), "bf16", "C5 step Xhat", slab=1)
    ref = oracle_grads(p, use_planes=True)
    for name in NAMES:
        gu.check(got[name], ref[name], "bf16", f"C5 step {name}")
    # sampled 8x8-tile blocks of C against the literal per-tile definition as well
    rng = np.random.default_rng(5)
    for _ in range(3):
        I0, J0 = int(rng.integers(0, 2048 - 8)), int(rng.integers(0, 1024 - 8))
        blk = oracle.forward_block(p["X"], p["What"], p["E_X"], p["D"], I0, I0 + 8, J0, J0 + 8)
        assert gu.rel(got["C"][4 * I0:4 * I0 + 32, 4 * J0:4 * J0 + 32], blk) <= 2 * gu.TOL["bf16"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_step_mid_size_every_entry(gu, dtype):
    """The same saved-plane step at a size that spans several blocks with ragged edges (M = 328, K = 136, N = 200 tile
    counts), both storage types, every output with the full set of checks."""
    p = stl_synth.stl_problem(1312, 544, 800, 24, seed=91, dtype=dtype, with_dC=True)
    got = gu.step(p, dtype)
    Cref, Yref = planes.forward(p["X"], p["What"], p["E_X"], p["D"], return_yhat=True)
    gu.check(got["C"], Cref, dtype, "C")
    gu.check(got["Yhat"], Yref, dtype, "Yhat", slab=1)
    gu.check(got["Xhat"], planes.encode(p["X"], p["E_X"]), dtype, "Xhat", slab=1)
    ref = oracle_grads(p, use_planes=True)
    for name in NAMES:
        gu.check(got[name], ref[name], dtype, name)


@pytest.mark.parametrize("dtype,shape", [("f32", (560004, 8, 8, 2)), ("bf16", (560000, 32, 32, 8)), ("bf16", (560004, 24, 8, 5))])
def test_tall_matrix_beyond_one_grid_extent(gu, dtype, shape):
    """More tile rows (140 000) than a grid extent holds (65 535): the row loops of the tile maps and of the any-shape plane
    products wrap around.  Forward and backward, every entry of C and dX sampled by whole row blocks, all of the small
    gradients; the oracle runs on the sampled rows only (rows are independent in C and dX) and on all rows for the sums."""
    m, k, n, r = shape
    p = stl_synth.stl_problem(m, k, n, r, seed=77, dtype=dtype, with_dC=True)
    res = gu.step(p, dtype)
    ref = dict(zip(NAMES, planes.backward(p["X"], p["What"], p["E_X"], p["D"], p["dC"])))
    C_ref = planes.forward(p["X"], p["What"], p["E_X"], p["D"])
    tol = gu.TOL[dtype]
    for lo in (0, 4 * 32768 - 8, 4 * 65535 - 8, 4 * 65536, 4 * 131072 - 4, m - 16):
        sl = slice(lo, lo + 16)
        assert gu.rel(res["C"][sl], C_ref[sl]) <= tol, ("C", lo)
        assert gu.rel(res["dX"][sl], ref["dX"][sl]) <= tol, ("dX", lo)
    assert gu.rel(res["C"], C_ref) <= tol and gu.rel(res["dX"], ref["dX"]) <= tol
    for name in ("dWhat", "dE_X", "dD"):
        assert gu.rel(res[name], ref[name]) <= tol, name
