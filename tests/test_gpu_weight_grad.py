"""GPU parity of the gradients through the weight encoding (dW, dE_W) against the fp64 oracle."""
import numpy as np
import pytest

import oracle
import stl_synth
from oracle import bases, planes

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import gpu_util
    return gpu_util


def _inputs(rng, k, n, r, dtype):
    W = stl_synth.round_to(rng.standard_normal((k, n)) * k ** -0.5, dtype)
    E_W = stl_synth.round_to(rng.standard_normal((r, 16)) * 0.25, dtype)
    dWhat = rng.standard_normal((r, k // 4, n // 4)).astype(np.float32)
    return W, E_W, dWhat


@pytest.mark.parametrize("dtype,k,n,r", [
    ("bf16", 256, 384, 24),      # one-pass kernel (tile columns a multiple of 8)
    ("bf16", 1000, 328, 49),     # ragged chunks, two 32-plane groups
    ("bf16", 64, 36, 8),         # 9 tile columns: generic kernels on the rounded planes
    ("f32", 96, 160, 17),
    ("f32", 8, 4, 1),
])
def test_weight_encoding_gradients(gu, dtype, k, n, r):
    rng = np.random.default_rng(7000 + k + n + r)
    W, E_W, dWhat = _inputs(rng, k, n, r, dtype)
    ref_dW, ref_dE = planes.encode_weight_backward(W, E_W, dWhat)
    got = gu.encode_weight_backward(W, E_W, dWhat, dtype)
    assert gu.rel(got["dW"], ref_dW) <= gu.TOL[dtype]
    assert gu.rel(got["dE_W"], ref_dE) <= gu.TOL[dtype]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_accumulate_and_skipped_outputs(gu, dtype):
    rng = np.random.default_rng(7100)
    W, E_W, dWhat = _inputs(rng, 128, 192, 32, dtype)
    ref_dW, ref_dE = planes.encode_weight_backward(W, E_W, dWhat)
    init = rng.standard_normal((32, 16)).astype(np.float32) * 10
    got = gu.encode_weight_backward(W, E_W, dWhat, dtype, accumulate=1, init=init)
    assert gu.rel(got["dE_W"] - init, ref_dE) <= 2 * gu.TOL[dtype]
    assert gu.rel(got["dW"], ref_dW) <= gu.TOL[dtype]
    only_dw = gu.encode_weight_backward(W, E_W, dWhat, dtype, skip=("dE_W",))
    assert np.isnan(only_dw["dE_W"]).all() and np.array_equal(only_dw["dW"], got["dW"])
    only_de = gu.encode_weight_backward(W, E_W, dWhat, dtype, skip=("dW",))
    assert np.isnan(only_de["dW"]).all() and gu.rel(only_de["dE_W"], ref_dE) <= gu.TOL[dtype]
    # run-to-run reproducible
    again = gu.encode_weight_backward(W, E_W, dWhat, dtype)
    first = gu.encode_weight_backward(W, E_W, dWhat, dtype)
    assert np.array_equal(again["dE_W"], first["dE_W"]) and np.array_equal(again["dW"], first["dW"])


def test_chain_to_textbook_weight_gradient_fp32(gu):
    """fp32, Strassen-squared basis: encode W, forward, backward, then back through the encoding gives dW = X^T dC."""
    import torch
    import paper_2503_12211_amd as stl
    E_X, E_W, D = bases.strassen_4x4()
    rng = np.random.default_rng(7200)
    m, k, n = 64, 48, 80
    X = rng.standard_normal((m, k)).astype(np.float32)
    W = (rng.standard_normal((k, n)) / np.sqrt(k)).astype(np.float32)
    dC = rng.standard_normal((m, n)).astype(np.float32)
    prob = stl.Problem(m, k, n, 49, stl.STL_F32)
    Wd, EWd = gu.dev(W, "f32"), gu.dev(E_W, "f32")
    What = torch.empty((49, k // 4, n // 4), dtype=torch.float32, device="cuda")
    stl.stl_encode_weight(prob, Wd, EWd, What)
    p = {"X": X, "What": gu.host(What), "E_X": E_X, "D": D, "dC": dC}
    g = gu.backward(p, "f32")
    got = gu.encode_weight_backward(W, E_W, g["dWhat"], "f32")
    assert gu.rel(got["dW"], X.astype(np.float64).T @ dC.astype(np.float64)) <= 2 * gu.TOL["f32"]


def test_full_size_weight_gradients(gu):
    """k = n = 4096, r = 32, bf16: the size of the forward+backward workload's weight."""
    rng = np.random.default_rng(7300)
    W, E_W, dWhat = _inputs(rng, 4096, 4096, 32, "bf16")
    ref_dW, ref_dE = planes.encode_weight_backward(W, E_W, dWhat)
    got = gu.encode_weight_backward(W, E_W, dWhat, "bf16")
    assert gu.rel(got["dW"], ref_dW) <= gu.TOL["bf16"]
    assert gu.rel(got["dE_W"], ref_dE) <= gu.TOL["bf16"]
