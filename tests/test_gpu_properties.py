"""Property tests on the GPU path (random small shapes): parity with the oracle, bilinearity, rank additivity."""
import numpy as np
import pytest

import oracle
import stl_synth

hyp = pytest.importorskip("hypothesis")
from hypothesis import given, settings, strategies as st, HealthCheck

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import gpu_util
    return gpu_util


dims = st.integers(min_value=1, max_value=24).map(lambda v: 4 * v)


# derandomize: the same 40 shapes on every run.  With a handful of tiles a near-cancelling decode sum can push the bf16
# relative error of a random example past the bar (worst seen over 1500 tiny bf16 shapes: 0.0074 against 0.01), so the
# examples are fixed rather than drawn afresh each time.
@settings(max_examples=40, deadline=None, derandomize=True, database=None,
          suppress_health_check=[HealthCheck.function_scoped_fixture])
@given(m=dims, k=dims, n=dims, r=st.integers(1, 64), seed=st.integers(0, 2 ** 16), dtype=st.sampled_from(["f32", "bf16"]))
def test_forward_backward_random_shapes(gu, m, k, n, r, seed, dtype):
    p = stl_synth.stl_problem(m, k, n, r, seed=seed, dtype=dtype, with_dC=True)
    C = gu.forward(p, dtype)
    assert gu.rel(C, oracle.forward(p["X"], p["What"], p["E_X"], p["D"])) <= gu.TOL[dtype]
    got = gu.backward(p, dtype)
    ref = oracle.backward(p["X"], p["What"], p["E_X"], p["D"], p["dC"])
    for name, g in zip(("dX", "dWhat", "dE_X", "dD"), ref):
        assert gu.rel(got[name], g) <= gu.TOL[dtype], name


@settings(max_examples=30, deadline=None, database=None, suppress_health_check=[HealthCheck.function_scoped_fixture])
@given(m=dims, k=dims, n=dims, r=st.integers(1, 64), seed=st.integers(0, 2 ** 31 - 1), dtype=st.sampled_from(["f32", "bf16"]))
def test_forward_and_input_gradient_fresh_draws_entrywise_bound(gu, m, k, n, r, seed, dtype):
    """Fresh examples on every run, against a bound that holds for EVERY draw: the roundings of the path (encoded operand,
    encoded product, output: relative 2^-8 each for bf16, whose significand has 8 bits; fp32 accumulation over the contraction and the planes) bound the
    error of an entry by a multiple of the same expression evaluated on absolute values,
        |C - C_exact| <= (3 u + (K + r + 24) 2^-24) * decode_|D|( encode_|E_X|(|X|) . |What| ),
    however much the signed sums cancel (which is what makes a relative-norm bar unsafe for tiny random shapes).  The same
    for dX with (D, dC) as encoder and input, What transposed, and E_X as decoder."""
    from oracle import planes
    p = stl_synth.stl_problem(m, k, n, r, seed=seed, dtype=dtype, with_dC=True)
    u = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -24
    a = {k_: np.abs(np.asarray(v, dtype=np.float64)) for k_, v in p.items()}
    C = gu.forward(p, dtype)
    ref = oracle.forward(p["X"], p["What"], p["E_X"], p["D"])
    S = planes.decode(planes.plane_products(planes.encode(a["X"], a["E_X"]), a["What"]), a["D"])
    c = 3 * u * 1.01 + (k // 4 + r + 24) * 2.0 ** -24
    assert np.all(np.abs(C - ref) <= c * S + 1e-30), float(np.max(np.abs(C - ref) / (c * S + 1e-30)))
    dX = gu.backward(p, dtype, skip=("dWhat", "dE_X", "dD"))["dX"]
    dX_ref = oracle.backward(p["X"], p["What"], p["E_X"], p["D"], p["dC"])[0]
    S2 = planes.decode(planes.plane_products(planes.encode(a["dC"], a["D"]), a["What"].transpose(0, 2, 1)), a["E_X"])
    c2 = 3 * u * 1.01 + (n // 4 + r + 24) * 2.0 ** -24
    assert np.all(np.abs(dX - dX_ref) <= c2 * S2 + 1e-30), float(np.max(np.abs(dX - dX_ref) / (c2 * S2 + 1e-30)))


def test_fp32_bilinearity_and_rank_additivity(gu):
    """fp32 path: f(aX1+bX2) = a f(X1) + b f(X2); planes [0,r1) plus planes [r1,r) add up to all planes."""
    rng = np.random.default_rng(5)
    p = stl_synth.stl_problem(64, 96, 128, 24, seed=9, dtype="f32")
    X2 = rng.standard_normal(p["X"].shape).astype(np.float32)
    q = dict(p)
    q["X"] = (0.5 * p["X"] - 2.0 * X2).astype(np.float32)
    q2 = dict(p)
    q2["X"] = X2
    lhs = gu.forward(q, "f32")
    rhs = 0.5 * gu.forward(p, "f32") - 2.0 * gu.forward(q2, "f32")
    assert gu.rel(lhs, rhs) <= 1e-5
    part = 0
    for sl in (slice(0, 10), slice(10, 24)):
        s = {"X": p["X"], "What": p["What"][sl], "E_X": p["E_X"][sl], "D": p["D"][sl]}
        part = part + gu.forward(s, "f32")
    assert gu.rel(part, gu.forward(p, "f32")) <= 1e-5


small = st.integers(min_value=1, max_value=12).map(lambda v: 4 * v)


@settings(max_examples=25, deadline=None, derandomize=True, database=None,
          suppress_health_check=[HealthCheck.function_scoped_fixture])
@given(nb=st.integers(1, 5), m=small, k=small, n=small, r=st.integers(1, 64), seed=st.integers(0, 2 ** 16),
       dtype=st.sampled_from(["f32", "bf16"]))
def test_two_activations_random_shapes(gu, nb, m, k, n, r, seed, dtype):
    from oracle import planes
    p = stl_synth.aa_problem(nb, m, k, n, r, seed=seed, dtype=dtype, with_dC=True)
    args = (p["A"], p["B"], p["E_A"], p["E_B"], p["D"])
    tol = gu.TOL[dtype]
    assert gu.rel(gu.aa_forward(*args, nb, dtype), planes.aa_forward(*args, nbatch=nb)) <= tol
    got = gu.aa_backward(*args, p["dC"], nb, dtype)
    ref = planes.aa_backward(*args, p["dC"], nbatch=nb)
    for name, g in zip(("dA", "dB", "dE_A", "dE_B", "dD"), ref):
        assert gu.rel(got[name], g) <= tol, name


@settings(max_examples=25, deadline=None, derandomize=True, database=None,
          suppress_health_check=[HealthCheck.function_scoped_fixture])
@given(nimg=st.integers(1, 5), rows=st.integers(4, 45), k=small, n=small, r=st.integers(1, 64), seed=st.integers(0, 2 ** 16),
       dtype=st.sampled_from(["f32", "bf16"]))
def test_ragged_rows_random_shapes(gu, nimg, rows, k, n, r, seed, dtype):
    from oracle import planes
    p = stl_synth.ragged_problem(nimg, rows, k, n, r, seed=seed, dtype=dtype, with_dC=True)
    tol = gu.TOL[dtype]
    ref = planes.ragged_forward(p["X"], p["What"], p["E_X"], p["D"], p["fold"], rows)
    assert gu.rel(gu.ragged_forward(p, rows, dtype), ref) <= tol
    got = gu.ragged_backward(p, rows, dtype)
    refs = planes.ragged_backward(p["X"], p["What"], p["E_X"], p["D"], p["fold"], p["dC"], rows)
    for name, g in zip(("dX", "dWhat", "dE_X", "dD", "dfold"), refs):
        if g is None:
            assert got[name] is None
        else:
            assert gu.rel(got[name], g) <= tol, name
