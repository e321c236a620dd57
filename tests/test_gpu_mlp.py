"""GPU parity of the stacked-layer path (Algorithm 2): the one-pass decode -> activation -> encode step and
the whole layer pair, through the C ABI, against the fp64 plane oracle."""
import numpy as np
import pytest

import stl_synth
from oracle import bases, planes

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import gpu_util
    return gpu_util


def _planes_input(rng, r1, M, N1, r2):
    """Encoded first-layer output at the workload's scale (Var Yhat = 1/4) and bases N(0, 1/16), on the bf16 grid."""
    Y = stl_synth.round_to(rng.standard_normal((r1, M, N1)) * 0.5, "bf16")
    D1 = stl_synth.round_to(rng.standard_normal((r1, 16)) * 0.25, "bf16")
    E2 = stl_synth.round_to(rng.standard_normal((r2, 16)) * 0.25, "bf16")
    return Y, D1, E2


@pytest.mark.parametrize("r1,M,N1,r2", [
    (24, 8, 64, 24),      # one full chunk of 64 tiles per row
    (24, 5, 72, 24),      # ragged: a chunk of 64 and a tail of 8 tiles
    (32, 3, 200, 17),     # three chunks and a tail of 8; r2 not a multiple of 16
    (49, 4, 136, 64),     # two 32-plane groups in, four 16-plane groups out
    (8, 7, 8, 5),         # a single 8-tile chunk, small ranks
    (64, 2, 64, 1),
])
@pytest.mark.parametrize("act", ["gelu", None])
def test_recode_one_pass(gu, r1, M, N1, r2, act):
    import paper_2503_12211_amd as stl
    rng = np.random.default_rng(4100 + r1 + N1)
    Y, D1, E2 = _planes_input(rng, r1, M, N1, r2)
    flags = stl.STL_FLAG_GELU if act == "gelu" else 0
    got = gu.recode(Y, D1, E2, "bf16", flags)
    assert np.isfinite(got).all()
    assert gu.rel(got, planes.recode(Y, D1, E2, activation=act)) <= gu.TOL["bf16"]
    # the two-launch form (decode, hidden activation in HBM, encode) rounds at the same places
    two = gu.recode(Y, D1, E2, "bf16", flags | stl.STL_FLAG_UNFUSED, with_scratch=True)
    assert gu.rel(got, two) <= 2e-3


def test_recode_fp32_and_ineligible_shapes_use_the_two_launch_form(gu):
    import paper_2503_12211_amd as stl
    rng = np.random.default_rng(4200)
    Y = rng.standard_normal((10, 3, 9)).astype(np.float32)       # 9 tiles per row: not a multiple of 8
    D1 = (rng.standard_normal((10, 16)) * 0.25).astype(np.float32)
    E2 = (rng.standard_normal((6, 16)) * 0.25).astype(np.float32)
    got = gu.recode(Y, D1, E2, "f32", stl.STL_FLAG_GELU, with_scratch=True)
    assert gu.rel(got, planes.recode(Y, D1, E2)) <= gu.TOL["f32"]
    Yb, Db, Eb = (stl_synth.round_to(a, "bf16") for a in (Y, D1, E2))
    got = gu.recode(Yb, Db, Eb, "bf16", 0, with_scratch=True)
    assert gu.rel(got, planes.recode(Yb, Db, Eb, activation=None)) <= gu.TOL["bf16"]


def test_recode_linear_exact_on_integer_data(gu):
    """Small integers are exact in bf16 and in fp32 sums: the linear step must equal Yhat (D1 E2^T) bit for bit."""
    rng = np.random.default_rng(4300)
    Y = rng.integers(-3, 4, size=(16, 4, 64)).astype(np.float64)
    D1 = rng.integers(-1, 2, size=(16, 16)).astype(np.float64)
    E2 = rng.integers(-1, 2, size=(16, 16)).astype(np.float64)
    # keep the hidden activation exactly representable in bf16 (|h| <= 48 with 8 significant bits)
    want = planes.recode(Y, D1, E2, activation=None)
    got = gu.recode(Y, D1, E2, "bf16", 0)
    exact = np.abs(want) <= 256                                   # integers up to 256 are bf16-exact
    assert exact.mean() > 0.5
    assert np.array_equal(got[exact], want[exact])


@pytest.mark.parametrize("flag", ["auto", "unfused"])
@pytest.mark.parametrize("act", ["gelu", None])
def test_layer_pair_small(gu, flag, act):
    import paper_2503_12211_amd as stl
    m, d, h = 512, 256, 1024
    p1 = stl_synth.stl_problem(m, d, h, 24, seed=stl_synth.SEEDS["C4_up"], dtype="bf16")
    p2 = stl_synth.stl_problem(m, h, d, 24, seed=stl_synth.SEEDS["C4_down"], dtype="bf16")
    flags = (stl.STL_FLAG_GELU if act else 0) | (stl.STL_FLAG_UNFUSED if flag == "unfused" else 0)
    out = gu.mlp_forward(p1, p2, "bf16", flags)
    ref = planes.mlp_pair(p1["X"], p1["What"], p1["E_X"], p1["D"], p2["What"], p2["E_X"], p2["D"], activation=act)
    assert gu.rel(out, ref) <= gu.TOL["bf16"]


def test_layer_pair_ranks_differ_and_ragged(gu):
    import paper_2503_12211_amd as stl
    m, d, h, o = 260, 132, 328, 68            # 65 x 33 x 82 x 17 tiles
    p1 = stl_synth.stl_problem(m, d, h, 32, seed=51, dtype="bf16")
    p2 = stl_synth.stl_problem(m, h, o, 17, seed=52, dtype="bf16")
    out = gu.mlp_forward(p1, p2, "bf16", stl.STL_FLAG_GELU)
    ref = planes.mlp_pair(p1["X"], p1["What"], p1["E_X"], p1["D"], p2["What"], p2["E_X"], p2["D"])
    assert gu.rel(out, ref) <= gu.TOL["bf16"]


def test_layer_pair_fp32_exact_bases_is_textbook_mlp(gu):
    """fp32 storage, Strassen-squared basis in both layers: the pair is gelu(X W1) W2 to fp32 accuracy."""
    import oracle
    import paper_2503_12211_amd as stl
    E_X, E_W, D = bases.strassen_4x4()
    rng = np.random.default_rng(53)
    m, d, h = 64, 48, 96
    X = rng.standard_normal((m, d)).astype(np.float32)
    W1 = (rng.standard_normal((d, h)) / np.sqrt(d)).astype(np.float32)
    W2 = (rng.standard_normal((h, d)) / np.sqrt(h)).astype(np.float32)
    p1 = {"X": X, "What": oracle.encode_weight(W1, E_W).astype(np.float32), "E_X": E_X, "D": D}
    p2 = {"What": oracle.encode_weight(W2, E_W).astype(np.float32), "E_X": E_X, "D": D}
    out = gu.mlp_forward(p1, p2, "f32", stl.STL_FLAG_GELU)
    ref = planes.gelu(X.astype(np.float64) @ W1.astype(np.float64)) @ W2.astype(np.float64)
    assert gu.rel(out, ref) <= gu.TOL["f32"]


def test_layer_pair_full_mlp_shape(gu):
    """m=16384, 1024 -> 4096 -> 1024, r=24, GELU: the one-pass path at the size the bench times."""
    import paper_2503_12211_amd as stl
    m, d, h, r = 16384, 1024, 4096, 24
    p1 = stl_synth.stl_problem(m, d, h, r, seed=stl_synth.SEEDS["C4_up"], dtype="bf16")
    p2 = stl_synth.stl_problem(m, h, d, r, seed=stl_synth.SEEDS["C4_down"], dtype="bf16")
    out = gu.mlp_forward(p1, p2, "bf16", stl.STL_FLAG_GELU)
    ref = planes.mlp_pair(p1["X"], p1["What"], p1["E_X"], p1["D"], p2["What"], p2["E_X"], p2["D"])
    assert gu.rel(out, ref) <= gu.TOL["bf16"]
