"""GPU parity of the ragged-row path (images whose row count the tile size does not divide) against the fp64 oracle."""
import numpy as np
import pytest

import stl_synth
from oracle import bases, planes

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import gpu_util
    return gpu_util


NAMES = ("dX", "dWhat", "dE_X", "dD", "dfold")

CASES = [
    # dtype, nimg, rows, k, n, r
    ("bf16", 8, 197, 256, 512, 32),     # the paper's token count; matrix-core tile maps, pipelined plane products
    ("bf16", 3, 198, 64, 96, 24),       # two remaining rows
    ("bf16", 5, 39, 96, 160, 49),       # three remaining rows, two 32-plane groups
    ("bf16", 4, 21, 40, 36, 7),         # tile columns not a multiple of 8: generic kernels
    ("bf16", 1, 5, 32, 32, 16),         # a single image of two tile rows
    ("f32", 3, 13, 24, 20, 11),
    ("f32", 2, 6, 8, 4, 1),
    ("bf16", 4, 64, 64, 64, 32),        # rows divisible by 4: the plain operator
    ("f32", 2, 8, 8, 8, 3),
]


@pytest.mark.parametrize("dtype,nimg,rows,k,n,r", CASES)
def test_ragged_forward_matches_oracle(gu, dtype, nimg, rows, k, n, r):
    p = stl_synth.ragged_problem(nimg, rows, k, n, r, seed=9000 + rows + k + n + r, dtype=dtype)
    ref = planes.ragged_forward(p["X"], p["What"], p["E_X"], p["D"], p["fold"], rows)
    got, Xh, Yh = gu.ragged_forward(p, rows, dtype, save=True)
    assert got.shape == ref.shape and np.isfinite(got).all()
    assert gu.rel(got, ref) <= gu.TOL[dtype]
    Mt, nrho = (rows + 3) // 4, rows % 4
    if nrho:
        # the folded rows on their own (a slip there would drown in the norm of the whole output)
        last = np.concatenate([np.arange(i * rows + 4 * (Mt - 1), (i + 1) * rows) for i in range(nimg)])
        assert gu.rel(got[last], ref[last]) <= gu.TOL[dtype]
    refX = planes.encode(planes.pad_rows(p["X"], rows), p["E_X"])
    assert gu.rel(Xh, refX) <= gu.TOL[dtype]
    assert gu.rel(Yh, planes.plane_products(refX, p["What"])) <= gu.TOL[dtype]
    assert np.array_equal(gu.ragged_forward(p, rows, dtype), got)


@pytest.mark.parametrize("dtype,nimg,rows,k,n,r", CASES)
def test_ragged_backward_matches_oracle(gu, dtype, nimg, rows, k, n, r):
    p = stl_synth.ragged_problem(nimg, rows, k, n, r, seed=9100 + rows + k + n + r, dtype=dtype, with_dC=True)
    ref = dict(zip(NAMES, planes.ragged_backward(p["X"], p["What"], p["E_X"], p["D"], p["fold"], p["dC"], rows)))
    got = gu.ragged_backward(p, rows, dtype)
    for name in NAMES:
        if ref[name] is None:
            assert got[name] is None
            continue
        assert np.isfinite(got[name]).all(), name
        assert gu.rel(got[name], ref[name]) <= gu.TOL[dtype], name


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ragged_saved_planes_accumulate_and_skips(gu, dtype):
    nimg, rows, k, n, r = 4, 29, 64, 96, 24
    p = stl_synth.ragged_problem(nimg, rows, k, n, r, seed=9200, dtype=dtype, with_dC=True)
    ref = dict(zip(NAMES, planes.ragged_backward(p["X"], p["What"], p["E_X"], p["D"], p["fold"], p["dC"], rows)))
    _, Xh, Yh = gu.ragged_forward(p, rows, dtype, save=True)
    base = gu.ragged_backward(p, rows, dtype)
    saved = gu.ragged_backward(p, rows, dtype, saved=(Xh, Yh))
    for name in NAMES:
        assert np.array_equal(saved[name], base[name]), name
    rng = np.random.default_rng(9201)
    init = [rng.standard_normal(s).astype(np.float32) * 10 for s in ((r, k // 4, n // 4), (r, 16), (r, 16), (1, 4))]
    acc = gu.ragged_backward(p, rows, dtype, accumulate=1, init=init)
    for i, name in enumerate(NAMES[1:]):
        assert gu.rel(acc[name] - init[i], ref[name]) <= 3 * gu.TOL[dtype], name
    only = gu.ragged_backward(p, rows, dtype, skip=("dX", "dWhat", "dE_X", "dD"))
    assert np.array_equal(only["dfold"], base["dfold"])
    assert all(np.isnan(only[nm]).all() for nm in ("dX", "dWhat", "dE_X", "dD"))
    nofold = gu.ragged_backward(p, rows, dtype, skip=("dfold",))
    for name in NAMES[:4]:
        assert np.array_equal(nofold[name], base[name]), name


def test_ragged_exact_basis_closed_form_fp32(gu):
    """At the rank-49 basis the padded operator is X_pad @ W: complete tile rows give X @ W, the folded row of each
    image is fold[0][0] * (x_last @ W) because the null rows contribute nothing."""
    import oracle
    nimg, rows, k, n = 3, 9, 16, 12
    E_X, E_W, D = bases.strassen_4x4()
    rng = np.random.default_rng(9300)
    X = rng.standard_normal((nimg * rows, k)).astype(np.float32)
    W = rng.standard_normal((k, n)).astype(np.float32)
    fold = rng.standard_normal((1, 4)).astype(np.float32)
    p = {"X": X, "What": oracle.encode_weight(W, E_W).astype(np.float32), "E_X": E_X.astype(np.float32),
         "D": D.astype(np.float32), "fold": fold}
    got = gu.ragged_forward(p, rows, "f32")
    want = X.astype(np.float64) @ W.astype(np.float64)
    for i in range(nimg):
        want[rows * i + 8] *= float(fold[0, 0])
    assert gu.rel(got, want) <= 1e-5


def test_ragged_vit_shape_full_size_sampled(gu):
    """The benchmarked ViT-shaped workload (256 images of 197 tokens, 768 -> 3072): sampled images against the oracle."""
    nimg, rows, k, n, r = 256, 197, 768, 3072, 32
    p = stl_synth.ragged_problem(nimg, rows, k, n, r, seed=9400, dtype="bf16")
    got = gu.ragged_forward(p, rows, "bf16")
    assert np.isfinite(got).all()
    for i in (0, 101, 255):
        sub = dict(p, X=p["X"][i * rows:(i + 1) * rows])
        ref = planes.ragged_forward(sub["X"], p["What"], p["E_X"], p["D"], p["fold"], rows)
        assert gu.rel(got[i * rows:(i + 1) * rows], ref) <= gu.TOL["bf16"], i
        assert gu.rel(got[(i + 1) * rows - 1], ref[-1]) <= gu.TOL["bf16"], i
