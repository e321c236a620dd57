"""GPU parity: stl_forward / stl_encode_weight / the three stage entry points against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
import stl_synth
from oracle import bases, planes

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import gpu_util
    return gpu_util


def test_config1_fp32_strassen_exact(gu):
    """fp32, m=k=n=256, r=49 two-level Strassen basis: output equals X.W to fp32 rounding."""
    import paper_2503_12211_amd as stl
    cfg, p = stl_synth.config_problem("C1")
    E_X, E_W, D = bases.strassen_4x4()
    prob = stl.Problem(256, 256, 256, 49, stl.STL_F32)
    W = gu.dev(p["W"], "f32")
    What = torch.empty((49, 64, 64), dtype=torch.float32, device="cuda")
    stl.stl_encode_weight(prob, W, gu.dev(E_W, "f32"), What)
    torch.cuda.synchronize()
    What_ref = oracle.encode_weight(p["W"], E_W)
    assert gu.rel(gu.host(What), What_ref) <= 1e-6
    q = {"X": p["X"], "What": gu.host(What), "E_X": E_X, "D": D}
    C = gu.forward(q, "f32")
    ref = oracle.forward(p["X"], What_ref, E_X, D)
    exact = p["X"].astype(np.float64) @ p["W"].astype(np.float64)
    assert gu.rel(ref, exact) < 1e-13
    assert gu.rel(C, ref) <= gu.TOL["f32"]
    assert gu.rel(C, exact) <= gu.TOL["f32"]


SMALL = [  # (m, k, n, r): single tile, ragged everything, several blocks + ragged tail
    (4, 4, 4, 1), (4, 8, 4, 64), (20, 36, 28, 7), (68, 132, 76, 24), (260, 132, 520, 32), (132, 260, 68, 49),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SMALL)
def test_forward_small_and_ragged(gu, dtype, shape):
    m, k, n, r = shape
    p = stl_synth.stl_problem(m, k, n, r, seed=11 + m + r, dtype=dtype)
    C = gu.forward(p, dtype)
    ref = oracle.forward(p["X"], p["What"], p["E_X"], p["D"])
    assert gu.rel(C, ref) <= gu.TOL[dtype]


MFMA_SHAPES = [  # tile counts are multiples of 8 (matrix-core path), not multiples of the block sizes
    (1056, 544, 800, 5), (512, 1024, 512, 32), (288, 2080, 1312, 16), (2048, 256, 96, 64), (32, 32, 32, 3),
    (1024, 512, 1056, 49), (1152, 1152, 1152, 3), (1184, 1152, 1216, 2),
]


@pytest.mark.parametrize("shape", MFMA_SHAPES)
def test_forward_bf16_matrix_core_shapes(gu, shape):
    m, k, n, r = shape
    p = stl_synth.stl_problem(m, k, n, r, seed=23 + n + r, dtype="bf16")
    C, Y = gu.forward(p, "bf16", save_yhat=True)
    Cref, Yref = planes.forward(p["X"], p["What"], p["E_X"], p["D"], return_yhat=True)
    assert gu.rel(Y, Yref) <= gu.TOL["bf16"]
    assert gu.rel(C, Cref) <= gu.TOL["bf16"]
    # literal Eq. (2) on a ragged corner block
    M, N = m // 4, n // 4
    blk = oracle.forward_block(p["X"], p["What"], p["E_X"], p["D"], max(M - 5, 0), M, max(N - 3, 0), N)
    assert gu.rel(C[4 * max(M - 5, 0):, 4 * max(N - 3, 0):], blk) <= 2 * gu.TOL["bf16"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stage_entry_points(gu, dtype):
    """Each of Algorithm 1's three steps against the oracle's step, fed the same (rounded) operands."""
    import paper_2503_12211_amd as stl
    m, k, n, r = 136, 264, 72, 24
    p = stl_synth.stl_problem(m, k, n, r, seed=5, dtype=dtype)
    prob = stl.Problem(m, k, n, r, gu.STL_DT[dtype])
    tdt = gu.TORCH_DT[dtype]
    X, What, E_X, D = (gu.dev(p[s], dtype) for s in ("X", "What", "E_X", "D"))
    Xhat = gu.planes_buffer(r, m // 4, k // 4, dtype)
    stl.stl_encode_activation(prob, X, E_X, Xhat)
    torch.cuda.synchronize()
    Xh = gu.planes_to_host(Xhat, r, m // 4, k // 4)
    assert gu.rel(Xh, oracle.encode_x(p["X"], p["E_X"])) <= gu.TOL[dtype]
    Yhat = gu.planes_buffer(r, m // 4, n // 4, dtype)
    stl.stl_plane_matmul(prob, Xhat, What, Yhat)
    torch.cuda.synchronize()
    Yh = gu.planes_to_host(Yhat, r, m // 4, n // 4)
    assert gu.rel(Yh, planes.plane_products(Xh, p["What"])) <= gu.TOL[dtype]
    C = torch.empty((m, n), dtype=tdt, device="cuda")
    stl.stl_decode(prob, Yhat, D, C)
    torch.cuda.synchronize()
    assert gu.rel(gu.host(C), planes.decode(Yh, p["D"])) <= gu.TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gelu_epilogue(gu, dtype):
    import paper_2503_12211_amd as stl
    p = stl_synth.stl_problem(64, 96, 160, 24, seed=9, dtype=dtype)
    C = gu.forward(p, dtype, flags=stl.STL_FLAG_GELU)
    ref = planes.gelu(oracle.forward(p["X"], p["What"], p["E_X"], p["D"]))
    assert gu.rel(C, ref) <= gu.TOL[dtype]


def test_gelu_entrywise_accuracy_fp32(gu):
    """The device GELU entry by entry: with r = 16 and D the identity the decode of planes holding a grid of
    values h is gelu(h) itself.  fp32 storage; the bar covers the whole range, tails included."""
    import torch
    import paper_2503_12211_amd as stl
    h = np.linspace(-9.0, 9.0, 16 * 8 * 8).astype(np.float32).reshape(16, 8, 8)
    prob = stl.Problem(32, 32, 32, 16, stl.STL_F32)
    Yhat, D = gu.planes_to_dev(h, "f32"), gu.dev(np.eye(16, dtype=np.float32), "f32")
    C = torch.empty((32, 32), dtype=torch.float32, device="cuda")
    stl.stl_decode(prob, Yhat, D, C, stl.STL_FLAG_GELU)
    torch.cuda.synchronize()
    got = planes.tiles(gu.host(C)).transpose(2, 0, 1)              # back to (entry = plane, I, J)
    want = planes.gelu(h.astype(np.float64))
    assert np.abs(got - want).max() <= 2e-7 * 9.0
    assert np.all(np.abs(got - want) <= 2e-7 * np.maximum(np.abs(h), 1.0))


def test_exact_bases_bf16_inputs(gu):
    """bf16 storage, trivial r=64 basis, small-integer inputs: every intermediate is exactly
    representable, so the result must equal X.W exactly."""
    import paper_2503_12211_amd as stl
    rng = np.random.default_rng(3)
    m, k, n = 64, 32, 96
    X = rng.integers(-3, 4, size=(m, k)).astype(np.float32)
    W = rng.integers(-2, 3, size=(k, n)).astype(np.float32)
    E_X, E_W, D = bases.trivial(4)
    prob = stl.Problem(m, k, n, 64, stl.STL_BF16)
    What = torch.empty((64, k // 4, n // 4), dtype=torch.bfloat16, device="cuda")
    stl.stl_encode_weight(prob, gu.dev(W, "bf16"), gu.dev(E_W, "bf16"), What)
    C = gu.forward({"X": X, "What": gu.host(What), "E_X": E_X, "D": D}, "bf16")
    assert np.array_equal(C, (X @ W).astype(np.float64))


def test_config2_full_size(gu):
    """bf16, m=k=n=4096, r=32 at full size: whole output against the plane oracle, and sampled
    8x8-tile blocks against literal Eq. (2)."""
    cfg, p = stl_synth.config_problem("C2")
    C = gu.forward(p, "bf16")
    Cref = planes.forward(p["X"], p["What"], p["E_X"], p["D"])
    gu.check(C, Cref, "bf16", "C2 C")
    rng = np.random.default_rng(0)
    for _ in range(3):
        I0, J0 = (int(v) for v in rng.integers(0, 1024 - 8, size=2))
        blk = oracle.forward_block(p["X"], p["What"], p["E_X"], p["D"], I0, I0 + 8, J0, J0 + 8)
        assert gu.rel(C[4 * I0:4 * I0 + 32, 4 * J0:4 * J0 + 32], blk) <= 2 * gu.TOL["bf16"]
    # statistical property of the workload: Var C = sum_p |D_p|^2 |E_p|^2-weighted, order r/64
    assert 0.2 < C.var() / (32 / 64) < 5.0


@pytest.mark.parametrize("r", [8, 16, 24, 32, 49, 64])
def test_config3_rank_sweep_full_size(gu, r):
    """bf16, m=8192, k=n=4096 at every rank of the sweep, the forward as the sweep times it (nothing saved, row slabs):
    output rows are independent, so whole row slabs are checked against the plane oracle run on those rows of X alone
    (norm, every entry, every 256 x 256 block and tile row), and sampled 8x8-tile blocks against literal Eq. (2).  At
    r = 32, the rank of the timed step, the whole output is compared."""
    p = stl_synth.stl_problem(8192, 4096, 4096, r, seed=stl_synth.SEEDS["C3"] + 100 * r, dtype="bf16")
    C = gu.forward(p, "bf16")
    assert np.isfinite(C).all()
    for r0, r1 in (((0, 8192),) if r == 32 else ((0, 256), (4096 - 128, 4096 + 128), (8192 - 64, 8192))):
        ref = planes.forward(p["X"][r0:r1], p["What"], p["E_X"], p["D"])
        gu.check(C[r0:r1], ref, "bf16", f"C3 r={r} rows {r0}:{r1}")
    rng = np.random.default_rng(r)
    for _ in range(2):
        I0, J0 = int(rng.integers(0, 2048 - 8)), int(rng.integers(0, 1024 - 8))
        blk = oracle.forward_block(p["X"], p["What"], p["E_X"], p["D"], I0, I0 + 8, J0, J0 + 8)
        assert gu.rel(C[4 * I0:4 * I0 + 32, 4 * J0:4 * J0 + 32], blk) <= 2 * gu.TOL["bf16"]
    assert 0.2 < C.var() / (r / 64) < 5.0


def test_forward_row_slabs_with_ragged_tail(gu):
    """m = 8736 (2184 tile rows), k = n = 4096, r = 32 without saved planes: the forward takes 1024-tile-row slabs that
    share the plane scratch, the last one 136 tile rows long; rows around every slab boundary and the tail are checked
    against the plane oracle run on those rows alone, and the result must equal the single-pass result bit for bit."""
    p = stl_synth.stl_problem(8736, 4096, 4096, 32, seed=4321, dtype="bf16")
    C = gu.forward(p, "bf16")
    assert np.isfinite(C).all()
    for r0, r1 in ((0, 64), (4096 - 64, 4096 + 64), (8192 - 64, 8192 + 64), (8736 - 100, 8736)):
        ref = planes.forward(p["X"][r0:r1], p["What"], p["E_X"], p["D"])
        assert gu.rel(C[r0:r1], ref) <= gu.TOL["bf16"], (r0, r1)
    C1, _ = gu.forward(p, "bf16", save_yhat=True)              # saving Yhat keeps the whole problem in one pass
    assert np.array_equal(C, C1)


def test_forward_is_deterministic(gu):
    p = stl_synth.stl_problem(512, 512, 512, 32, seed=77, dtype="bf16")
    a = gu.forward(p, "bf16")
    b = gu.forward(p, "bf16")
    assert np.array_equal(a, b)


VARIANT_SHAPES = [  # (m, k, n, r): k % 64 == 0, n % 32 == 0; blocks hang over the edge in m and n
    (128, 64, 32, 1), (132, 128, 96, 7), (1056, 576, 800, 24), (516, 1024, 544, 32), (2048, 512, 1024, 8),
]


@pytest.mark.parametrize("variant", ["epilogue", "fused"])
@pytest.mark.parametrize("shape", VARIANT_SHAPES)
def test_forward_block_resident_variants(gu, variant, shape):
    """Decode-in-epilogue and single-launch fused forward against Eq. (2); Yhat written on request."""
    import paper_2503_12211_amd as stl
    m, k, n, r = shape
    flag = {"epilogue": stl.STL_FLAG_EPILOGUE, "fused": stl.STL_FLAG_FUSED}[variant]
    p = stl_synth.stl_problem(m, k, n, r, seed=301 + m + r, dtype="bf16")
    Cref, Yref = planes.forward(p["X"], p["What"], p["E_X"], p["D"], return_yhat=True)
    C, Y = gu.forward(p, "bf16", flags=flag, save_yhat=True)
    assert gu.rel(C, Cref) <= gu.TOL["bf16"]
    assert gu.rel(Y, Yref) <= gu.TOL["bf16"]
    C2 = gu.forward(p, "bf16", flags=flag | stl.STL_FLAG_GELU)
    assert gu.rel(C2, planes.gelu(Cref)) <= gu.TOL["bf16"]
    M, N = m // 4, n // 4
    blk = oracle.forward_block(p["X"], p["What"], p["E_X"], p["D"], max(M - 3, 0), M, max(N - 5, 0), N)
    assert gu.rel(C[4 * max(M - 3, 0):, 4 * max(N - 5, 0):], blk) <= 2 * gu.TOL["bf16"]


@pytest.mark.parametrize("shape", [(128, 256, 256, 8), (128, 512, 512, 8), (64, 512, 512, 16), (256, 1024, 1024, 8)])
def test_automatic_variant_choice_on_launch_bound_shapes(gu, shape):
    """Problems of a few microseconds: the automatic choice takes the single-launch variant up to about four million
    tile products (and the three-launch path above); either way the result is the operator's, and equal bit for bit
    to the variant it stands for."""
    import paper_2503_12211_amd as stl
    m, k, n, r = shape
    p = stl_synth.stl_problem(m, k, n, r, seed=611 + m + k, dtype="bf16")
    ref = planes.forward(p["X"], p["What"], p["E_X"], p["D"])
    auto = gu.forward(p, "bf16", flags=stl.STL_FLAG_AUTO)
    gu.check(auto, ref, "bf16", f"auto {shape}")
    small = (m // 4) * (k // 4) * (n // 4) * r <= 4.2e6
    same = gu.forward(p, "bf16", flags=stl.STL_FLAG_FUSED if small else stl.STL_FLAG_UNFUSED)
    assert np.array_equal(auto, same)
    auto_y, Y = gu.forward(p, "bf16", flags=stl.STL_FLAG_AUTO, save_yhat=True)
    assert np.array_equal(auto_y, auto)
    assert gu.rel(Y, planes.forward(p["X"], p["What"], p["E_X"], p["D"], return_yhat=True)[1]) <= gu.TOL["bf16"]


def test_forward_variants_agree_at_config2_shape(gu):
    """bf16, m=k=n=4096, r=32: all three forward variants against the plane oracle."""
    import paper_2503_12211_amd as stl
    cfg, p = stl_synth.config_problem("C2")
    Cref = planes.forward(p["X"], p["What"], p["E_X"], p["D"])
    for flag in (stl.STL_FLAG_UNFUSED, stl.STL_FLAG_EPILOGUE, stl.STL_FLAG_FUSED):
        assert gu.rel(gu.forward(p, "bf16", flags=flag), Cref) <= gu.TOL["bf16"], flag


@pytest.mark.parametrize("full", [False, True])
def test_mlp_shaped_pair(gu, full):
    """Up-projection, GELU (in the first layer's decode), down-projection, r=24; the hidden activation is rounded
    to bf16 between the layers on the GPU, the oracle stays in fp64 throughout."""
    import paper_2503_12211_amd as stl
    m, d, h, r = (16384, 1024, 4096, 24) if full else (512, 256, 1024, 24)
    p1 = stl_synth.stl_problem(m, d, h, r, seed=stl_synth.SEEDS["C4_up"], dtype="bf16")
    p2 = stl_synth.stl_problem(m, h, d, r, seed=stl_synth.SEEDS["C4_down"], dtype="bf16")
    H = gu.forward(p1, "bf16", flags=stl.STL_FLAG_GELU)
    q2 = dict(p2)
    q2["X"] = H.astype(np.float32)
    out = gu.forward(q2, "bf16")
    ref = planes.mlp_pair(p1["X"], p1["What"], p1["E_X"], p1["D"], p2["What"], p2["E_X"], p2["D"])
    assert gu.rel(out, ref) <= gu.TOL["bf16"]
