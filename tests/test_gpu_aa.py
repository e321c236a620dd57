"""GPU parity of the STL of two run-time encoded operands (stacked batch) against the fp64 oracle."""
import numpy as np
import pytest

import stl_synth
from oracle import bases, planes

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import gpu_util
    return gpu_util


def _ref_forward(p, nb):
    return planes.aa_forward(p["A"], p["B"], p["E_A"], p["E_B"], p["D"], nbatch=nb)


CASES = [
    # dtype, nbatch, m, k, n, r
    ("bf16", 3, 256, 128, 256, 32),     # register-staged matrix-core plane products on stacked problems
    ("bf16", 2, 512, 256, 384, 24),
    ("bf16", 4, 200, 64, 200, 32),      # attention-shaped: 200 tokens, head width 64 (50 tile rows: any-shape plane products)
    ("bf16", 3, 200, 200, 64, 16),      # attention x values
    ("bf16", 5, 72, 40, 56, 49),        # nothing a multiple of 32; two 32-plane groups
    ("bf16", 2, 36, 20, 28, 7),         # tile counts not multiples of 8: generic kernels
    ("bf16", 1, 128, 128, 128, 32),     # nbatch = 1
    ("bf16", 2, 1024, 640, 768, 16),    # stacked problems on the 256 x 256 tiles of the register-staged kernel
    ("f32", 3, 64, 32, 48, 17),
    ("f32", 2, 8, 4, 4, 1),
]


@pytest.mark.parametrize("dtype,nb,m,k,n,r", CASES)
def test_aa_forward_matches_oracle(gu, dtype, nb, m, k, n, r):
    p = stl_synth.aa_problem(nb, m, k, n, r, seed=8000 + m + k + n + r, dtype=dtype)
    got, Ah, Bh, Yh = gu.aa_forward(p["A"], p["B"], p["E_A"], p["E_B"], p["D"], nb, dtype, save=True)
    assert gu.rel(got, _ref_forward(p, nb)) <= gu.TOL[dtype]
    # the handed-back plane tensors are the stacked encodings and the per-problem plane products
    refA = planes.encode(p["A"], p["E_A"])
    refB = planes.encode(p["B"], p["E_B"])
    assert gu.rel(Ah, refA) <= gu.TOL[dtype] and gu.rel(Bh, refB) <= gu.TOL[dtype]
    M, K = m // 4, k // 4
    refY = np.concatenate([planes.plane_products(refA[:, b * M:(b + 1) * M], refB[:, b * K:(b + 1) * K]) for b in range(nb)],
                          axis=1)
    assert gu.rel(Yh, refY) <= gu.TOL[dtype]
    # without the saves the result is the same bits
    again = gu.aa_forward(p["A"], p["B"], p["E_A"], p["E_B"], p["D"], nb, dtype)
    assert np.array_equal(again, got)


@pytest.mark.parametrize("dtype,nb,m,k,n,r", CASES)
def test_aa_backward_matches_oracle(gu, dtype, nb, m, k, n, r):
    p = stl_synth.aa_problem(nb, m, k, n, r, seed=8100 + m + k + n + r, dtype=dtype, with_dC=True)
    ref = dict(zip(("dA", "dB", "dE_A", "dE_B", "dD"),
                   planes.aa_backward(p["A"], p["B"], p["E_A"], p["E_B"], p["D"], p["dC"], nbatch=nb)))
    got = gu.aa_backward(p["A"], p["B"], p["E_A"], p["E_B"], p["D"], p["dC"], nb, dtype)
    for name in ref:
        assert gu.rel(got[name], ref[name]) <= gu.TOL[dtype], name


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_aa_backward_saved_planes_accumulate_and_skips(gu, dtype):
    nb, m, k, n, r = 3, 128, 64, 96, 24
    p = stl_synth.aa_problem(nb, m, k, n, r, seed=8200, dtype=dtype, with_dC=True)
    args = (p["A"], p["B"], p["E_A"], p["E_B"], p["D"])
    ref = dict(zip(("dA", "dB", "dE_A", "dE_B", "dD"), planes.aa_backward(*args, p["dC"], nbatch=nb)))
    _, Ah, Bh, Yh = gu.aa_forward(*args, nb, dtype, save=True)
    base = gu.aa_backward(*args, p["dC"], nb, dtype)
    saved = gu.aa_backward(*args, p["dC"], nb, dtype, saved=(Ah, Bh, Yh))
    for name in ref:
        assert np.array_equal(saved[name], base[name]), name          # saved planes are the recomputed ones, bit for bit
    rng = np.random.default_rng(8201)
    init = [rng.standard_normal((r, 16)).astype(np.float32) * 10 for _ in range(3)]
    acc = gu.aa_backward(*args, p["dC"], nb, dtype, accumulate=1, init=init)
    for i, name in enumerate(("dE_A", "dE_B", "dD")):
        assert gu.rel(acc[name] - init[i], ref[name]) <= 2 * gu.TOL[dtype], name
    only_a = gu.aa_backward(*args, p["dC"], nb, dtype, skip=("dB", "dE_B", "dD"))
    assert np.isnan(only_a["dB"]).all() and np.isnan(only_a["dE_B"]).all() and np.isnan(only_a["dD"]).all()
    assert np.array_equal(only_a["dA"], base["dA"]) and np.array_equal(only_a["dE_A"], base["dE_A"])
    only_b = gu.aa_backward(*args, p["dC"], nb, dtype, skip=("dA", "dE_A"))
    assert np.isnan(only_b["dA"]).all() and np.array_equal(only_b["dB"], base["dB"])
    assert np.array_equal(only_b["dD"], base["dD"])


def test_aa_exact_basis_is_batched_matmul_fp32(gu):
    """At the rank-49 basis every stacked problem is the plain product A_b B_b, and its gradients the textbook ones."""
    nb, m, k, n = 3, 48, 32, 40
    E_A, E_B, D = (x.astype(np.float32) for x in bases.strassen_4x4())
    rng = np.random.default_rng(8300)
    A = rng.standard_normal((nb * m, k)).astype(np.float32)
    B = rng.standard_normal((nb * k, n)).astype(np.float32)
    dC = rng.standard_normal((nb * m, n)).astype(np.float32)
    got = gu.aa_forward(A, B, E_A, E_B, D, nb, "f32")
    g = gu.aa_backward(A, B, E_A, E_B, D, dC, nb, "f32")
    for b in range(nb):
        Ab, Bb, dCb = (x[b * s:(b + 1) * s].astype(np.float64) for x, s in ((A, m), (B, k), (dC, m)))
        assert gu.rel(got[b * m:(b + 1) * m], Ab @ Bb) <= 1e-5
        assert gu.rel(g["dA"][b * m:(b + 1) * m], dCb @ Bb.T) <= 1e-5
        assert gu.rel(g["dB"][b * k:(b + 1) * k], Ab.T @ dCb) <= 1e-5


def test_aa_attention_shape_full_size_sampled(gu):
    """The benchmarked attention-shaped workload (nbatch = 32 heads, 1024 tokens, head width 128): sampled problems
    against the oracle, the rest against properties (finite, right scale)."""
    nb, m, k, n, r = 32, 1024, 128, 1024, 32
    p = stl_synth.aa_problem(nb, m, k, n, r, seed=8400, dtype="bf16")
    got = gu.aa_forward(p["A"], p["B"], p["E_A"], p["E_B"], p["D"], nb, "bf16")
    assert np.isfinite(got).all()
    for b in (0, 13, 31):
        ref = planes.aa_forward(p["A"][b * m:(b + 1) * m], p["B"][b * k:(b + 1) * k], p["E_A"], p["E_B"], p["D"])
        assert gu.rel(got[b * m:(b + 1) * m], ref) <= gu.TOL["bf16"], b


@pytest.mark.parametrize("dtype,nb,m,k,n,r", [
    ("bf16", 3, 256, 128, 256, 32),
    ("bf16", 32, 1024, 128, 1024, 32),     # attention scores Q K^T with K as it is stored (tokens x width), full size
    ("bf16", 2, 200, 64, 72, 24),          # 50 / 18 tile rows: any-shape kernels
    ("bf16", 4, 64, 96, 40, 49),
    ("f32", 3, 48, 32, 40, 17),
])
def test_aa_transposed_second_operand(gu, dtype, nb, m, k, n, r):
    """STL_FLAG_B_TRANSPOSED: B is stored (nb*n, k); forward, the handed-back planes ([p][J][L]) and all gradients."""
    import paper_2503_12211_amd as stl
    FL = stl.STL_FLAG_B_TRANSPOSED
    p = stl_synth.aa_problem(nb, m, k, n, r, seed=8500 + m + k + n + r, dtype=dtype, with_dC=True)
    Bt = np.ascontiguousarray(np.concatenate([p["B"][b * k:(b + 1) * k].T for b in range(nb)], axis=0))    # (nb*n, k)
    args = (p["A"], Bt, p["E_A"], p["E_B"], p["D"])
    full = nb * m * n <= 1 << 22
    got, Ah, Bh, Yh = gu.aa_forward(*args, nb, dtype, flags=FL, save=True)
    if full:
        ref = planes.aa_forward(*args, nbatch=nb, b_transposed=True)
        assert gu.rel(got, ref) <= gu.TOL[dtype]
        # the stored planes are the encoding of B^T with tile rows and columns swapped
        refB = planes.encode(p["B"], p["E_B"])                                   # (r, nb*K, N)
        K, N = k // 4, n // 4
        refBt = np.concatenate([refB[:, b * K:(b + 1) * K].transpose(0, 2, 1) for b in range(nb)], axis=1)
        assert gu.rel(Bh, refBt) <= gu.TOL[dtype]
        g = gu.aa_backward(*args, p["dC"], nb, dtype, flags=FL)
        refs = dict(zip(("dA", "dB", "dE_A", "dE_B", "dD"), planes.aa_backward(*args, p["dC"], nbatch=nb, b_transposed=True)))
        for name in refs:
            assert gu.rel(g[name], refs[name]) <= gu.TOL[dtype], name
        sv = gu.aa_backward(*args, p["dC"], nb, dtype, flags=FL, saved=(Ah, Bh, Yh))
        for name in refs:
            assert np.array_equal(sv[name], g[name]), name
        rng = np.random.default_rng(1)
        init = [rng.standard_normal((r, 16)).astype(np.float32) * 10 for _ in range(3)]
        acc = gu.aa_backward(*args, p["dC"], nb, dtype, flags=FL, accumulate=1, init=init)
        assert gu.rel(acc["dE_B"] - init[1], refs["dE_B"]) <= 2 * gu.TOL[dtype]
    else:
        # the same product with B given the other way round must agree bit for bit in C (same planes, same sums)
        assert np.isfinite(got).all()
        plain = gu.aa_forward(p["A"], p["B"], p["E_A"], p["E_B"], p["D"], nb, dtype)
        for b in (0, 17, 31):
            ref = planes.aa_forward(p["A"][b * m:(b + 1) * m], Bt[b * n:(b + 1) * n], p["E_A"], p["E_B"], p["D"], b_transposed=True)
            assert gu.rel(got[b * m:(b + 1) * m], ref) <= gu.TOL[dtype], b
        assert gu.rel(got, plain) <= 2e-3
