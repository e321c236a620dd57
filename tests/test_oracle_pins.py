"""Pins for the fp64 oracle: what the paper and the mathematics fix, independent of the oracle.

Each test is chosen so that a plausible slip in oracle/ (dropped term, wrong sign or
index, transposed operand, wrong vec order, decode before the L-sum) fails it.
"""
import numpy as np
import pytest

import oracle
from oracle import bases, planes

RNG = np.random.default_rng(7)


def rel(a, b):
    return np.linalg.norm(np.asarray(a) - np.asarray(b)) / max(np.linalg.norm(b), 1e-300)


def rand_problem(m, k, n, r, t=4, rng=RNG):
    X = rng.standard_normal((m, k))
    W = rng.standard_normal((k, n))
    E_X = rng.standard_normal((r, t * t))
    E_W = rng.standard_normal((r, t * t))
    D = rng.standard_normal((r, t * t))
    return X, W, E_X, E_W, D


# ---------------------------------------------------------------- exact bases
def matmul_tensor(t):
    """T[a*t+l, l'*t+b, a'*t+b'] = [l==l'][a==a'][b==b'] : the t x t product as a 3-tensor."""
    T = np.zeros((t * t,) * 3)
    for a in range(t):
        for l in range(t):
            for b in range(t):
                T[a * t + l, l * t + b, a * t + b] = 1.0
    return T


@pytest.mark.parametrize("name,t,r", [("strassen2", 2, 7), ("strassen4", 4, 49),
                                      ("trivial2", 2, 8), ("trivial4", 4, 64)])
def test_basis_is_matmul_tensor(name, t, r):
    """Integer-exact: sum_p E_X[p,.] (x) E_W[p,.] (x) D[p,.] is the t x t product tensor."""
    E_X, E_W, D = {"strassen2": bases.strassen_2x2, "strassen4": bases.strassen_4x4,
                   "trivial2": lambda: bases.trivial(2), "trivial4": lambda: bases.trivial(4)}[name]()
    assert E_X.shape == E_W.shape == D.shape == (r, t * t)
    T = np.einsum("pa,pb,pc->abc", E_X, E_W, D)
    assert np.array_equal(T, matmul_tensor(t))


def test_strassen4_is_sparse_pm1():
    for F in bases.strassen_4x4():
        assert set(np.unique(F)) <= {-1.0, 0.0, 1.0}
        assert np.count_nonzero(F) == 144


@pytest.mark.parametrize("t,basis", [(2, bases.strassen_2x2), (4, bases.strassen_4x4),
                                     (2, lambda: bases.trivial(2)), (4, lambda: bases.trivial(4))])
@pytest.mark.parametrize("shape", [(4, 4, 4), (8, 12, 16), (20, 8, 12), (32, 32, 32)])
def test_exact_bases_reproduce_matmul(t, basis, shape):
    """r=t^3 trivial and Strassen bases give X@W (library product) for any tile counts."""
    m, k, n = shape
    E_X, E_W, D = basis()
    X = RNG.standard_normal((m, k))
    W = RNG.standard_normal((k, n))
    What = oracle.encode_weight(W, E_W, t)
    assert rel(oracle.forward(X, What, E_X, D, t), X @ W) < 1e-13
    assert rel(planes.forward(X, planes.encode(W, E_W, t), E_X, D, t), X @ W) < 1e-13


def test_config1_shape_exact():
    """The fp32 workload's shape (256^3, r=49) in fp64: equals X@W; finishes well under a second."""
    import time
    E_X, E_W, D = bases.strassen_4x4()
    X = RNG.standard_normal((256, 256))
    W = RNG.standard_normal((256, 256))
    What = oracle.encode_weight(W, E_W)
    t0 = time.perf_counter()
    C = oracle.forward(X, What, E_X, D)
    dt = time.perf_counter() - t0
    assert rel(C, X @ W) < 1e-13
    assert dt < 5.0


# ------------------------------------------------- random bases: tensor contraction
@pytest.mark.parametrize("t,r,shape", [(4, 5, (8, 8, 8)), (4, 24, (12, 8, 16)), (2, 3, (6, 4, 8)),
                                       (4, 1, (4, 4, 4)), (3, 10, (6, 9, 3))])
def test_random_basis_equals_bilinear_tensor_contraction(t, r, shape):
    """Contract p first (the bilinear-map tensor of the tile-level normal form), then tiles:
    a different order of operations from both oracle formulations."""
    m, k, n = shape
    X, W, E_X, E_W, D = rand_problem(m, k, n, r, t)
    T = np.einsum("pa,pb,pc->abc", E_X, E_W, D)
    x = X.reshape(m // t, t, k // t, t).transpose(0, 2, 1, 3).reshape(m // t, k // t, t * t)
    w = W.reshape(k // t, t, n // t, t).transpose(0, 2, 1, 3).reshape(k // t, n // t, t * t)
    c = np.einsum("abc,ILa,LJb->IJc", T, x, w)
    C_ref = c.reshape(m // t, n // t, t, t).transpose(0, 2, 1, 3).reshape(m, n)
    What = oracle.encode_weight(W, E_W, t)
    assert rel(oracle.forward(X, What, E_X, D, t), C_ref) < 1e-13
    assert rel(planes.forward(X, What, E_X, D, t), C_ref) < 1e-13


def test_single_tile_is_normal_form():
    """m=k=n=t: Eq. (2) collapses to the normal form D^T((E_X vec X) . (E_W vec W)), by hand."""
    X, W, E_X, E_W, D = rand_problem(4, 4, 4, 9)
    expect = np.zeros(16)
    for p in range(9):
        ex = sum(E_X[p, 4 * a + b] * X[a, b] for a in range(4) for b in range(4))
        ew = sum(E_W[p, 4 * a + b] * W[a, b] for a in range(4) for b in range(4))
        expect += D[p] * ex * ew
    C = oracle.forward(X, oracle.encode_weight(W, E_W), E_X, D)
    assert rel(C.reshape(16), expect) < 1e-13


# ------------------------------------------------------------ two formulations agree
@pytest.mark.parametrize("shape,r", [((16, 24, 8), 7), ((64, 32, 48), 32), ((36, 20, 28), 49)])
def test_claim_3_4_two_formulations_agree(shape, r):
    m, k, n = shape
    X, W, E_X, E_W, D = rand_problem(m, k, n, r)
    What = oracle.encode_weight(W, E_W)
    assert rel(What, planes.encode(W, E_W)) < 1e-14
    assert rel(oracle.encode_x(X, E_X), planes.encode(X, E_X)) < 1e-14
    C1, Y1 = oracle.forward(X, What, E_X, D, return_yhat=True)
    C2, Y2 = planes.forward(X, What, E_X, D, return_yhat=True)
    assert rel(C1, C2) < 1e-13 and rel(Y1, Y2) < 1e-13
    dC = RNG.standard_normal((m, n))
    for g1, g2 in zip(oracle.backward(X, What, E_X, D, dC), planes.backward(X, What, E_X, D, dC)):
        assert rel(g1, g2) < 1e-13


def test_forward_block_matches_full():
    X, W, E_X, E_W, D = rand_problem(32, 16, 40, 6)
    What = oracle.encode_weight(W, E_W)
    C = oracle.forward(X, What, E_X, D)
    blk = oracle.forward_block(X, What, E_X, D, 2, 7, 3, 9)
    assert np.array_equal(blk, C[8:28, 12:36])


# -------------------------------------------------------------- algebraic invariants
def test_bilinearity_and_linearity_in_bases():
    X, W, E_X, E_W, D = rand_problem(12, 16, 8, 11)
    X2 = RNG.standard_normal(X.shape)
    What = oracle.encode_weight(W, E_W)
    What2 = RNG.standard_normal(What.shape)
    E2 = RNG.standard_normal(E_X.shape)
    D2 = RNG.standard_normal(D.shape)
    a, b = 0.7, -1.9
    f = oracle.forward
    assert rel(f(a * X + b * X2, What, E_X, D), a * f(X, What, E_X, D) + b * f(X2, What, E_X, D)) < 1e-13
    assert rel(f(X, a * What + b * What2, E_X, D), a * f(X, What, E_X, D) + b * f(X, What2, E_X, D)) < 1e-13
    assert rel(f(X, What, a * E_X + b * E2, D), a * f(X, What, E_X, D) + b * f(X, What, E2, D)) < 1e-13
    assert rel(f(X, What, E_X, a * D + b * D2), a * f(X, What, E_X, D) + b * f(X, What, E_X, D2)) < 1e-13


def test_decode_is_applied_after_the_sum():
    """Decode linearity: splitting the contraction range and adding decoded halves is the same."""
    X, W, E_X, E_W, D = rand_problem(8, 24, 8, 10)
    What = oracle.encode_weight(W, E_W)
    full = oracle.forward(X, What, E_X, D)
    h1 = oracle.forward(X[:, :8], What[:, :2], E_X, D)
    h2 = oracle.forward(X[:, 8:], What[:, 2:], E_X, D)
    assert rel(h1 + h2, full) < 1e-13


def test_additivity_over_rank_subsets_and_random_strassen_rows():
    """Row subsets of the rank-49 basis (the appendix's initialisation): parts add up to X@W."""
    E_X, E_W, D = bases.strassen_4x4()
    X = RNG.standard_normal((16, 12))
    W = RNG.standard_normal((12, 20))
    perm = RNG.permutation(49)
    S1, S2 = perm[:20], perm[20:]
    parts = []
    for S in (S1, S2):
        What = oracle.encode_weight(W, E_W[S])
        parts.append(oracle.forward(X, What, E_X[S], D[S]))
    assert rel(parts[0] + parts[1], X @ W) < 1e-13
    assert rel(parts[0], X @ W) > 1e-2     # a strict subset is not exact


def test_gauge_invariance():
    X, W, E_X, E_W, D = rand_problem(8, 8, 12, 13)
    What = oracle.encode_weight(W, E_W)
    C = oracle.forward(X, What, E_X, D)
    s = RNG.uniform(0.5, 2.0, size=13)
    assert rel(oracle.forward(X, What, E_X * s[:, None], D / s[:, None]), C) < 1e-13
    perm = RNG.permutation(13)
    assert rel(oracle.forward(X, What[perm], E_X[perm], D[perm]), C) < 1e-13


def test_output_statistics_at_workload_distributions():
    """With X~N(0,1), What~N(0,1/k), bases~N(0,1/16): Var Xhat=1, Var Yhat=1/4, Var C=r/64."""
    import stl_synth
    p = stl_synth.stl_problem(256, 256, 256, 32, seed=5, dtype="f32")
    C, Y = planes.forward(p["X"], p["What"], p["E_X"], p["D"], return_yhat=True)
    Xh = planes.encode(p["X"], p["E_X"])
    rowvar = (p["E_X"].astype(np.float64) ** 2).sum(axis=1)        # exact conditional variances
    assert abs(Xh.var() / rowvar.mean() - 1) < 0.05
    assert abs(Y.var() / (rowvar.mean() * 0.25) - 1) < 0.1
    assert 0.3 < C.var() / (32 / 64) < 3.0


# ------------------------------------------------------------------------- gradients
def loss(X, What, E_X, D, dC):
    return float(np.sum(dC * oracle.forward(X, What, E_X, D)))


def test_gradients_finite_differences_32():
    """m=k=n=32: the loss <dC,C> is linear in each argument, so a central difference along a
    random direction equals <grad, direction> up to fp64 rounding."""
    X, W, E_X, E_W, D = rand_problem(32, 32, 32, 12)
    What = oracle.encode_weight(W, E_W)
    dC = RNG.standard_normal((32, 32))
    grads = oracle.backward(X, What, E_X, D, dC)
    args = [X, What, E_X, D]
    for i, g in enumerate(grads):
        V = RNG.standard_normal(args[i].shape)
        h = 1e-3
        plus = [a.copy() for a in args]
        minus = [a.copy() for a in args]
        plus[i] += h * V
        minus[i] -= h * V
        fd = (loss(*plus, dC) - loss(*minus, dC)) / (2 * h)
        an = float(np.sum(g * V))
        assert abs(fd - an) <= 1e-9 * max(abs(an), 1.0), (i, fd, an)


def test_gradients_entrywise_finite_differences_tiny():
    X, W, E_X, E_W, D = rand_problem(8, 4, 8, 3)
    What = oracle.encode_weight(W, E_W)
    dC = RNG.standard_normal((8, 8))
    grads = oracle.backward(X, What, E_X, D, dC)
    args = [X, What, E_X, D]
    base = loss(*args, dC)
    for i, g in enumerate(grads):
        fd = np.zeros_like(args[i])
        it = np.nditer(args[i], flags=["multi_index"])
        for _ in it:
            pert = [a.copy() for a in args]
            pert[i][it.multi_index] += 1.0          # linear => unit step is exact
            fd[it.multi_index] = loss(*pert, dC) - base
        assert rel(g, fd) < 1e-11, i


def test_euler_identities():
    X, W, E_X, E_W, D = rand_problem(16, 24, 12, 20)
    What = oracle.encode_weight(W, E_W)
    dC = RNG.standard_normal((16, 12))
    dX, dWhat, dE_X, dD = oracle.backward(X, What, E_X, D, dC)
    ref = loss(X, What, E_X, D, dC)
    for g, a in ((dX, X), (dWhat, What), (dE_X, E_X), (dD, D)):
        assert abs(np.sum(g * a) - ref) < 1e-11 * abs(ref) + 1e-11


def test_gradients_at_exact_basis_are_textbook():
    """At the rank-49 basis C = X@W, so dX = dC W^T and <dWhat, enc_W(V)> = <X^T dC, V>."""
    E_X, E_W, D = bases.strassen_4x4()
    X = RNG.standard_normal((12, 16))
    W = RNG.standard_normal((16, 8))
    dC = RNG.standard_normal((12, 8))
    What = oracle.encode_weight(W, E_W)
    dX, dWhat, _, _ = oracle.backward(X, What, E_X, D, dC)
    assert rel(dX, dC @ W.T) < 1e-13
    V = RNG.standard_normal(W.shape)
    lhs = np.sum(dWhat * oracle.encode_weight(V, E_W))
    rhs = np.sum((X.T @ dC) * V)
    assert abs(lhs - rhs) < 1e-11 * abs(rhs)


def test_weight_encoding_gradients():
    """dW and dE_W through What = encode(W, E_W): adjoint identities with random directions, entrywise finite
    differences of the whole loss <dC, X <> W> (exact: the loss is linear in W and in E_W), and the textbook
    dW = X^T dC at the exact basis."""
    m, k, n, r = 8, 12, 16, 11
    X = RNG.standard_normal((m, k))
    W = RNG.standard_normal((k, n))
    E_X, E_W, D = (RNG.standard_normal((r, 16)) * 0.5 for _ in range(3))
    dC = RNG.standard_normal((m, n))
    loss = lambda W_, E_: float(np.sum(dC * oracle.forward(X, oracle.encode_weight(W_, E_), E_X, D)))
    _, dWhat, _, _ = oracle.backward(X, oracle.encode_weight(W, E_W), E_X, D, dC)
    dW, dE_W = planes.encode_weight_backward(W, E_W, dWhat)
    assert dW.shape == W.shape and dE_W.shape == E_W.shape
    V, F = RNG.standard_normal(W.shape), RNG.standard_normal(E_W.shape)
    assert abs(np.sum(dWhat * oracle.encode_weight(V, E_W)) - np.sum(dW * V)) < 1e-11 * abs(np.sum(dW * V))
    assert abs(np.sum(dWhat * oracle.encode_weight(W, F)) - np.sum(dE_W * F)) < 1e-11 * abs(np.sum(dE_W * F))
    base = loss(W, E_W)
    for (a, b) in [(0, 0), (3, 7), (11, 15), (5, 2)]:
        Wp = W.copy()
        Wp[a, b] += 0.5
        assert abs((loss(Wp, E_W) - base) / 0.5 - dW[a, b]) < 1e-10 * max(1.0, abs(dW[a, b]))
    for (p_, q) in [(0, 0), (4, 9), (10, 15)]:
        Ep = E_W.copy()
        Ep[p_, q] += 0.5
        assert abs((loss(W, Ep) - base) / 0.5 - dE_W[p_, q]) < 1e-10 * max(1.0, abs(dE_W[p_, q]))
    # exact basis: the operator is X @ W, so dW must be X^T dC
    E_X, E_W, D = bases.strassen_4x4()
    _, dWhat, _, _ = oracle.backward(X, oracle.encode_weight(W, E_W), E_X, D, dC)
    dW, _ = planes.encode_weight_backward(W, E_W, dWhat)
    assert rel(dW, X.T @ dC) < 1e-12


# --------------------------------------------------------------- inter-layer identity
def test_algorithm2_fused_decode_encode_identity():
    """Algorithm 2: encoding a decoded output equals one r x r map per tile, Yhat (D E_X^T)."""
    r = 10
    Y = RNG.standard_normal((r, 5, 6))
    D = RNG.standard_normal((r, 16))
    E = RNG.standard_normal((r, 16))
    enc_of_dec = planes.encode(planes.decode(Y, D), E)
    direct = np.einsum("pIJ,ps->sIJ", Y, D @ E.T)
    assert rel(enc_of_dec, direct) < 1e-13


def test_recode_is_decode_activation_encode():
    """The inter-layer step against its parts: linear case = one (r2 x r1) map per tile (Algorithm 2);
    GELU case = entrywise GELU of the decoded tiles, checked entry by entry with math.erf."""
    import math
    r1, r2 = 7, 5
    Y = RNG.standard_normal((r1, 3, 4))
    D = RNG.standard_normal((r1, 16))
    E = RNG.standard_normal((r2, 16))
    lin = planes.recode(Y, D, E, activation=None)
    assert rel(lin, np.einsum("pIJ,sp->sIJ", Y, E @ D.T)) < 1e-13
    got = planes.recode(Y, D, E, activation="gelu")
    want = np.zeros((r2, 3, 4))
    for I in range(3):
        for J in range(4):
            h = [sum(D[p, q] * Y[p, I, J] for p in range(r1)) for q in range(16)]
            g = [0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in h]
            for s_ in range(r2):
                want[s_, I, J] = sum(E[s_, q] * g[q] for q in range(16))
    assert rel(got, want) < 1e-13
    with pytest.raises(ValueError):
        planes.recode(Y, D, E, activation="relu")


@pytest.mark.parametrize("basis", ["strassen", "trivial"])
def test_mlp_pair_at_exact_bases_is_textbook_mlp(basis):
    """With exact bases in both layers the pair equals act(X W1) W2 computed with plain matrix products."""
    E_X, E_W, D = bases.strassen_4x4() if basis == "strassen" else bases.trivial(4)
    m, d, h = 8, 12, 16
    X = RNG.standard_normal((m, d))
    W1 = RNG.standard_normal((d, h)) / np.sqrt(d)
    W2 = RNG.standard_normal((h, d)) / np.sqrt(h)
    Wh1, Wh2 = oracle.encode_weight(W1, E_W), oracle.encode_weight(W2, E_W)
    lin = planes.mlp_pair(X, Wh1, E_X, D, Wh2, E_X, D, activation=None)
    assert rel(lin, X @ W1 @ W2) < 1e-12
    act = planes.mlp_pair(X, Wh1, E_X, D, Wh2, E_X, D)
    assert rel(act, planes.gelu(X @ W1) @ W2) < 1e-12
    # and the pair is the composition of two single-layer forwards of the tile-by-tile oracle
    two = oracle.forward(planes.gelu(oracle.forward(X, Wh1, E_X, D)), Wh2, E_X, D)
    assert rel(act, two) < 1e-12


# --------------------------------------------------------------- both operands encoded at run time
def test_aa_forward_brute_force_and_exact_basis():
    """Two activations: (a) tile by tile from the operator's definition with the second operand encoded by E_B,
    written with Python loops; (b) at the exact rank-49 basis every stacked product is A_b @ B_b."""
    nb, m, k, n, r = 3, 8, 12, 4, 9
    A = RNG.standard_normal((nb * m, k))
    B = RNG.standard_normal((nb * k, n))
    E_A, E_B, D = (RNG.standard_normal((r, 16)) for _ in range(3))
    got = planes.aa_forward(A, B, E_A, E_B, D, nbatch=nb)
    want = np.zeros((nb * m, n))
    for b in range(nb):
        for I in range(m // 4):
            for J in range(n // 4):
                acc = np.zeros(r)
                for L in range(k // 4):
                    a = A[b * m + 4 * I:b * m + 4 * I + 4, 4 * L:4 * L + 4].reshape(16)
                    bb = B[b * k + 4 * L:b * k + 4 * L + 4, 4 * J:4 * J + 4].reshape(16)
                    acc += (E_A @ a) * (E_B @ bb)
                want[b * m + 4 * I:b * m + 4 * I + 4, 4 * J:4 * J + 4] = (D.T @ acc).reshape(4, 4)
    assert rel(got, want) < 1e-13
    E_A, E_B, D = bases.strassen_4x4()
    got = planes.aa_forward(A, B, E_A, E_B, D, nbatch=nb)
    for b in range(nb):
        assert rel(got[b * m:(b + 1) * m], A[b * m:(b + 1) * m] @ B[b * k:(b + 1) * k]) < 1e-12
    with pytest.raises(ValueError):
        planes.aa_forward(A, B[:-4], E_A, E_B, D, nbatch=nb)


def test_aa_backward_finite_differences_and_textbook():
    """Gradients of sum_b <dC_b, C_b>: the loss is linear in each of A, B, E_A, E_B, D, so a one-sided difference
    with any step is exact up to rounding; at the exact basis dA_b = dC_b B_b^T and dB_b = A_b^T dC_b."""
    nb, m, k, n, r = 2, 8, 8, 12, 6
    A = RNG.standard_normal((nb * m, k))
    B = RNG.standard_normal((nb * k, n))
    E_A, E_B, D = (RNG.standard_normal((r, 16)) * 0.5 for _ in range(3))
    dC = RNG.standard_normal((nb * m, n))
    args = [A, B, E_A, E_B, D]
    loss = lambda a: float(np.sum(dC * planes.aa_forward(*a, nbatch=nb)))
    grads = planes.aa_backward(A, B, E_A, E_B, D, dC, nbatch=nb)
    base = loss(args)
    for which, g in enumerate(grads):
        assert g.shape == args[which].shape
        for idx in [(0, 0), (args[which].shape[0] - 1, args[which].shape[1] - 1), (3, 5), (5, 2)]:
            pert = [x.copy() for x in args]
            pert[which][idx] += 0.5
            assert abs((loss(pert) - base) / 0.5 - g[idx]) < 1e-9 * max(1.0, abs(g[idx])), (which, idx)
    E_A, E_B, D = bases.strassen_4x4()
    dA, dB, _, _, _ = planes.aa_backward(A, B, E_A, E_B, D, dC, nbatch=nb)
    for b in range(nb):
        Ab, Bb, dCb = A[b * m:(b + 1) * m], B[b * k:(b + 1) * k], dC[b * m:(b + 1) * m]
        assert rel(dA[b * m:(b + 1) * m], dCb @ Bb.T) < 1e-12
        assert rel(dB[b * k:(b + 1) * k], Ab.T @ dCb) < 1e-12


def test_aa_transposed_second_operand():
    """Q K^T with K stored tokens x width: at the exact basis C_b = A_b @ B_b^T, dA_b = dC_b B_b, dB_b = dC_b^T A_b;
    for a generic basis, tile by tile with the transposed tile written out (tile (L, J) of B^T is the transpose of
    tile (J, L) of B), and finite differences on B in its stored shape."""
    nb, m, k, n, r = 2, 8, 12, 4, 7
    A = RNG.standard_normal((nb * m, k))
    B = RNG.standard_normal((nb * n, k))              # stored transposed
    dC = RNG.standard_normal((nb * m, n))
    E_A, E_B, D = bases.strassen_4x4()
    C = planes.aa_forward(A, B, E_A, E_B, D, nbatch=nb, b_transposed=True)
    dA, dB, _, _, _ = planes.aa_backward(A, B, E_A, E_B, D, dC, nbatch=nb, b_transposed=True)
    for b in range(nb):
        Ab, Bb, dCb = A[b * m:(b + 1) * m], B[b * n:(b + 1) * n], dC[b * m:(b + 1) * m]
        assert rel(C[b * m:(b + 1) * m], Ab @ Bb.T) < 1e-12
        assert rel(dA[b * m:(b + 1) * m], dCb @ Bb) < 1e-12
        assert rel(dB[b * n:(b + 1) * n], dCb.T @ Ab) < 1e-12
    E_A, E_B, D = (RNG.standard_normal((r, 16)) * 0.5 for _ in range(3))
    got = planes.aa_forward(A, B, E_A, E_B, D, nbatch=nb, b_transposed=True)
    want = np.zeros((nb * m, n))
    for b in range(nb):
        for I in range(m // 4):
            for J in range(n // 4):
                acc = np.zeros(r)
                for L in range(k // 4):
                    a = A[b * m + 4 * I:b * m + 4 * I + 4, 4 * L:4 * L + 4].reshape(16)
                    bt = B[b * n + 4 * J:b * n + 4 * J + 4, 4 * L:4 * L + 4].T.reshape(16)
                    acc += (E_A @ a) * (E_B @ bt)
                want[b * m + 4 * I:b * m + 4 * I + 4, 4 * J:4 * J + 4] = (D.T @ acc).reshape(4, 4)
    assert rel(got, want) < 1e-13
    loss = lambda B_: float(np.sum(dC * planes.aa_forward(A, B_, E_A, E_B, D, nbatch=nb, b_transposed=True)))
    g = planes.aa_backward(A, B, E_A, E_B, D, dC, nbatch=nb, b_transposed=True)
    assert g[1].shape == B.shape
    base = loss(B)
    for idx in [(0, 0), (3, 11), (7, 5)]:
        Bp = B.copy()
        Bp[idx] += 0.5
        assert abs((loss(Bp) - base) / 0.5 - g[1][idx]) < 1e-9 * max(1.0, abs(g[1][idx]))
    lossE = lambda E_: float(np.sum(dC * planes.aa_forward(A, B, E_A, E_, D, nbatch=nb, b_transposed=True)))
    for idx in [(0, 1), (6, 14)]:
        Ep = E_B.copy()
        Ep[idx] += 0.5
        assert abs((lossE(Ep) - base) / 0.5 - g[3][idx]) < 1e-9 * max(1.0, abs(g[3][idx]))


# --------------------------------------------------------------- row counts that t does not divide
def test_pad_and_fold_rows():
    """197-token images (Class-1 appendix): 3 null rows are appended per image; on the way back complete tile rows
    are copied and the last 4 rows become one row with 4 coefficients.  Written out with loops."""
    rows, nimg, k = 9, 3, 4            # 9 = 2*4 + 1, the paper's 197 = 49*4 + 1 in small
    X = RNG.standard_normal((nimg * rows, k))
    Xp = planes.pad_rows(X, rows)
    assert Xp.shape == (nimg * 12, k)
    for i in range(nimg):
        assert np.array_equal(Xp[12 * i:12 * i + 9], X[9 * i:9 * i + 9])
        assert np.all(Xp[12 * i + 9:12 * i + 12] == 0.0)
    Y = RNG.standard_normal((nimg * 12, 5))
    c = RNG.standard_normal((1, 4))
    F = planes.fold_rows(Y, c, rows)
    assert F.shape == (nimg * 9, 5)
    for i in range(nimg):
        assert np.array_equal(F[9 * i:9 * i + 8], Y[12 * i:12 * i + 8])
        want = sum(c[0, a] * Y[12 * i + 8 + a] for a in range(4))
        assert np.allclose(F[9 * i + 8], want, rtol=0, atol=1e-14)
    # rho = 3: one combination per remaining row; rows divisible by t: nothing happens
    c3 = RNG.standard_normal((3, 4))
    F3 = planes.fold_rows(Y, c3, 11)
    assert np.allclose(F3[11 * 1 + 8:11 * 1 + 11], c3 @ Y[12 + 8:12 + 12], rtol=0, atol=1e-14)
    assert np.array_equal(planes.fold_rows(Y, None, 12), Y)
    with pytest.raises(ValueError):
        planes.fold_rows(Y, np.zeros((2, 4)), rows)
    with pytest.raises(ValueError):
        planes.pad_rows(X[:-1], rows)


def test_ragged_forward_closed_forms():
    """At the exact basis the padded operator is X_pad @ W, whose null rows are zero: the folded last row is
    fold[0] * (x_last @ W) and all other rows are X @ W.  With a generic basis the null rows of the last tile row
    do produce output (tiles mix rows), and the fold must use all four: checked against the tile-by-tile oracle."""
    rows, nimg, k, n = 5, 2, 8, 12
    X = RNG.standard_normal((nimg * rows, k))
    W = RNG.standard_normal((k, n))
    c = RNG.standard_normal((1, 4))
    E_X, E_W, D = bases.strassen_4x4()
    got = planes.ragged_forward(X, oracle.encode_weight(W, E_W), E_X, D, c, rows)
    want = X @ W
    for i in range(nimg):
        want[rows * i + 4] *= c[0, 0]
    assert rel(got, want) < 1e-12
    r = 7
    E_X, E_W, D = (RNG.standard_normal((r, 16)) for _ in range(3))
    What = oracle.encode_weight(W, E_W)
    got = planes.ragged_forward(X, What, E_X, D, c, rows)
    Xp = np.zeros((nimg * 8, k))
    for i in range(nimg):
        Xp[8 * i:8 * i + 5] = X[5 * i:5 * i + 5]
    Yp = oracle.forward(Xp, What, E_X, D)
    assert np.abs(Yp[5:8]).max() > 1e-3                      # null rows are not silent under a generic basis
    for i in range(nimg):
        assert rel(got[5 * i:5 * i + 4], Yp[8 * i:8 * i + 4]) < 1e-13
        assert rel(got[5 * i + 4], c[0] @ Yp[8 * i + 4:8 * i + 8]) < 1e-13


def test_ragged_backward_finite_differences():
    """The loss <dC, ragged_forward> is linear in X, What, E_X, D and fold: one-sided differences are exact."""
    rows, nimg, k, n, r = 6, 2, 8, 4, 5          # rho = 2
    X = RNG.standard_normal((nimg * rows, k))
    What = RNG.standard_normal((r, k // 4, n // 4))
    E_X, D = (RNG.standard_normal((r, 16)) * 0.5 for _ in range(2))
    fold = RNG.standard_normal((2, 4))
    dC = RNG.standard_normal((nimg * rows, n))
    args = [X, What, E_X, D, fold]
    loss = lambda a: float(np.sum(dC * planes.ragged_forward(*a, rows)))
    grads = planes.ragged_backward(X, What, E_X, D, fold, dC, rows)
    base = loss(args)
    for which, g in enumerate(grads):
        assert g.shape == args[which].shape
        flat = g.reshape(-1)
        for j in sorted({0, flat.size - 1, flat.size // 2, flat.size // 3}):
            idx = np.unravel_index(j, g.shape)
            pert = [x.copy() for x in args]
            pert[which][idx] += 0.5
            assert abs((loss(pert) - base) / 0.5 - g[idx]) < 1e-9 * max(1.0, abs(g[idx])), (which, idx)
    # rows divisible by t: identical to the plain operator, no fold gradient
    g4 = planes.ragged_backward(X[:8], What, E_X, D, None, dC[:8], 4)
    ref = planes.backward(X[:8], What, E_X, D, dC[:8])
    assert g4[4] is None and all(rel(a, b) < 1e-14 for a, b in zip(g4[:4], ref))


def test_gelu_values():
    """Exact-erf GELU against closed-form values: gelu(0)=0, gelu(x)-gelu(-x)=x, gelu(1)=Phi(1)."""
    assert planes.gelu(0.0) == 0.0
    x = np.linspace(-4, 4, 33)
    assert np.allclose(planes.gelu(x) - planes.gelu(-x), x, atol=1e-15)
    assert abs(planes.gelu(1.0) - 0.8413447460685429) < 1e-15


def test_argument_checks():
    with pytest.raises(ValueError):
        oracle.forward(np.zeros((6, 8)), np.zeros((3, 2, 2)), np.zeros((3, 16)), np.zeros((3, 16)))
    with pytest.raises(ValueError):
        oracle.forward(np.zeros((8, 8)), np.zeros((3, 3, 2)), np.zeros((3, 16)), np.zeros((3, 16)))
