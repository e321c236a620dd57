"""GPU parity of the single-launch pipelined forward (encode and decode items running between the plane-product blocks
of one persistent launch): bit-identical to the three-launch path, and the operator's result against the oracle."""
import numpy as np
import pytest

import stl_synth
from oracle import planes

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import gpu_util
    return gpu_util


SHAPES = [  # (m, k, n, r, gelu)
    (2048, 256, 1024, 32, False),     # two row blocks, one contraction chunk, one column block
    (2336, 256, 1024, 17, False),     # ragged last row block (M = 584 = 2 * 256 + 72), plane slots beyond r
    (2340, 256, 1024, 17, False),     # M = 585: the three-launch path multiplies in fp32 here (its bf16 kernels want M % 8 == 0)
    (4096, 512, 1280, 8, True),       # N = 320: the second column block hangs over the edge; GELU in the decode items
    (3072, 1024, 2048, 24, False),
    (8192, 1024, 1024, 5, True),      # many row blocks, few planes
]


@pytest.mark.parametrize("shape", SHAPES)
def test_pipelined_forward_equals_three_launches(gu, shape):
    import paper_2503_12211_amd as stl
    m, k, n, r, gelu = shape
    fl = stl.STL_FLAG_GELU if gelu else 0
    p = stl_synth.stl_problem(m, k, n, r, seed=7100 + m + r, dtype="bf16")
    print(f"pipelined forward m={m} k={k} n={n} r={r} gelu={gelu}", flush=True)
    C_a, Xh_a, Y_a = gu.forward(p, "bf16", flags=stl.STL_FLAG_PIPELINED | fl, save_yhat=True, save_xhat=True)
    C_u, Xh_u, Y_u = gu.forward(p, "bf16", flags=stl.STL_FLAG_UNFUSED | fl, save_yhat=True, save_xhat=True)
    assert np.array_equal(Xh_a, Xh_u)
    if (m // 4) % 8 == 0:             # both paths run the same bf16 block code: bit-identical
        assert np.array_equal(Y_a, Y_u)
        assert np.array_equal(C_a, C_u)
    else:                             # fp32 products on the other side: equal up to the rounding of Yhat
        assert gu.rel(Y_a, Y_u) <= 1e-3 and gu.rel(C_a, C_u) <= 1e-3
    C_n = gu.forward(p, "bf16", flags=stl.STL_FLAG_PIPELINED | fl)         # planes in the workspace
    assert np.array_equal(C_n, C_a)
    Cref, Yref = planes.forward(p["X"], p["What"], p["E_X"], p["D"], return_yhat=True)
    gu.check(C_a, planes.gelu(Cref) if gelu else Cref, "bf16", f"pipelined C {shape}", entry_ref=Cref)
    gu.check(Y_a, Yref, "bf16", f"pipelined Yhat {shape}", slab=1)


def test_pipelined_forward_repeats_bit_for_bit(gu):
    """The counters live in the workspace and are cleared by every call: ten calls in a row on the same buffers."""
    import torch
    import paper_2503_12211_amd as stl
    m, k, n, r = 4096, 1024, 1024, 32
    p = stl_synth.stl_problem(m, k, n, r, seed=7200, dtype="bf16")
    prob = stl.Problem(m, k, n, r, stl.STL_BF16)
    X, What, E_X, D = (gu.dev(p[s], "bf16") for s in ("X", "What", "E_X", "D"))
    nbytes = stl.stl_workspace_bytes(prob, stl.STL_OP_FORWARD, stl.STL_FLAG_PIPELINED)
    assert nbytes > stl.stl_workspace_bytes(prob, stl.STL_OP_FORWARD, stl.STL_FLAG_UNFUSED)      # the item counters
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    outs = []
    for i in range(10):
        C = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device="cuda")
        stl.stl_forward(prob, X, What, E_X, D, C, None, None, ws, nbytes, stl.STL_FLAG_PIPELINED)
        outs.append(C)
    torch.cuda.synchronize()
    for C in outs[1:]:
        assert torch.equal(C.view(torch.int16), outs[0].view(torch.int16))
    assert gu.rel(gu.host(outs[0]), planes.forward(p["X"], p["What"], p["E_X"], p["D"])) <= gu.TOL["bf16"]
