"""The library under HIP graph capture: every call only enqueues kernels on the given stream (no allocation, no
synchronisation, no memset nodes), so a forward + backward step can be captured once and replayed."""
import numpy as np
import pytest

import stl_synth

pytestmark = pytest.mark.gpu


def test_step_captured_in_a_graph_replays_identically():
    import torch
    import gpu_util as gu
    import paper_2503_12211_amd as stl
    m, k, n, r = 1024, 512, 768, 32
    p = stl_synth.stl_problem(m, k, n, r, seed=31, dtype="bf16", with_dC=True)
    prob = stl.Problem(m, k, n, r, stl.STL_BF16)
    X, What, E_X, D, dC = (gu.dev(p[s], "bf16") for s in ("X", "What", "E_X", "D", "dC"))
    bf = torch.bfloat16
    C = torch.empty((m, n), dtype=bf, device="cuda")
    Xh = torch.empty(stl.stl_plane_elems(m // 4, k // 4, r), dtype=bf, device="cuda")
    Yh = torch.empty(stl.stl_plane_elems(m // 4, n // 4, r), dtype=bf, device="cuda")
    dX = torch.empty((m, k), dtype=bf, device="cuda")
    dW = torch.empty((r, k // 4, n // 4), dtype=torch.float32, device="cuda")
    dE = torch.empty((r, 16), dtype=torch.float32, device="cuda")
    dD = torch.empty((r, 16), dtype=torch.float32, device="cuda")
    nf, nb = stl.stl_workspace_bytes(prob, stl.STL_OP_FORWARD), stl.stl_workspace_bytes(prob, stl.STL_OP_BACKWARD)
    wf = torch.empty(nf, dtype=torch.uint8, device="cuda")
    wb = torch.empty(nb, dtype=torch.uint8, device="cuda")
    outs = (C, dX, dW, dE, dD)

    def step(stream=None):
        stl.stl_forward(prob, X, What, E_X, D, C, Xh, Yh, wf, nf, 0, stream=stream)
        stl.stl_backward(prob, X, What, E_X, D, dC, Xh, Yh, dX, dW, dE, dD, 0, wb, nb, stream=stream)

    step()                                              # eager: the reference, and every kernel has been loaded once
    torch.cuda.synchronize()
    want = [o.clone() for o in outs]
    side = torch.cuda.Stream()                          # default priority
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                                          # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step(stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for replay in range(4):
        for o in outs:
            o.fill_(float("nan"))                       # eager work between the replays
        wf.random_(0, 255)
        wb.random_(0, 255)                              # the scratch keeps no state between calls
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, w in zip(outs, want):
            assert torch.equal(o, w), replay
    # and a new input through the same graph
    X.copy_(gu.dev(stl_synth.stl_problem(m, k, n, r, seed=32, dtype="bf16")["X"], "bf16"))
    graph.replay()
    torch.cuda.synchronize()
    got = [o.clone() for o in outs]
    step()
    torch.cuda.synchronize()
    for o, g in zip(outs, got):
        assert torch.equal(o, g)
