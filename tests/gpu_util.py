"""Helpers for the GPU parity tests: upload seeded inputs, call the C ABI, download results."""
import numpy as np
import torch

import paper_2503_12211_amd as stl

TOL = {"f32": 1e-5, "bf16": 1e-2}          # relative Frobenius error bars (fp32 / bf16 with fp32 accumulation)
TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}
STL_DT = {"f32": stl.STL_F32, "bf16": stl.STL_BF16}


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


# Per-entry bar, as a multiple of rms(O).  With bf16 storage an output passes through three roundings to bf16 (encoded
# operand, encoded product, output); one rounding of a value with a log-uniform significand has relative rms
# eps = 2^-8 / sqrt(3) * 0.736 = 1.66e-3, the first two reach the output through the decode sum, whose terms are
# independent, so each contributes eps * rms(O) and the three together sqrt(3) * eps = 2.9e-3 (the measured relative
# Frobenius error).  An entry's error is a sum of many independent terms, so it is close to normal; among 1e8 entries
# the largest |z| stays below 6.5, and an entry whose planes happen to be large has up to 2.5 times the average
# deviation: c = 6.5 * 2.5 * 2.9e-3 = 0.047 -> 0.05.  One wrong entry (error ~ rms(O)) is twenty times over it.
# fp32 storage: the same with 2^-24 in place of 2^-8 and fp32 accumulation over the contraction, 5e-5.
ENTRY_C = {"f32": 5e-5, "bf16": 5e-2}


def _block_sums(a2, bh, bw):
    """Sums of a 2-D array over bh x bw blocks (ragged last blocks included)."""
    r_idx = np.arange(0, a2.shape[0], bh)
    c_idx = np.arange(0, a2.shape[1], bw)
    return np.add.reduceat(np.add.reduceat(a2, r_idx, axis=0), c_idx, axis=1)


def check(G, O, dtype, name, block=256, slab=4, entry_ref=None):
    """Full comparison of a GPU result with the oracle's: (1) relative Frobenius error of the whole tensor within
    TOL[dtype]; (2) every entry within ENTRY_C[dtype] * rms(O); (3) the relative Frobenius error of every
    block x block sub-matrix and of every slab of `slab` rows (a tile row for matrices) within TOL[dtype] as well, so
    that a wrong tile row, block edge or plane cannot hide in the headroom of one norm.  Tensors with three
    dimensions are taken plane by plane.  entry_ref: the tensor whose rms scales the per-entry bar when it is not O
    itself (the pre-activation values for an output that went through GELU, whose own rms is smaller than the scale of
    the rounding errors that reach it).  Returns the measured figures."""
    G = np.asarray(G, dtype=np.float64)
    O = np.asarray(O, dtype=np.float64)
    assert G.shape == O.shape, (name, G.shape, O.shape)
    assert np.isfinite(G).all(), f"{name}: non-finite entries"
    diff = G - O
    e2, o2 = diff * diff, O * O
    tol = TOL[dtype]
    whole = float(np.sqrt(e2.sum() / max(o2.sum(), 1e-300)))
    rms = float(np.sqrt(o2.mean())) if entry_ref is None else float(np.sqrt(np.mean(np.square(np.asarray(entry_ref, dtype=np.float64)))))
    worst = float(np.abs(diff).max() / max(rms, 1e-300))
    out = {"rel": whole, "max_entry_over_rms": worst}
    assert whole <= tol, f"{name}: relative Frobenius error {whole:.3e} > {tol}"
    assert worst <= ENTRY_C[dtype], f"{name}: an entry is off by {worst:.3e} x rms(O) > {ENTRY_C[dtype]}"
    if G.ndim >= 2 and G.shape[-1] >= 64 and G.shape[-2] >= 64:
        e3 = e2.reshape(-1, G.shape[-2], G.shape[-1])
        o3 = o2.reshape(-1, G.shape[-2], G.shape[-1])
        wb, ws = 0.0, 0.0
        for pl in range(e3.shape[0]):
            be, bo = _block_sums(e3[pl], block, block), _block_sums(o3[pl], block, block)
            wb = max(wb, float(np.sqrt((be / np.maximum(bo, 1e-300)).max())))
            se = np.add.reduceat(e3[pl].sum(axis=1), np.arange(0, e3.shape[1], slab))
            so = np.add.reduceat(o3[pl].sum(axis=1), np.arange(0, o3.shape[1], slab))
            ws = max(ws, float(np.sqrt((se / np.maximum(so, 1e-300)).max())))
        out["worst_block_rel"], out["worst_slab_rel"] = wb, ws
        assert wb <= tol, f"{name}: a {block}x{block} block has relative error {wb:.3e} > {tol}"
        assert ws <= tol, f"{name}: a slab of {slab} rows has relative error {ws:.3e} > {tol}"
    print(f"    parity {name}: " + "  ".join(f"{k_}={v:.3e}" for k_, v in out.items()), flush=True)
    return out


def dev(a, dtype):
    """float32 numpy values (already representable in dtype) -> device tensor of that dtype."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda").to(TORCH_DT[dtype]).contiguous()


def host(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


PG = stl.STL_PLANE_GROUP


def group_planes(a):
    """Plane-major (r, R, Cc) numpy -> the library's activation-side layout (groups of PG tile rows), flat."""
    a = np.asarray(a)
    r, R, Cc = a.shape
    Rp = (R + PG - 1) // PG * PG
    pad = np.zeros((r, Rp, Cc), dtype=a.dtype)
    pad[:, :R] = a
    return np.ascontiguousarray(pad.reshape(r, Rp // PG, PG, Cc).transpose(1, 0, 2, 3)).reshape(-1)


def ungroup_planes(flat, r, R, Cc):
    """Inverse of group_planes: flat grouped array -> plane-major (r, R, Cc)."""
    Rp = (R + PG - 1) // PG * PG
    a = np.asarray(flat).reshape(Rp // PG, r, PG, Cc).transpose(1, 0, 2, 3).reshape(r, Rp, Cc)
    return np.ascontiguousarray(a[:, :R])


def planes_buffer(r, R, Cc, dtype, fill=float("nan")):
    return torch.full((stl.stl_plane_elems(R, Cc, r),), fill, dtype=TORCH_DT[dtype], device="cuda")


def planes_to_dev(a, dtype):
    """plane-major numpy (r, R, Cc) -> device tensor in the grouped layout"""
    return dev(group_planes(np.asarray(a, dtype=np.float32)), dtype)


def planes_to_host(t, r, R, Cc):
    return ungroup_planes(host(t), r, R, Cc)


class Guard:
    """Device buffers with 4 KB of sentinel bytes on either side: check() fails if a kernel wrote outside a buffer it
    was given (reads outside cannot be seen this way)."""
    PAD, BYTE = 4096, 0xA5

    def __init__(self):
        self.bufs = []

    def alloc(self, shape, dtype, fill=float("nan")):
        n = int(np.prod(shape))
        es = torch.empty((), dtype=dtype).element_size()
        raw = torch.full((n * es + 2 * self.PAD,), self.BYTE, dtype=torch.uint8, device="cuda")
        body = raw[self.PAD:self.PAD + n * es].view(dtype).view(*shape)
        if fill is not None:
            body.fill_(fill)
        self.bufs.append(raw)
        return body

    def check(self):
        torch.cuda.synchronize()
        for i, raw in enumerate(self.bufs):
            lo, hi = raw[:self.PAD], raw[-self.PAD:]
            assert bool((lo == self.BYTE).all()) and bool((hi == self.BYTE).all()), f"buffer {i}: write outside its bounds"


def workspace(prob, op, flags=0):
    nbytes = stl.stl_workspace_bytes(prob, op, flags)
    return torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda"), nbytes


def forward(p, dtype, flags=0, save_yhat=False, save_xhat=False):
    """p: dict with X, What, E_X, D (numpy).  Returns C (and Yhat) as float64 numpy."""
    m, k = p["X"].shape
    r, K, N = p["What"].shape
    n = 4 * N
    prob = stl.Problem(m, k, n, r, STL_DT[dtype])
    X, What, E_X, D = (dev(p[s], dtype) for s in ("X", "What", "E_X", "D"))
    gd = Guard()
    C = gd.alloc((m, n), TORCH_DT[dtype])
    Y = gd.alloc((stl.stl_plane_elems(m // 4, N, r),), TORCH_DT[dtype]) if save_yhat else None
    Xh = gd.alloc((stl.stl_plane_elems(m // 4, k // 4, r),), TORCH_DT[dtype]) if save_xhat else None
    nbytes = stl.stl_workspace_bytes(prob, stl.STL_OP_FORWARD, flags)
    ws = gd.alloc((max(nbytes, 16),), torch.uint8, fill=None)
    stl.stl_forward(prob, X, What, E_X, D, C, Xh, Y, ws, nbytes, flags)
    gd.check()
    if save_xhat:
        return host(C), planes_to_host(Xh, r, m // 4, k // 4), planes_to_host(Y, r, m // 4, N)
    return (host(C), planes_to_host(Y, r, m // 4, N)) if save_yhat else host(C)


def backward(p, dtype, yhat=None, accumulate=0, init=None, skip=(), xhat=None):
    m, k = p["X"].shape
    r, K, N = p["What"].shape
    n = 4 * N
    prob = stl.Problem(m, k, n, r, STL_DT[dtype])
    X, What, E_X, D, dC = (dev(p[s], dtype) for s in ("X", "What", "E_X", "D", "dC"))
    Y = planes_to_dev(yhat, dtype) if yhat is not None else None
    Xh = planes_to_dev(xhat, dtype) if xhat is not None else None
    gd = Guard()
    outs = {"dX": gd.alloc((m, k), TORCH_DT[dtype]), "dWhat": gd.alloc((r, K, N), torch.float32),
            "dE_X": gd.alloc((r, 16), torch.float32), "dD": gd.alloc((r, 16), torch.float32)}
    if init is not None:
        for name, a in zip(("dWhat", "dE_X", "dD"), init):
            outs[name].copy_(torch.from_numpy(np.asarray(a, dtype=np.float32)))
    args = {k_: (None if k_ in skip else v) for k_, v in outs.items()}
    nbytes = stl.stl_workspace_bytes(prob, stl.STL_OP_BACKWARD)
    ws = gd.alloc((max(nbytes, 16),), torch.uint8, fill=None)
    stl.stl_backward(prob, X, What, E_X, D, dC, Xh, Y, args["dX"], args["dWhat"], args["dE_X"], args["dD"],
                     accumulate, ws, nbytes)
    gd.check()
    return {k_: host(v) for k_, v in outs.items()}


def step(p, dtype, flags=0):
    """One training step exactly as bench.py runs it: stl_forward writing Xhat_save and Yhat_save, then stl_backward
    reading those same device buffers.  Returns C, Xhat, Yhat (plane-major) and the four gradients as float64 numpy."""
    m, k = p["X"].shape
    r, K, N = p["What"].shape
    n, M = 4 * N, m // 4
    prob = stl.Problem(m, k, n, r, STL_DT[dtype])
    X, What, E_X, D, dC = (dev(p[s], dtype) for s in ("X", "What", "E_X", "D", "dC"))
    gd = Guard()
    C = gd.alloc((m, n), TORCH_DT[dtype])
    Xh = gd.alloc((stl.stl_plane_elems(M, K, r),), TORCH_DT[dtype])
    Y = gd.alloc((stl.stl_plane_elems(M, N, r),), TORCH_DT[dtype])
    outs = {"dX": gd.alloc((m, k), TORCH_DT[dtype]), "dWhat": gd.alloc((r, K, N), torch.float32),
            "dE_X": gd.alloc((r, 16), torch.float32), "dD": gd.alloc((r, 16), torch.float32)}
    nf = stl.stl_workspace_bytes(prob, stl.STL_OP_FORWARD, flags)
    nb = stl.stl_workspace_bytes(prob, stl.STL_OP_BACKWARD)
    ws_f = gd.alloc((max(nf, 16),), torch.uint8, fill=None)
    ws_b = gd.alloc((max(nb, 16),), torch.uint8, fill=None)
    stl.stl_forward(prob, X, What, E_X, D, C, Xh, Y, ws_f, nf, flags)
    stl.stl_backward(prob, X, What, E_X, D, dC, Xh, Y, outs["dX"], outs["dWhat"], outs["dE_X"], outs["dD"], 0, ws_b, nb)
    gd.check()
    res = {k_: host(v) for k_, v in outs.items()}
    res.update(C=host(C), Xhat=planes_to_host(Xh, r, M, K), Yhat=planes_to_host(Y, r, M, N))
    return res


def mlp_forward(p1, p2, dtype, flags=0):
    """p1, p2: dicts with What, E_X, D of the two layers (p1 also X).  Returns C of the pair as float64 numpy."""
    m, k1 = p1["X"].shape
    r1, _, N1 = p1["What"].shape
    r2, K2, N2 = p2["What"].shape
    assert K2 == N1
    up = stl.Problem(m, k1, 4 * N1, r1, STL_DT[dtype])
    down = stl.Problem(m, 4 * K2, 4 * N2, r2, STL_DT[dtype])
    X, W1, E1, D1 = (dev(p1[s], dtype) for s in ("X", "What", "E_X", "D"))
    W2, E2, D2 = (dev(p2[s], dtype) for s in ("What", "E_X", "D"))
    C = torch.full((m, 4 * N2), float("nan"), dtype=TORCH_DT[dtype], device="cuda")
    nbytes = stl.stl_mlp_workspace_bytes(up, down, flags)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    stl.stl_mlp_forward(up, down, X, W1, E1, D1, W2, E2, D2, C, ws, nbytes, flags)
    torch.cuda.synchronize()
    return host(C)


def recode(Yhat1, D1, E2, dtype, flags=0, with_scratch=False):
    """Inter-layer step on its own: Yhat1 (r1, M, N1) -> Xhat2 (r2, M, N1) as float64 numpy."""
    r1, M, N1 = Yhat1.shape
    r2 = E2.shape[0]
    up = stl.Problem(4 * M, 4, 4 * N1, r1, STL_DT[dtype])          # k of the first layer plays no part in this step
    down = stl.Problem(4 * M, 4 * N1, 4, r2, STL_DT[dtype])
    Y, D, E = planes_to_dev(Yhat1, dtype), dev(D1, dtype), dev(E2, dtype)
    Xh2 = planes_buffer(r2, M, N1, dtype)
    H = torch.empty((4 * M, 4 * N1), dtype=TORCH_DT[dtype], device="cuda") if with_scratch else None
    stl.stl_recode(up, down, Y, D, E, Xh2, H, flags)
    torch.cuda.synchronize()
    return planes_to_host(Xh2, r2, M, N1)


def encode_weight_backward(W, E_W, dWhat, dtype, accumulate=0, init=None, skip=()):
    """W (k, n), E_W (r, 16), dWhat (r, K, N) fp32 -> dict(dW, dE_W) as float64 numpy."""
    k, n = W.shape
    r = E_W.shape[0]
    prob = stl.Problem(4, k, n, r, STL_DT[dtype])                 # m plays no part in the weight encoding
    Wd, Ed = dev(W, dtype), dev(E_W, dtype)
    dWh = torch.from_numpy(np.ascontiguousarray(dWhat, dtype=np.float32)).cuda()
    dW = torch.full((k, n), float("nan"), dtype=TORCH_DT[dtype], device="cuda")
    dE = (torch.full((r, 16), float("nan"), dtype=torch.float32, device="cuda") if init is None
          else torch.from_numpy(np.asarray(init, dtype=np.float32)).cuda())
    ws, nbytes = workspace(prob, stl.STL_OP_ENCODE_WEIGHT_BACKWARD)
    stl.stl_encode_weight_backward(prob, Wd, Ed, dWh, None if "dW" in skip else dW, None if "dE_W" in skip else dE,
                                   accumulate, ws, nbytes)
    torch.cuda.synchronize()
    return {"dW": host(dW), "dE_W": host(dE)}


def aa_forward(A, B, E_A, E_B, D, nb, dtype, flags=0, save=False):
    """Stacked two-activation STL through the C ABI.  Returns C (and Ahat, Bhat, Yhat, plane-major) as float64 numpy.
    With STL_FLAG_B_TRANSPOSED in flags B is (nb*n, k) and Bhat comes back as [p][J][L] over nb*N tile rows."""
    bt = bool(flags & stl.STL_FLAG_B_TRANSPOSED)
    m, k, n, r = A.shape[0] // nb, A.shape[1], (B.shape[0] // nb if bt else B.shape[1]), D.shape[0]
    prob = stl.Problem(m, k, n, r, STL_DT[dtype])
    Ad, Bd, Ea, Eb, Dd = (dev(x, dtype) for x in (A, B, E_A, E_B, D))
    gd = Guard()
    C = gd.alloc((nb * m, n), TORCH_DT[dtype])
    shapes = [(nb * m // 4, k // 4), (nb * n // 4, k // 4) if bt else (nb * k // 4, n // 4), (nb * m // 4, n // 4)]
    bufs = [gd.alloc((stl.stl_plane_elems(R, Cc, r),), TORCH_DT[dtype]) for R, Cc in shapes] if save else [None] * 3
    nbytes = stl.stl_aa_workspace_bytes(prob, nb, stl.STL_OP_FORWARD)
    ws = gd.alloc((max(nbytes, 16),), torch.uint8, fill=None)
    stl.stl_aa_forward(prob, nb, Ad, Bd, Ea, Eb, Dd, C, bufs[0], bufs[1], bufs[2], ws, nbytes, flags)
    gd.check()
    if save:
        return (host(C),) + tuple(planes_to_host(b, r, R, Cc) for b, (R, Cc) in zip(bufs, shapes))
    return host(C)


def aa_backward(A, B, E_A, E_B, D, dC, nb, dtype, saved=None, accumulate=0, init=None, skip=(), flags=0):
    """Returns dict(dA, dB, dE_A, dE_B, dD) as float64 numpy.  saved: (Ahat, Bhat, Yhat) plane-major numpy or None."""
    bt = bool(flags & stl.STL_FLAG_B_TRANSPOSED)
    m, k, n, r = A.shape[0] // nb, A.shape[1], (B.shape[0] // nb if bt else B.shape[1]), D.shape[0]
    prob = stl.Problem(m, k, n, r, STL_DT[dtype])
    Ad, Bd, Ea, Eb, Dd, dCd = (dev(x, dtype) for x in (A, B, E_A, E_B, D, dC))
    sv = [planes_to_dev(x, dtype) for x in saved] if saved is not None else [None] * 3
    gd = Guard()
    outs = {"dA": gd.alloc((nb * m, k), TORCH_DT[dtype]), "dB": gd.alloc(tuple(B.shape), TORCH_DT[dtype])}
    for i, name in enumerate(("dE_A", "dE_B", "dD")):
        outs[name] = gd.alloc((r, 16), torch.float32)
        if init is not None:
            outs[name].copy_(torch.from_numpy(np.asarray(init[i], dtype=np.float32)))
    a = {k_: (None if k_ in skip else v) for k_, v in outs.items()}
    nbytes = stl.stl_aa_workspace_bytes(prob, nb, stl.STL_OP_BACKWARD)
    ws = gd.alloc((max(nbytes, 16),), torch.uint8, fill=None)
    stl.stl_aa_backward(prob, nb, Ad, Bd, Ea, Eb, Dd, dCd, sv[0], sv[1], sv[2], a["dA"], a["dB"], a["dE_A"], a["dE_B"],
                        a["dD"], accumulate, ws, nbytes, flags)
    gd.check()
    return {k_: host(v) for k_, v in outs.items()}


def _f32dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def ragged_forward(p, rows, dtype, save=False):
    """p: dict with X (nimg*rows, k), What, E_X, D, fold.  Returns C (and Xhat, Yhat plane-major over the padded tile rows)."""
    m, k = p["X"].shape
    r, K, N = p["What"].shape
    prob = stl.Problem(m, k, 4 * N, r, STL_DT[dtype])
    X, What, E_X, D = (dev(p[s], dtype) for s in ("X", "What", "E_X", "D"))
    fold = _f32dev(p.get("fold"))
    Rp = (m // rows) * ((rows + 3) // 4)
    gd = Guard()
    C = gd.alloc((m, 4 * N), TORCH_DT[dtype])
    Xh = gd.alloc((stl.stl_plane_elems(Rp, K, r),), TORCH_DT[dtype]) if save else None
    Yh = gd.alloc((stl.stl_plane_elems(Rp, N, r),), TORCH_DT[dtype]) if save else None
    nbytes = stl.stl_ragged_workspace_bytes(prob, rows, stl.STL_OP_FORWARD)
    ws = gd.alloc((max(nbytes, 16),), torch.uint8, fill=None)
    stl.stl_ragged_forward(prob, rows, X, What, E_X, D, fold, C, Xh, Yh, ws, nbytes)
    gd.check()
    if save:
        return host(C), planes_to_host(Xh, r, Rp, K), planes_to_host(Yh, r, Rp, N)
    return host(C)


def ragged_backward(p, rows, dtype, saved=None, accumulate=0, init=None, skip=()):
    """Returns dict(dX, dWhat, dE_X, dD, dfold) as float64 numpy.  saved: (Xhat, Yhat) plane-major numpy or None."""
    m, k = p["X"].shape
    r, K, N = p["What"].shape
    nrho = rows % 4
    prob = stl.Problem(m, k, 4 * N, r, STL_DT[dtype])
    X, What, E_X, D, dC = (dev(p[s], dtype) for s in ("X", "What", "E_X", "D", "dC"))
    fold = _f32dev(p.get("fold"))
    sv = [planes_to_dev(x, dtype) for x in saved] if saved is not None else [None, None]
    gd = Guard()
    outs = {"dX": gd.alloc((m, k), TORCH_DT[dtype])}
    shapes = {"dWhat": (r, K, N), "dE_X": (r, 16), "dD": (r, 16), "dfold": (max(nrho, 1), 4)}
    for i, (name, shp) in enumerate(shapes.items()):
        outs[name] = gd.alloc(shp, torch.float32)
        if init is not None:
            outs[name].copy_(_f32dev(init[i]))
    a = {k_: (None if k_ in skip else v) for k_, v in outs.items()}
    nbytes = stl.stl_ragged_workspace_bytes(prob, rows, stl.STL_OP_BACKWARD)
    ws = gd.alloc((max(nbytes, 16),), torch.uint8, fill=None)
    stl.stl_ragged_backward(prob, rows, X, What, E_X, D, fold, dC, sv[0], sv[1], a["dX"], a["dWhat"], a["dE_X"], a["dD"],
                            a["dfold"], accumulate, ws, nbytes)
    gd.check()
    res = {k_: host(v) for k_, v in outs.items()}
    res["dfold"] = res["dfold"][:nrho] if nrho else None
    return res
