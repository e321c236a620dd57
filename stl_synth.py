"""Seeded synthetic inputs for the STL hot path.

This module only draws random numbers and rounds them to the storage dtype; it
contains none of the operator's arithmetic.  Both the GPU tests/benchmark and the
CPU oracle take their inputs from here, so that both sides see the same bits.

Distributions are those of the workload list: activations X ~ N(0,1), encoded
weight planes What ~ N(0, 1/k), encoder/decoder entries ~ N(0, 1/16), upstream
gradient dC ~ N(0,1); the second argument of N(.,.) is a variance.  Draw order
is fixed: X, W-or-What, E_X, D, dC, from one ``numpy.random.default_rng(seed)``.
Values are returned as float32 arrays that are exactly representable in the
requested storage dtype ("f32" or "bf16", round-to-nearest-even).
"""
from __future__ import annotations

import numpy as np

# name -> (m, k, n, r, dtype); the workload list of this build
CONFIGS = {
    "C1": dict(m=256, k=256, n=256, r=49, dtype="f32"),
    "C2": dict(m=4096, k=4096, n=4096, r=32, dtype="bf16"),
    "C3": dict(m=8192, k=4096, n=4096, r=32, dtype="bf16"),       # r swept over {8,16,24,32,49,64}
    "C4_up": dict(m=16384, k=1024, n=4096, r=24, dtype="bf16"),
    "C4_down": dict(m=16384, k=4096, n=1024, r=24, dtype="bf16"),
    "C5": dict(m=8192, k=4096, n=4096, r=32, dtype="bf16"),
}
SEEDS = {"C1": 1001, "C2": 1002, "C3": 1003, "C4_up": 1004, "C4_down": 1014, "C5": 1005}


def bf16_bits(a):
    """float32 array -> uint16 bfloat16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits):
    """uint16 bfloat16 bit patterns -> float32 values."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to(a, dtype: str):
    """Round a float array to the storage dtype and return it as float32."""
    a = np.asarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    if dtype == "bf16":
        return bf16_to_f32(bf16_bits(a)).reshape(a.shape)
    raise ValueError(f"unknown dtype {dtype!r}")


def _normal(rng, shape, sigma, dtype):
    return round_to(rng.standard_normal(shape, dtype=np.float32) * np.float32(sigma), dtype)


def dense_problem(m, k, n, seed, dtype="f32"):
    """X (m x k) and a true weight matrix W (k x n), both N(0,1): for the exact-basis case."""
    rng = np.random.default_rng(seed)
    X = _normal(rng, (m, k), 1.0, dtype)
    W = _normal(rng, (k, n), 1.0, dtype)
    return {"X": X, "W": W}


def stl_problem(m, k, n, r, seed, dtype="bf16", t=4, with_dC=False):
    """Gaussian STL problem with pre-encoded ("fake encoding") weight planes."""
    if m % t or k % t or n % t:
        raise ValueError("m, k, n must be divisible by t")
    rng = np.random.default_rng(seed)
    out = {
        "X": _normal(rng, (m, k), 1.0, dtype),
        "What": _normal(rng, (r, k // t, n // t), k ** -0.5, dtype),
        "E_X": _normal(rng, (r, t * t), 0.25, dtype),
        "D": _normal(rng, (r, t * t), 0.25, dtype),
    }
    if with_dC:
        out["dC"] = _normal(rng, (m, n), 1.0, dtype)
    return out


def aa_problem(nbatch, m, k, n, r, seed, dtype="bf16", t=4, with_dC=False):
    """Two stacked activation operands (attention-shaped products: nbatch = heads x images): A (nbatch*m, k) ~ N(0,1),
    B (nbatch*k, n) ~ N(0, 1/k), three bases ~ N(0, 1/16).  Draw order: A, B, E_A, E_B, D, dC."""
    if m % t or k % t or n % t:
        raise ValueError("m, k, n must be divisible by t")
    rng = np.random.default_rng(seed)
    out = {
        "A": _normal(rng, (nbatch * m, k), 1.0, dtype),
        "B": _normal(rng, (nbatch * k, n), k ** -0.5, dtype),
        "E_A": _normal(rng, (r, t * t), 0.25, dtype),
        "E_B": _normal(rng, (r, t * t), 0.25, dtype),
        "D": _normal(rng, (r, t * t), 0.25, dtype),
    }
    if with_dC:
        out["dC"] = _normal(rng, (nbatch * m, n), 1.0, dtype)
    return out


def ragged_problem(nimg, rows, k, n, r, seed, dtype="bf16", t=4, with_dC=False):
    """Images of `rows` token rows each (197 in the ViT workload), stacked: X (nimg*rows, k) ~ N(0,1), encoded weight
    planes ~ N(0, 1/k), bases ~ N(0, 1/16), fold coefficients (rows mod t, t) = "keep the real rows" plus N(0, 1/16) noise
    (fp32 whatever the dtype), dC ~ N(0,1).  Draw order: X, What, E_X, D, fold, dC."""
    if k % t or n % t:
        raise ValueError("k, n must be divisible by t")
    rng = np.random.default_rng(seed)
    nrho = rows % t
    out = {
        "X": _normal(rng, (nimg * rows, k), 1.0, dtype),
        "What": _normal(rng, (r, k // t, n // t), k ** -0.5, dtype),
        "E_X": _normal(rng, (r, t * t), 0.25, dtype),
        "D": _normal(rng, (r, t * t), 0.25, dtype),
        "fold": (np.eye(nrho, t, dtype=np.float32) + _normal(rng, (nrho, t), 0.25, "f32")) if nrho else None,
    }
    if with_dC:
        out["dC"] = _normal(rng, (nimg * rows, n), 1.0, dtype)
    return out


def config_problem(name, r=None, with_dC=False):
    """Inputs of a named workload (optionally with another r for the sweep)."""
    c = dict(CONFIGS[name])
    if r is not None:
        c["r"] = r
    seed = SEEDS[name] + (0 if r is None else 100 * r)
    if name == "C1":
        return c, dense_problem(c["m"], c["k"], c["n"], seed, c["dtype"])
    return c, stl_problem(c["m"], c["k"], c["n"], c["r"], seed, c["dtype"], with_dC=with_dC)
