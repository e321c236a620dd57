"""fp64 CPU oracle of the Strassen-Tile (STL) operator -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares nothing with the HIP library.

Two independently written formulations live here:

* ``stl_oracle.c`` (wrapped below): Definition 3.1 / Eq. (2) evaluated literally,
  output tile by output tile, and the chain-rule gradients.  Plain loops, fp64.
* ``oracle.planes``: the three-step plane algorithm (Claim 3.4 / Algorithm 1),
  with numpy ``matmul`` as the per-plane product.  Used where the literal loops
  would take too long (full-size sampled checks).

All arrays are C-contiguous float64.  Layouts: X m x k, W k x n, C m x n
row-major; E_X, E_W, D are r x t^2 row-major; What is r x K x N plane-major.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "stl_oracle.c"
_LIB = _HERE / "libstl_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile the C oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".{os.getpid()}.tmp")
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-Wall", "-Wextra", "-o", str(tmp), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


_D = ctypes.POINTER(ctypes.c_double)
_I64 = ctypes.c_int64
_INT = ctypes.c_int


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        lib.stl_oracle_num_threads.restype = _INT
        lib.stl_oracle_set_threads.argtypes = [_INT]
        lib.stl_oracle_encode_weight.argtypes = [_I64, _I64, _INT, _INT, _D, _D, _D]
        lib.stl_oracle_encode_x.argtypes = [_I64, _I64, _INT, _INT, _D, _D, _D]
        lib.stl_oracle_forward_block.argtypes = [_I64, _I64, _I64, _INT, _INT, _D, _D, _D, _D,
                                                 _I64, _I64, _I64, _I64, _D, _D]
        lib.stl_oracle_backward.argtypes = [_I64, _I64, _I64, _INT, _INT, _D, _D, _D, _D, _D,
                                            _D, _D, _D, _D]
        _lib = lib
    return _lib


def _f64(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _p(a):
    return a.ctypes.data_as(_D) if a is not None else None


def num_threads() -> int:
    return int(_load().stl_oracle_num_threads())


def set_threads(n: int) -> None:
    _load().stl_oracle_set_threads(int(n))


def _check_dims(t, r, *dims):
    if t < 1 or r < 1:
        raise ValueError("t and r must be positive")
    for d in dims:
        if d % t:
            raise ValueError(f"dimension {d} is not divisible by t={t}")


def encode_weight(W, E_W, t: int = 4):
    """What[p,L,J] = (E_W vec W_{L,J})_p  (plane definition before Claim 3.4)."""
    W = _f64(W)
    k, n = W.shape
    E_W = _f64(E_W)
    r = E_W.shape[0]
    _check_dims(t, r, k, n)
    E_W = _f64(E_W, (r, t * t))
    What = np.empty((r, k // t, n // t))
    _load().stl_oracle_encode_weight(k, n, t, r, _p(W), _p(E_W), _p(What))
    return What


def encode_x(X, E_X, t: int = 4):
    """Xhat[p,I,L] = (E_X vec X_{I,L})_p  (step (i))."""
    X = _f64(X)
    m, k = X.shape
    E_X = _f64(E_X)
    r = E_X.shape[0]
    _check_dims(t, r, m, k)
    E_X = _f64(E_X, (r, t * t))
    Xhat = np.empty((r, m // t, k // t))
    _load().stl_oracle_encode_x(m, k, t, r, _p(X), _p(E_X), _p(Xhat))
    return Xhat


def forward_block(X, What, E_X, D, I0, I1, J0, J1, t: int = 4, return_yhat: bool = False):
    """Eq. (2) for output tiles I0<=I<I1, J0<=J<J1 only (full contraction over L)."""
    X = _f64(X)
    m, k = X.shape
    What = _f64(What)
    r, K, N = What.shape
    n = N * t
    _check_dims(t, r, m, k)
    if K * t != k:
        raise ValueError("What does not match X")
    E_X = _f64(E_X, (r, t * t))
    D = _f64(D, (r, t * t))
    if not (0 <= I0 <= I1 <= m // t and 0 <= J0 <= J1 <= N):
        raise ValueError("tile range out of bounds")
    C = np.empty(((I1 - I0) * t, (J1 - J0) * t))
    Y = np.empty((r, I1 - I0, J1 - J0)) if return_yhat else None
    _load().stl_oracle_forward_block(m, k, n, t, r, _p(X), _p(What), _p(E_X), _p(D),
                                     I0, I1, J0, J1, _p(C), _p(Y))
    return (C, Y) if return_yhat else C


def forward(X, What, E_X, D, t: int = 4, return_yhat: bool = False):
    """C = X <> W given the encoded weight planes (Definition 3.1 / Eq. (2))."""
    X = np.asarray(X)
    What = np.asarray(What)
    return forward_block(X, What, E_X, D, 0, X.shape[0] // t, 0, What.shape[2], t, return_yhat)


def backward(X, What, E_X, D, dC, t: int = 4):
    """Chain-rule gradients of <dC, C>: returns dX, dWhat, dE_X, dD."""
    X = _f64(X)
    m, k = X.shape
    What = _f64(What)
    r, K, N = What.shape
    n = N * t
    _check_dims(t, r, m, k)
    if K * t != k:
        raise ValueError("What does not match X")
    E_X = _f64(E_X, (r, t * t))
    D = _f64(D, (r, t * t))
    dC = _f64(dC, (m, n))
    dX = np.empty((m, k))
    dWhat = np.empty((r, K, N))
    dE_X = np.empty((r, t * t))
    dD = np.empty((r, t * t))
    _load().stl_oracle_backward(m, k, n, t, r, _p(X), _p(What), _p(E_X), _p(D), _p(dC),
                                _p(dX), _p(dWhat), _p(dE_X), _p(dD))
    return dX, dWhat, dE_X, dD
