"""ctypes binding with the same names as the entry points declared in include/stl.h.

Argument marshalling only: device tensors (anything with ``data_ptr()``) or raw integer
addresses go in, the status code is checked, nothing is computed here.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from pathlib import Path

_HERE = Path(__file__).resolve().parent
_LIB_PATH = Path(os.environ.get("STL_LIBRARY", _HERE / "libstl_mi355x.so"))   # STL_LIBRARY: another build of the library

STL_F32, STL_BF16 = 0, 1
STL_OP_ENCODE_WEIGHT, STL_OP_FORWARD, STL_OP_BACKWARD, STL_OP_ENCODE_WEIGHT_BACKWARD = 0, 1, 2, 3
STL_FLAG_AUTO, STL_FLAG_UNFUSED, STL_FLAG_EPILOGUE, STL_FLAG_FUSED, STL_FLAG_PIPELINED = 0, 1, 2, 3, 4
STL_FLAG_GELU = 0x100
STL_FLAG_B_TRANSPOSED = 0x200

# every symbol include/stl.h declares
SYMBOLS = (
    "stl_plane_elems", "stl_workspace_bytes", "stl_encode_weight", "stl_encode_weight_backward", "stl_forward", "stl_forward_static", "stl_backward", "stl_encode_activation",
    "stl_plane_matmul", "stl_decode", "stl_mlp_workspace_bytes", "stl_mlp_forward", "stl_recode",
    "stl_aa_workspace_bytes", "stl_aa_forward", "stl_aa_backward",
    "stl_ragged_workspace_bytes", "stl_ragged_forward", "stl_ragged_backward",
    "stl_status_string", "stl_last_error", "stl_version",
)


class StlError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"STL status {status}: {message}")
        self.status = status


class _CProblem(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int64), ("k", ctypes.c_int64), ("n", ctypes.c_int64),
                ("t", ctypes.c_int32), ("r", ctypes.c_int32), ("dtype", ctypes.c_int32)]


@dataclass(frozen=True)
class Problem:
    m: int
    k: int
    n: int
    r: int
    dtype: int = STL_BF16
    t: int = 4

    def c(self) -> _CProblem:
        return _CProblem(self.m, self.k, self.n, self.t, self.r, self.dtype)


_lib = None
_P = ctypes.c_void_p


def library_path() -> Path:
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not _LIB_PATH.exists():
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2503_12211_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(str(_LIB_PATH))
    pp = ctypes.POINTER(_CProblem)
    lib.stl_plane_elems.restype = ctypes.c_size_t
    lib.stl_plane_elems.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
    lib.stl_workspace_bytes.restype = ctypes.c_size_t
    lib.stl_workspace_bytes.argtypes = [pp, ctypes.c_int, ctypes.c_int]
    lib.stl_encode_weight.argtypes = [pp, _P, _P, _P, _P]
    lib.stl_encode_weight_backward.argtypes = [pp, _P, _P, _P, _P, _P, ctypes.c_int, _P, ctypes.c_size_t, _P]
    lib.stl_forward.argtypes = [pp, _P, _P, _P, _P, _P, _P, _P, _P, ctypes.c_size_t, ctypes.c_int, _P]
    lib.stl_forward_static.argtypes = [pp, _P, _P, _P, _P, _P, ctypes.c_int, _P]
    lib.stl_forward_static.restype = ctypes.c_int
    lib.stl_backward.argtypes = [pp, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, ctypes.c_int, _P, ctypes.c_size_t, _P]
    lib.stl_encode_activation.argtypes = [pp, _P, _P, _P, _P]
    lib.stl_plane_matmul.argtypes = [pp, _P, _P, _P, _P]
    lib.stl_decode.argtypes = [pp, _P, _P, _P, ctypes.c_int, _P]
    lib.stl_mlp_workspace_bytes.restype = ctypes.c_size_t
    lib.stl_mlp_workspace_bytes.argtypes = [pp, pp, ctypes.c_int]
    lib.stl_mlp_forward.argtypes = [pp, pp, _P, _P, _P, _P, _P, _P, _P, _P, _P, ctypes.c_size_t, ctypes.c_int, _P]
    lib.stl_recode.argtypes = [pp, pp, _P, _P, _P, _P, _P, ctypes.c_int, _P]
    lib.stl_aa_workspace_bytes.restype = ctypes.c_size_t
    lib.stl_aa_workspace_bytes.argtypes = [pp, ctypes.c_int64, ctypes.c_int]
    lib.stl_aa_forward.argtypes = [pp, ctypes.c_int64] + [_P] * 10 + [ctypes.c_size_t, ctypes.c_int, _P]
    lib.stl_aa_backward.argtypes = [pp, ctypes.c_int64] + [_P] * 14 + [ctypes.c_int, _P, ctypes.c_size_t, ctypes.c_int, _P]
    lib.stl_ragged_workspace_bytes.restype = ctypes.c_size_t
    lib.stl_ragged_workspace_bytes.argtypes = [pp, ctypes.c_int64, ctypes.c_int]
    lib.stl_ragged_forward.argtypes = [pp, ctypes.c_int64] + [_P] * 9 + [ctypes.c_size_t, _P]
    lib.stl_ragged_backward.argtypes = [pp, ctypes.c_int64] + [_P] * 13 + [ctypes.c_int, _P, ctypes.c_size_t, _P]
    for name in ("stl_ragged_forward", "stl_ragged_backward", "stl_aa_forward", "stl_aa_backward", "stl_encode_weight", "stl_forward", "stl_backward", "stl_encode_activation", "stl_plane_matmul",
                 "stl_decode", "stl_mlp_forward", "stl_recode", "stl_encode_weight_backward"):
        getattr(lib, name).restype = ctypes.c_int
    lib.stl_status_string.restype = ctypes.c_char_p
    lib.stl_status_string.argtypes = [ctypes.c_int]
    lib.stl_last_error.restype = ctypes.c_char_p
    lib.stl_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def exported_symbols():
    """Names from include/stl.h that the built library exports."""
    lib = _load()
    return [s for s in SYMBOLS if hasattr(lib, s)]


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status: int):
    if status != 0:
        raise StlError(status, stl_last_error() or stl_status_string(status))


def stl_status_string(status: int) -> str:
    return _load().stl_status_string(status).decode()


def stl_last_error() -> str:
    return _load().stl_last_error().decode()


def stl_version() -> str:
    return _load().stl_version().decode()


STL_PLANE_GROUP = 64


def stl_plane_elems(R: int, Cc: int, r: int) -> int:
    return int(_load().stl_plane_elems(R, Cc, r))


def stl_workspace_bytes(prob: Problem, op: int, flags: int = 0) -> int:
    return int(_load().stl_workspace_bytes(ctypes.byref(prob.c()), op, flags))


def stl_encode_weight(prob: Problem, W, E_W, What, stream=None) -> None:
    _check(_load().stl_encode_weight(ctypes.byref(prob.c()), _ptr(W), _ptr(E_W), _ptr(What), _stream(stream)))


def stl_encode_weight_backward(prob: Problem, W, E_W, dWhat, dW, dE_W, accumulate: int = 0, ws=None, ws_bytes: int = 0,
                               stream=None) -> None:
    _check(_load().stl_encode_weight_backward(ctypes.byref(prob.c()), _ptr(W), _ptr(E_W), _ptr(dWhat), _ptr(dW), _ptr(dE_W),
                                              accumulate, _ptr(ws), ws_bytes, _stream(stream)))


def stl_forward(prob: Problem, X, What, E_X, D, C, Xhat_save=None, Yhat_save=None, ws=None, ws_bytes: int = 0,
                flags: int = STL_FLAG_AUTO, stream=None) -> None:
    _check(_load().stl_forward(ctypes.byref(prob.c()), _ptr(X), _ptr(What), _ptr(E_X), _ptr(D), _ptr(C),
                               _ptr(Xhat_save), _ptr(Yhat_save), _ptr(ws), ws_bytes, flags, _stream(stream)))


STL_STATIC_SCRATCH_BYTES = 64 << 20


def stl_forward_static(prob: Problem, X, What, E_X, D, C, flags: int = 0, stream=None) -> None:
    _check(_load().stl_forward_static(ctypes.byref(prob.c()), _ptr(X), _ptr(What), _ptr(E_X), _ptr(D), _ptr(C), flags,
                                      _stream(stream)))


def stl_backward(prob: Problem, X, What, E_X, D, dC, Xhat_saved, Yhat_saved, dX, dWhat, dE_X, dD,
                 accumulate: int = 0, ws=None, ws_bytes: int = 0, stream=None) -> None:
    _check(_load().stl_backward(ctypes.byref(prob.c()), _ptr(X), _ptr(What), _ptr(E_X), _ptr(D), _ptr(dC),
                                _ptr(Xhat_saved), _ptr(Yhat_saved), _ptr(dX), _ptr(dWhat), _ptr(dE_X), _ptr(dD), accumulate,
                                _ptr(ws), ws_bytes, _stream(stream)))


def stl_encode_activation(prob: Problem, X, E_X, Xhat, stream=None) -> None:
    _check(_load().stl_encode_activation(ctypes.byref(prob.c()), _ptr(X), _ptr(E_X), _ptr(Xhat), _stream(stream)))


def stl_plane_matmul(prob: Problem, Xhat, What, Yhat, stream=None) -> None:
    _check(_load().stl_plane_matmul(ctypes.byref(prob.c()), _ptr(Xhat), _ptr(What), _ptr(Yhat), _stream(stream)))


def stl_decode(prob: Problem, Yhat, D, C, flags: int = 0, stream=None) -> None:
    _check(_load().stl_decode(ctypes.byref(prob.c()), _ptr(Yhat), _ptr(D), _ptr(C), flags, _stream(stream)))


def stl_mlp_workspace_bytes(up: Problem, down: Problem, flags: int = 0) -> int:
    return int(_load().stl_mlp_workspace_bytes(ctypes.byref(up.c()), ctypes.byref(down.c()), flags))


def stl_mlp_forward(up: Problem, down: Problem, X, What1, E_X1, D1, What2, E_X2, D2, C, ws=None, ws_bytes: int = 0,
                    flags: int = STL_FLAG_AUTO, stream=None) -> None:
    _check(_load().stl_mlp_forward(ctypes.byref(up.c()), ctypes.byref(down.c()), _ptr(X), _ptr(What1), _ptr(E_X1),
                                   _ptr(D1), _ptr(What2), _ptr(E_X2), _ptr(D2), _ptr(C), _ptr(ws), ws_bytes, flags,
                                   _stream(stream)))


def stl_recode(up: Problem, down: Problem, Yhat1, D1, E_X2, Xhat2, H=None, flags: int = STL_FLAG_AUTO,
               stream=None) -> None:
    _check(_load().stl_recode(ctypes.byref(up.c()), ctypes.byref(down.c()), _ptr(Yhat1), _ptr(D1), _ptr(E_X2),
                              _ptr(Xhat2), _ptr(H), flags, _stream(stream)))


def stl_aa_workspace_bytes(prob: Problem, nbatch: int, op: int) -> int:
    return int(_load().stl_aa_workspace_bytes(ctypes.byref(prob.c()), nbatch, op))


def stl_aa_forward(prob: Problem, nbatch: int, A, B, E_A, E_B, D, C, Ahat_save=None, Bhat_save=None, Yhat_save=None,
                   ws=None, ws_bytes: int = 0, flags: int = 0, stream=None) -> None:
    _check(_load().stl_aa_forward(ctypes.byref(prob.c()), nbatch, _ptr(A), _ptr(B), _ptr(E_A), _ptr(E_B), _ptr(D), _ptr(C),
                                  _ptr(Ahat_save), _ptr(Bhat_save), _ptr(Yhat_save), _ptr(ws), ws_bytes, flags,
                                  _stream(stream)))


def stl_aa_backward(prob: Problem, nbatch: int, A, B, E_A, E_B, D, dC, Ahat_saved, Bhat_saved, Yhat_saved, dA, dB, dE_A,
                    dE_B, dD, accumulate: int = 0, ws=None, ws_bytes: int = 0, flags: int = 0, stream=None) -> None:
    _check(_load().stl_aa_backward(ctypes.byref(prob.c()), nbatch, _ptr(A), _ptr(B), _ptr(E_A), _ptr(E_B), _ptr(D), _ptr(dC),
                                   _ptr(Ahat_saved), _ptr(Bhat_saved), _ptr(Yhat_saved), _ptr(dA), _ptr(dB), _ptr(dE_A),
                                   _ptr(dE_B), _ptr(dD), accumulate, _ptr(ws), ws_bytes, flags, _stream(stream)))


def stl_ragged_workspace_bytes(prob: Problem, rows: int, op: int) -> int:
    return int(_load().stl_ragged_workspace_bytes(ctypes.byref(prob.c()), rows, op))


def stl_ragged_forward(prob: Problem, rows: int, X, What, E_X, D, fold, C, Xhat_save=None, Yhat_save=None, ws=None,
                       ws_bytes: int = 0, stream=None) -> None:
    _check(_load().stl_ragged_forward(ctypes.byref(prob.c()), rows, _ptr(X), _ptr(What), _ptr(E_X), _ptr(D), _ptr(fold),
                                      _ptr(C), _ptr(Xhat_save), _ptr(Yhat_save), _ptr(ws), ws_bytes, _stream(stream)))


def stl_ragged_backward(prob: Problem, rows: int, X, What, E_X, D, fold, dC, Xhat_saved, Yhat_saved, dX, dWhat, dE_X, dD,
                        dfold, accumulate: int = 0, ws=None, ws_bytes: int = 0, stream=None) -> None:
    _check(_load().stl_ragged_backward(ctypes.byref(prob.c()), rows, _ptr(X), _ptr(What), _ptr(E_X), _ptr(D), _ptr(fold),
                                       _ptr(dC), _ptr(Xhat_saved), _ptr(Yhat_saved), _ptr(dX), _ptr(dWhat), _ptr(dE_X),
                                       _ptr(dD), _ptr(dfold), accumulate, _ptr(ws), ws_bytes, _stream(stream)))
