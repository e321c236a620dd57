"""The paper's FLOP / IO model of the three-step algorithm (Section "GPU Complexity Analysis").

Pure bookkeeping used by the benchmark to turn times into rates; no kernel code depends on it.
Square case of the paper: X and W are n x n, element size `es` bytes, |X| = es * n^2.
"""
from __future__ import annotations


def flops_stl(m: int, k: int, n: int, r: int, t: int = 4) -> float:
    """Steps (i)+(ii)+(iii): 2*m*k*r + 2*r*(m/t)(k/t)(n/t) + 2*m*n*r."""
    return 2.0 * m * k * r + 2.0 * r * (m // t) * (k // t) * (n // t) + 2.0 * m * n * r


def flops_dense(m: int, k: int, n: int) -> float:
    return 2.0 * m * k * n


def io_stl_over_x(r: int, t: int = 4) -> float:
    """IO_STL / |X| for square matrices: (1 + r/t^2) + 3 r/t^2 + (1 + r/t^2) = 2 + 5 r / t^2."""
    return 2.0 + 5.0 * r / (t * t)


def io_dense_over_x() -> float:
    return 3.0


def bytes_x(n: int, es: int = 2) -> float:
    return float(es) * n * n
