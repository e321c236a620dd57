"""The benchmark's FLOP/IO accounting against the numbers the paper prints (Example 3.5)."""
from pathlib import Path

from paper_2503_12211_amd import costmodel


def test_example_3_5():
    got = {
        "io_stl_over_x": costmodel.io_stl_over_x(32, 4),
        "io_dense_over_x": costmodel.io_dense_over_x(),
        "bytes_x": costmodel.bytes_x(8192, 2),
        "flops_stl": costmodel.flops_stl(8192, 8192, 8192, 32, 4),
        "flops_dense": costmodel.flops_dense(8192, 8192, 8192),
    }
    lines = (Path(__file__).parent / "golden" / "example_3_5.txt").read_text().splitlines()
    seen = 0
    for line in lines:
        if not line.strip() or line.startswith("#"):
            continue
        name, val, tol = line.split()
        assert abs(got[name] - float(val)) <= float(tol) * float(val), (name, got[name], val)
        seen += 1
    assert seen == 5


def test_asymptotic_speedup_is_t_cubed_over_r():
    n = 1 << 20
    ratio = costmodel.flops_dense(n, n, n) / costmodel.flops_stl(n, n, n, 24)
    assert abs(ratio - 64 / 24) < 1e-2          # the 2.66x quoted for r=24
