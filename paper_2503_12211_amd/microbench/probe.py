"""Runs the L2->LDS / MFMA probe (dma_mfma_probe.hip) at the benchmark shape of the plane products and prints a small
table.  Measurement aid for the figures about what bounds the plane-product kernel; not part of the library.

    python -m paper_2503_12211_amd.microbench.probe [--depth]  (builds the probe next to this file if needed)
"""
from __future__ import annotations

import ctypes
import subprocess
import sys
from pathlib import Path

HERE = Path(__file__).resolve().parent
SRC, LIB = HERE / "dma_mfma_probe.hip", HERE / "libstl_probe.so"
HIPCC = "/opt/rocm/bin/hipcc"


def build() -> Path:
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-unknown-warning-option", str(SRC), "-o", str(LIB)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(res.stderr)
    return LIB


def depth_table(lib, A, B, sink, Mi, Nj, Kl, r, cus):
    """Whole-line loads with the prefetch depth, the placement of the loads and a barrier per stage varied."""
    lib.stl_probe_depth_run.restype = ctypes.c_float
    lib.stl_probe_depth_run.argtypes = lib.stl_probe_run.argtypes
    rows = [(2000, "MFMA only"), (2001, "MFMA only, barrier per stage")]
    rows += [(1000 + d, f"loads only, {d} in flight") for d in (8, 16, 32)]
    rows += [(d, f"loads in front of the MFMAs, {d} in flight") for d in (4, 8, 16, 32, 48)]
    rows += [(100 + d, f"loads between the MFMAs, {d} in flight") for d in (4, 8, 16, 32)]
    rows += [(200 + d, f"between + barrier per stage, {d} in flight") for d in (4, 8, 16, 32)]
    rows += [(308, "staggered by wavefront pair, 8 in flight"), (408, "the same + barrier per stage"),
             (508, "staggered by wavefront index mod 4, 8 in flight"), (608, "the same + barrier per stage")]
    rows += [(716, "wavefronts 0-3 load for w and w + 4"), (816, "the same + barrier per stage"),
             (916, "even wavefronts load for 2i and 2i + 1"), (1116, "the same + barrier per stage")]
    rows += [(3000, "MFMA only, all-zero operands"), (3008, "loads between the MFMAs, all-zero operands")]
    rows += [(4004, "first operand straight into registers, 4 ahead"), (4008, "the same, 8 steps ahead")]
    print("depth form (whole-line loads; load instructions a wavefront may leave in flight at the end of a stage):")
    for ident, name in rows:
        ms = lib.stl_probe_depth_run(ident, A.data_ptr(), B.data_ptr(), Mi, Nj, Kl, r, sink.data_ptr(), cus, 20)
        if ms < 0:
            raise RuntimeError(f"probe {ident} failed ({ms})")
        print(f"  {name:46s} {ms * 1e3:8.1f} us", flush=True)


def main():
    import torch
    if not LIB.exists() or LIB.stat().st_mtime < SRC.stat().st_mtime:
        build()
    lib = ctypes.CDLL(str(LIB))
    lib.stl_probe_run.restype = ctypes.c_float
    lib.stl_probe_run.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int] * 4 + [ctypes.c_void_p, ctypes.c_int, ctypes.c_int]
    r, Mi, Kl, Nj = 32, 2048, 1024, 1024
    A = torch.randn((r, Mi, Kl), device="cuda").to(torch.bfloat16)
    B = (torch.randn((r, Kl, Nj), device="cuda") / 64).to(torch.bfloat16)
    sink = torch.zeros(512, device="cuda")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    flop = 2.0 * r * Mi * Kl * Nj
    lds_bytes = (Mi // 256) * (Nj // 256) * r * (Kl // 32) * 32768.0
    names = {2: "MFMA only", 1: "loads only, half lines", 5: "loads only, whole lines", 3: "loads + MFMA, half lines",
             7: "loads + MFMA, whole lines"}
    torch.cuda.synchronize()
    for _ in range(2):          # the second round runs with the clocks up
        rows = []
        for mode in (2, 1, 5, 3, 7):
            ms = lib.stl_probe_run(mode, A.data_ptr(), B.data_ptr(), Mi, Nj, Kl, r, sink.data_ptr(), cus, 20)
            if ms < 0:
                raise RuntimeError(f"probe mode {mode} failed ({ms})")
            rows.append((mode, ms))
    print(f"probe at r={r}, planes {Mi} x {Kl} times {Kl} x {Nj} tiles, {cus} workgroups of 512 threads, 20 launches each")
    for mode, ms in rows:
        line = f"  {names[mode]:28s} {ms * 1e3:8.1f} us"
        if mode & 1:
            line += f"   L2->LDS {lds_bytes / ms / 1e9:6.2f} TB/s"
        if mode & 2:
            line += f"   {flop / ms / 1e9:7.1f} TFLOP/s"
        print(line, flush=True)
    if "--depth" in sys.argv:
        depth_table(lib, A, B, sink, Mi, Nj, Kl, r, cus)


if __name__ == "__main__":
    sys.exit(main())
